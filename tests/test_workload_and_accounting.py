"""Pins for the seeded input generator and for the byte / flop accounting."""
import os

import numpy as np
import torch

from harness import workload as W
from paper_2506_10470_amd import accounting as A

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _kv(path):
    out = {}
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split()
        out[k] = float(v)
    return out


def test_kv_size_formula_reproduces_papers_worked_example():
    g = _kv(os.path.join(GOLD, "kv_size_example.txt"))
    per_tok = A.kv_bytes_per_token(int(g["llama30b_layers"]), 1, int(g["llama30b_hidden"]), int(g["elem_bytes"]))
    assert abs(per_tok / 2 ** 20 - g["kv_mb_per_token"]) < 0.01          # 1.52 MB per token
    total = per_tok * g["requests"] * g["avg_len"] / 2 ** 30
    assert abs(total - g["total_gb"]) < 1.0                              # about 178 GB


def test_weight_count_reproduces_table2_model_sizes():
    for line in open(os.path.join(GOLD, "table2_model_sizes.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, gb, layers, heads, hidden, bpp, ffn, kvh = line.split()
        p = A.matmul_params_per_layer(int(hidden), int(heads), int(kvh), int(hidden) // int(heads), int(ffn))
        size = p * int(layers) * int(bpp) / 1e9
        # embeddings / LM head (not part of a mid-pipeline stage) make up the rest
        assert 0.95 * float(gb) <= size <= 1.0 * float(gb), (name, size)


def test_stage_weight_bytes_of_the_70b_quarter_stage():
    sh = W.SHAPES["70b_quarter"]
    p = A.matmul_params_per_layer(sh.d_model, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.d_ff)
    assert p == 855_638_016
    assert abs(p * sh.n_layers * 2 / 1e9 - 34.2) < 0.1


def test_decode_work_counts():
    w = A.decode_step_work(2, 256, 4, 4, 64, 688, [16, 64])
    assert w["weight_bytes"] == 2 * 790_528 * 2
    assert w["kv_read_bytes"] == 2 * (2 * 4 * 64 * 2) * (17 + 65)
    assert w["kv_write_bytes"] == 2 * (2 * 4 * 64 * 2) * 2
    assert w["gemm_flops"] == 2 * 2 * 2 * 790_528


def test_generator_is_deterministic_and_sliceable():
    key = W.stream_key(W.BASE_SEED, 7, 3)
    a = W.normal_tensor(key, (37, 5, 11), 1.0)
    b = W.normal_tensor(key, (37, 5, 11), 1.0)
    assert torch.equal(a, b)
    c = W.normal_tensor(key, (37, 5, 11), 1.0, row0=10, rows=4)
    assert torch.equal(a[10:14], c)
    d = W.normal_flat(key, 0, 37 * 55, 1.0, chunk=100)
    assert torch.equal(a.flatten(), d)
    assert not torch.equal(a, W.normal_tensor(W.stream_key(W.BASE_SEED, 7, 4), (37, 5, 11), 1.0))


def test_generator_moments():
    x = W.normal_flat(W.stream_key(1, 2), 0, 1 << 20, 0.02).double()
    assert abs(x.mean().item()) < 1e-4
    assert abs(x.std().item() - 0.02) < 2e-4
    g = W.weight(W.SHAPES["tiny"], 0, "g_attn", dtype=torch.float32).double()
    assert abs(g.mean().item() - 1.0) < 5e-3


def test_hash_matches_reference_integer_arithmetic():
    key = W.stream_key(123, 4)
    h = W.hash_u64(key, 5, 3).numpy().view(np.uint64)
    for i in range(3):
        want = W._mix64_int(((5 + i) * 0x9E3779B97F4A7C15 + key) & ((1 << 64) - 1))
        assert int(h[i]) == want


def test_lengths_respect_their_ranges():
    for cfg, lo, hi in (("tiny", 16, 64), ("7b_quarter", 16, 2560), ("13b_quarter", 16, 4096), ("70b_quarter", 64, 4096)):
        c = W.decode_ctx_lens(cfg, 512)
        assert c.min() >= lo and c.max() <= hi
    c = W.decode_ctx_lens("70b_quarter", 512)
    assert 1100 < c.mean() < 1350          # lognormal mean = 1024 * exp(0.18) ~ 1226 before clipping
    p = W.prefill_seq_lens("13b_quarter", 32)
    assert p.min() >= 16 and p.max() <= 4096


def test_block_tables_are_a_partial_permutation():
    ctx = W.decode_ctx_lens("tiny", 4)
    b = W.make_decode_batch(ctx)
    used = b.tables[b.tables >= 0]
    assert len(np.unique(used)) == len(used)
    assert used.max() < b.num_pages
    need = (ctx + 1 + 15) // 16
    assert [(row >= 0).sum() for row in b.tables] == list(need)
    assert b.num_pages > len(used)          # spare pages exist
    assert not np.array_equal(used, np.sort(used))   # shuffled

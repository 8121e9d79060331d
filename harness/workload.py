"""Seeded synthetic workload generator for the pipeline-stage forward pass.

This module produces *inputs only*: model shapes, weights, hidden states,
request lengths, block tables and pre-existing KV contents.  It holds none of
the stage's arithmetic (no norm, no projection, no rotation, no attention) and
is the only code shared by the CPU oracle's tests and the GPU path's tests.

The paper evaluates on 5,000 ShareGPT-V3 requests (Sec. 4.1) with Llama-2 /
Qwen2.5 checkpoints (Table 2); neither is available, so lengths are drawn from
log-normal / uniform distributions and weights from N(0, 0.02), as the
benchmark configurations prescribe.

Everything is a pure function of (seed, stream, element index) through a
counter-based integer hash, so any slice can be regenerated anywhere and the
CPU and GPU (torch) evaluations are bit-identical: the hash and the
approximately-normal transform use only 64-bit integer operations followed by
one exactly-rounded fp32 multiply.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import Dict, List, Tuple

import numpy as np
import torch

BASE_SEED = 250610470
PAGE_SIZE = 16

_M64 = (1 << 64) - 1


def _s64(v: int) -> int:
    """Two's-complement reinterpretation of an unsigned 64-bit constant."""
    v &= _M64
    return v - (1 << 64) if v >= (1 << 63) else v


_GOLDEN = _s64(0x9E3779B97F4A7C15)
_MUL1 = _s64(0xBF58476D1CE4E5B9)
_MUL2 = _s64(0x94D049BB133111EB)


def _lsr(x: torch.Tensor, k: int) -> torch.Tensor:
    """Logical right shift of an int64 tensor (torch's >> is arithmetic)."""
    return (x >> k) & ((1 << (64 - k)) - 1)


def _mix64(x: torch.Tensor) -> torch.Tensor:
    """splitmix64 output function on int64 tensors (wrapping arithmetic)."""
    x = (x ^ _lsr(x, 30)) * _MUL1
    x = (x ^ _lsr(x, 27)) * _MUL2
    return x ^ _lsr(x, 31)


def _mix64_int(x: int) -> int:
    x &= _M64
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & _M64
    return x ^ (x >> 31)


def stream_key(seed: int, *stream: int) -> int:
    """Fold a seed and a tuple of stream identifiers into one 64-bit key."""
    k = _mix64_int(seed)
    for s in stream:
        k = _mix64_int(k ^ _mix64_int((int(s) + 0x632BE59BD9B4E019) & _M64))
    return k


def hash_u64(key: int, start: int, count: int, device="cpu") -> torch.Tensor:
    """64-bit hashes of counters start..start+count-1 under `key` (as int64)."""
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    return _mix64(idx * _GOLDEN + _s64(key))


_IH_MEAN = 8 * 127.5
_IH_STD = math.sqrt(8 * (256.0 ** 2 - 1.0) / 12.0)


def _byte_sum(h: torch.Tensor) -> torch.Tensor:
    """Sum of the eight bytes of each 64-bit word (0..2040)."""
    t = (h & 0x00FF00FF00FF00FF) + (_lsr(h, 8) & 0x00FF00FF00FF00FF)
    t = (t & 0x0000FFFF0000FFFF) + (_lsr(t, 16) & 0x0000FFFF0000FFFF)
    return (t & 0xFFFFFFFF) + _lsr(t, 32)


def normal_flat(key: int, start: int, count: int, std: float, mean: float = 0.0,
                device="cpu", chunk: int = 1 << 26) -> torch.Tensor:
    """Approximately normal fp32 samples: the sum of the 8 hash bytes
    (Irwin-Hall, n = 8; support +-4.88 sigma), centred and scaled.  Integer
    sum -> exact fp32 -> one fp32 multiply (+ one add if mean != 0)."""
    out = torch.empty(count, dtype=torch.float32, device=device)
    scale = float(np.float32(std / _IH_STD))
    for c0 in range(0, count, chunk):
        n = min(chunk, count - c0)
        s = _byte_sum(hash_u64(key, start + c0, n, device))
        z = (s.to(torch.float32) - _IH_MEAN) * scale
        if mean != 0.0:
            z = z + float(np.float32(mean))
        out[c0:c0 + n] = z
    return out


def normal_tensor(key: int, shape, std: float, mean: float = 0.0, device="cpu",
                  dtype=torch.float32, row0: int = 0, rows: int | None = None) -> torch.Tensor:
    """Tensor of logical shape `shape`; rows [row0, row0+rows) of its first
    dimension are generated (all rows by default)."""
    shape = tuple(int(s) for s in shape)
    inner = int(np.prod(shape[1:])) if len(shape) > 1 else 1
    rows = shape[0] - row0 if rows is None else rows
    flat = normal_flat(key, row0 * inner, rows * inner, std, mean, device)
    return flat.view((rows,) + shape[1:]).to(dtype)


# --------------------------------------------------------------------------
# Stage shapes
# --------------------------------------------------------------------------

@dataclass(frozen=True)
class StageShape:
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ff: int
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    page_size: int = PAGE_SIZE
    config_index: int = 0
    qkv_bias: bool = False

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def d_q(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def d_kv(self) -> int:
        return self.n_kv_heads * self.head_dim

    def with_layers(self, n: int) -> "StageShape":
        return replace(self, n_layers=n)


SHAPES: Dict[str, StageShape] = {
    "tiny": StageShape("tiny", 2, 256, 4, 4, 64, 688, config_index=0),
    "tiny_gqa": StageShape("tiny_gqa", 2, 256, 8, 2, 64, 688, config_index=0),
    "tiny_h128": StageShape("tiny_h128", 2, 512, 8, 2, 128, 1376, config_index=0),
    "7b_quarter": StageShape("7b_quarter", 8, 4096, 32, 32, 128, 11008, config_index=1),
    "13b_quarter": StageShape("13b_quarter", 10, 5120, 40, 40, 128, 13824, config_index=2),
    "70b_quarter": StageShape("70b_quarter", 20, 8192, 64, 8, 128, 28672, config_index=4),
    # Qwen2.5-32B-shaped (paper Table 2: 64 layers, hidden 5120, 40 heads; public model: 8 KV heads,
    # FFN 27648, q/k/v biases, eps 1e-6, rope base 1e6): a quarter is 16 layers
    "qwen32b_quarter": StageShape("qwen32b_quarter", 16, 5120, 40, 8, 128, 27648, rms_eps=1e-6,
                                  rope_base=1000000.0, config_index=5, qkv_bias=True),
    "tiny_bias": StageShape("tiny_bias", 2, 320, 10, 2, 64, 688, rms_eps=1e-6, rope_base=1000000.0,
                            config_index=0, qkv_bias=True),
    # one K/V head shared by sixteen query heads: the largest group the kernels take
    "tiny_mqa": StageShape("tiny_mqa", 2, 256, 16, 1, 64, 688, config_index=0),
    # groups of two query heads (head_dim 128)
    "tiny_g2": StageShape("tiny_g2", 2, 512, 6, 3, 128, 688, config_index=0),
    # a model dimension beyond 8192 (rows longer than what the row-wise kernels keep in registers)
    "tiny_wide": StageShape("tiny_wide", 1, 9216, 4, 2, 64, 256, config_index=0),
}

WEIGHT_NAMES = ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "g_attn", "g_mlp")
BIAS_NAMES = ("bq", "bk", "bv")   # only for shapes with qkv_bias


def weight_shape(sh: StageShape, which: str) -> Tuple[int, ...]:
    """Logical shapes; matrices are [in, out] (y = x W)."""
    return {
        "wq": (sh.d_model, sh.d_q), "wk": (sh.d_model, sh.d_kv), "wv": (sh.d_model, sh.d_kv),
        "wo": (sh.d_q, sh.d_model), "wg": (sh.d_model, sh.d_ff), "wu": (sh.d_model, sh.d_ff),
        "wd": (sh.d_ff, sh.d_model), "g_attn": (sh.d_model,), "g_mlp": (sh.d_model,),
        "bq": (sh.d_q,), "bk": (sh.d_kv,), "bv": (sh.d_kv,),
    }[which]


def weight(sh: StageShape, layer: int, which: str, device="cpu", dtype=torch.bfloat16,
           seed: int = BASE_SEED) -> torch.Tensor:
    """Matrices ~ N(0, 0.02); norm gains ~ 1 + N(0, 0.02) (a gain of exactly 1
    would hide a dropped-gain bug)."""
    shape = weight_shape(sh, which)
    if which in BIAS_NAMES:  # ~ N(0, 0.5): large enough that a dropped or misplaced bias is far outside tolerance
        key = stream_key(seed, 1000 * sh.config_index, 6, layer, BIAS_NAMES.index(which))
        return normal_tensor(key, shape, 0.5, 0.0, device, dtype)
    key = stream_key(seed, 1000 * sh.config_index, 1, layer, WEIGHT_NAMES.index(which))
    mean = 1.0 if which.startswith("g_") else 0.0
    return normal_tensor(key, shape, 0.02, mean, device, dtype)


def hidden_states(sh: StageShape, n_tokens: int, stream: int, device="cpu",
                  dtype=torch.bfloat16, seed: int = BASE_SEED) -> torch.Tensor:
    """Stage inputs ~ N(0, 1), [n_tokens, d_model]."""
    key = stream_key(seed, 1000 * sh.config_index, 2, stream)
    return normal_tensor(key, (n_tokens, sh.d_model), 1.0, 0.0, device, dtype)


def ends_weight(sh: StageShape, which: str, vocab: int, device="cpu", dtype=torch.bfloat16,
                seed: int = BASE_SEED) -> torch.Tensor:
    """Weights of the pipeline ends: "embedding" [vocab, d] ~ N(0, 1) (so that embedded tokens look
    like the N(0, 1) hidden states the stage is fed elsewhere), "lm_head" [d, vocab] ~ N(0, 0.02),
    "final_norm" [d] ~ 1 + N(0, 0.02)."""
    idx = {"embedding": 0, "lm_head": 1, "final_norm": 2}[which]
    key = stream_key(seed, 1000 * sh.config_index, 4, idx, vocab)
    if which == "embedding":
        return normal_tensor(key, (vocab, sh.d_model), 1.0, 0.0, device, dtype)
    if which == "lm_head":
        return normal_tensor(key, (sh.d_model, vocab), 0.02, 0.0, device, dtype)
    return normal_tensor(key, (sh.d_model,), 0.02, 1.0, device, dtype)


def token_ids(vocab: int, n: int, stream: int, seed: int = BASE_SEED) -> np.ndarray:
    """n token ids uniform in [0, vocab)."""
    u = _uniform01(stream_key(seed, 5, stream, vocab), n)
    return np.minimum((u * vocab).astype(np.int64), vocab - 1).astype(np.int32)


def kv_packed(sh: StageShape, layer: int, which: str, total_tokens: int, stream: int,
              device="cpu", dtype=torch.bfloat16, seed: int = BASE_SEED,
              tok0: int = 0, toks: int | None = None) -> torch.Tensor:
    """Pre-existing cache contents ~ N(0, 1) in logical order: token-major,
    [total_tokens, n_kv_heads, head_dim], the requests' contexts concatenated.
    `tok0/toks` select a token range so one request can be regenerated alone."""
    key = stream_key(seed, 1000 * sh.config_index, 3, stream, layer, 0 if which == "k" else 1)
    return normal_tensor(key, (total_tokens, sh.n_kv_heads, sh.head_dim), 1.0, 0.0, device, dtype,
                         row0=tok0, rows=toks)


# --------------------------------------------------------------------------
# Request lengths and block tables (small, host-side, numpy)
# --------------------------------------------------------------------------

def _uniform01(key: int, n: int) -> np.ndarray:
    h = hash_u64(key, 0, n).numpy().view(np.uint64)
    return ((h >> np.uint64(11)).astype(np.float64) + 0.5) / float(1 << 53)


def _std_normal(key: int, n: int) -> np.ndarray:
    u1 = _uniform01(stream_key(key, 1), n)
    u2 = _uniform01(stream_key(key, 2), n)
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


def lognormal_lengths(key: int, n: int, median: float, sigma: float, lo: int, hi: int) -> np.ndarray:
    z = _std_normal(key, n)
    return np.clip(np.rint(median * np.exp(sigma * z)), lo, hi).astype(np.int64)


def uniform_lengths(key: int, n: int, lo: int, hi: int) -> np.ndarray:
    """Integers uniform in [lo, hi] inclusive."""
    u = _uniform01(key, n)
    return np.minimum(lo + np.floor(u * (hi - lo + 1)), hi).astype(np.int64)


def permutation(key: int, n: int) -> np.ndarray:
    h = hash_u64(key, 0, n).numpy().view(np.uint64)
    return np.argsort(h, kind="stable").astype(np.int64)


def block_tables(key: int, n_tokens_per_seq: np.ndarray, page_size: int = PAGE_SIZE,
                 spare_frac: float = 0.125, max_pages_per_seq: int | None = None
                 ) -> Tuple[np.ndarray, int]:
    """Deal a random permutation of the physical pages out to the sequences.
    Returns (tables [n, max_pages_per_seq] int32, -1 where unused; num_pages)."""
    need = (np.asarray(n_tokens_per_seq, dtype=np.int64) + page_size - 1) // page_size
    total = int(need.sum())
    num_pages = total + max(1, int(math.ceil(total * spare_frac)))
    perm = permutation(key, num_pages)
    width = int(need.max()) if max_pages_per_seq is None else int(max_pages_per_seq)
    assert width >= int(need.max())
    tab = np.full((len(need), width), -1, dtype=np.int32)
    off = 0
    for i, c in enumerate(need):
        tab[i, :c] = perm[off:off + c]
        off += int(c)
    return tab, num_pages


# --------------------------------------------------------------------------
# The benchmark configurations' request mixes
# --------------------------------------------------------------------------

@dataclass
class DecodeBatch:
    ctx_lens: np.ndarray          # tokens already cached per request
    tables: np.ndarray            # [B, max_pages_per_seq] int32
    num_pages: int


@dataclass
class PrefillBatch:
    seq_lens: np.ndarray
    cu_seqlens: np.ndarray        # int32 [n+1]
    tables: np.ndarray
    num_pages: int


def decode_ctx_lens(config: str, batch: int, seed: int = BASE_SEED) -> np.ndarray:
    """Context lengths (tokens already in the cache) of each configuration."""
    k = stream_key(seed, 10, batch)
    if config == "tiny":
        return uniform_lengths(k, batch, 16, 64)
    if config == "7b_quarter":      # prompt LN(256, .8) in [16,2048] + generated U[0,512]
        return lognormal_lengths(stream_key(k, 1), batch, 256, 0.8, 16, 2048) + \
            uniform_lengths(stream_key(k, 2), batch, 0, 512)
    if config in ("13b_quarter", "qwen32b_quarter"):  # prompt LN(384, .7) + generated U[0,1024], clipped to 4096
        p = lognormal_lengths(stream_key(k, 1), batch, 384, 0.7, 16, 4096)
        return np.minimum(p + uniform_lengths(stream_key(k, 2), batch, 0, 1024), 4096)
    if config == "70b_quarter":     # LN(1024, .6) in [64,4096]
        return lognormal_lengths(stream_key(k, 1), batch, 1024, 0.6, 64, 4096)
    raise KeyError(config)


def prefill_seq_lens(config: str, n_seqs: int, seed: int = BASE_SEED) -> np.ndarray:
    k = stream_key(seed, 11, n_seqs)
    if config == "tiny":
        return uniform_lengths(k, n_seqs, 8, 32)
    if config == "7b_quarter":
        return lognormal_lengths(k, n_seqs, 256, 0.8, 16, 2048)
    if config in ("13b_quarter", "qwen32b_quarter"):
        return lognormal_lengths(k, n_seqs, 384, 0.7, 16, 4096)
    if config == "70b_quarter":
        return lognormal_lengths(k, n_seqs, 1024, 0.6, 64, 4096)
    raise KeyError(config)


def serving_requests(n: int, seed: int = BASE_SEED) -> np.ndarray:
    """Offline serving workload for the scheduler: int32 [n, 3] = (input length, output length,
    predicted output length).  Stands in for the conversation dataset of the paper's throughput
    runs (Sec. 4.1: prompts shorter than 1024 tokens, outputs from the model), which is not
    available: prompts ~ LN(median 160, sigma 1.0) clipped to [4, 1023], outputs ~ LN(median 180,
    sigma 0.9) clipped to [1, 1024]; the prediction is the output length times LN(1, 0.35), the
    error of a coarse length classifier."""
    ins = lognormal_lengths(stream_key(seed, 21, n), n, 160, 1.0, 4, 1023)
    outs = lognormal_lengths(stream_key(seed, 22, n), n, 180, 0.9, 1, 1024)
    noise = lognormal_lengths(stream_key(seed, 23, n), n, 1000, 0.35, 1, 10 ** 6).astype(np.float64) / 1000.0
    pred = np.clip(np.rint(outs * noise), 1, 2048)
    return np.stack([ins, outs, pred], axis=1).astype(np.int32)


def make_decode_batch(ctx_lens: np.ndarray, page_size: int = PAGE_SIZE, seed: int = BASE_SEED,
                      max_pages_per_seq: int | None = None, steps: int = 1) -> DecodeBatch:
    """Pages are reserved for ctx+steps tokens: every decode step appends one token."""
    ctx_lens = np.asarray(ctx_lens, dtype=np.int64)
    tab, npg = block_tables(stream_key(seed, 12, len(ctx_lens)), ctx_lens + steps, page_size,
                            max_pages_per_seq=max_pages_per_seq)
    return DecodeBatch(ctx_lens.astype(np.int32), tab, npg)


def make_prefill_batch(seq_lens: np.ndarray, page_size: int = PAGE_SIZE, seed: int = BASE_SEED,
                       max_pages_per_seq: int | None = None) -> PrefillBatch:
    seq_lens = np.asarray(seq_lens, dtype=np.int64)
    tab, npg = block_tables(stream_key(seed, 13, len(seq_lens)), seq_lens, page_size,
                            max_pages_per_seq=max_pages_per_seq)
    cu = np.zeros(len(seq_lens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(seq_lens)
    return PrefillBatch(seq_lens.astype(np.int32), cu, tab, npg)

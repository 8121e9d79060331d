"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle on the same seeded
inputs.  Outputs: max |gpu - oracle| / max |oracle row| <= 2e-2 (bf16 outputs, fp32 accumulation).
KV slot addressing: bit-exact (every slot that must not change keeps its poison bits)."""
import numpy as np
import pytest
import torch

from harness import workload as W
from oracle import stage_oracle as O
from stage_helpers import TOL, Stage, f64, i32, oracle_layers, oracle_shape, row_rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tdp():
    from paper_2506_10470_amd import tdp as _tdp
    return _tdp


# ----------------------------------------------------------------------------- plumbing

def test_generator_is_bit_identical_on_cpu_and_gpu():
    sh = W.SHAPES["tiny"]
    for name in ("wq", "wd", "g_mlp"):
        a = W.weight(sh, 1, name, device="cpu")
        b = W.weight(sh, 1, name, device="cuda").cpu()
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    a = W.kv_packed(sh, 0, "v", 100, 5, device="cpu", tok0=17, toks=9)
    b = W.kv_packed(sh, 0, "v", 100, 5, device="cuda")[17:26].cpu()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def import_kv(tdp, st: Stage, lens: np.ndarray, tables: np.ndarray, stream_id: int):
    """Fill the pages of sequences with generated K/V; returns per-sequence oracle caches."""
    sh = st.shape
    lens = np.asarray(lens, dtype=np.int64)
    total = int(lens.sum())
    cu = np.zeros(len(lens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lens)
    caches = [[None] * sh.n_layers for _ in lens]
    if total == 0:
        for b in range(len(lens)):
            for l in range(sh.n_layers):
                caches[b][l] = (O.empty_cache(oracle_shape(sh)), O.empty_cache(oracle_shape(sh)))
        return caches
    cu_d, tab_d = i32(cu), i32(tables)
    for l in range(sh.n_layers):
        k = W.kv_packed(sh, l, "k", total, stream_id, device="cuda")
        v = W.kv_packed(sh, l, "v", total, stream_id, device="cuda")
        tdp.tdp_stage_kv_import(st.h, l, k, v, cu_d, tab_d, len(lens), total)
        torch.cuda.synchronize()
        kc, vc = f64(k), f64(v)
        for b in range(len(lens)):
            caches[b][l] = (kc[cu[b]:cu[b + 1]], vc[cu[b]:cu[b + 1]])
    return caches


def export_kv(tdp, st: Stage, lens: np.ndarray, tables: np.ndarray, layer: int):
    sh = st.shape
    total = int(np.sum(lens))
    cu = np.zeros(len(lens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lens)
    k = torch.empty(total, sh.n_kv_heads, sh.head_dim, dtype=torch.bfloat16, device="cuda")
    v = torch.empty_like(k)
    tdp.tdp_stage_kv_export(st.h, layer, k, v, i32(cu), i32(tables), len(lens), total)
    torch.cuda.synchronize()
    return f64(k), f64(v), cu


def written_slot_mask(st: Stage, tables: np.ndarray, first: np.ndarray, last: np.ndarray):
    """Boolean masks over the K and V pools of the slots positions first[b]..last[b]-1 occupy,
    computed from the documented layout alone."""
    sh = st.shape
    mk = torch.zeros(st.num_pages, sh.n_kv_heads, 16, sh.head_dim, dtype=torch.bool)
    mv = torch.zeros(st.num_pages, sh.n_kv_heads, sh.head_dim, 16, dtype=torch.bool)
    for b in range(len(first)):
        for p in range(int(first[b]), int(last[b])):
            page, slot = int(tables[b, p // 16]), p % 16
            mk[page, :, slot, :] = True
            mv[page, :, :, slot] = True
    return mk, mv


def run_decode_case(tdp, shape_name, ctx_lens, n_layers=None, stream_id=1, max_pages_per_seq=None, span=0,
                    micro_batches=0):
    sh = shape_name if isinstance(shape_name, W.StageShape) else W.SHAPES[shape_name]
    if n_layers:
        sh = sh.with_layers(n_layers)
    ctx_lens = np.asarray(ctx_lens, dtype=np.int64)
    B = len(ctx_lens)
    batch = W.make_decode_batch(ctx_lens, max_pages_per_seq=max_pages_per_seq)
    with Stage(tdp, sh, batch.num_pages, B, 0, 0, batch.tables.shape[1], decode_micro_batches=micro_batches) as st:
        st.poison()
        tdp.tdp_stage_set_decode_span(st.h, span)
        caches = import_kv(tdp, st, ctx_lens, batch.tables, stream_id)
        before = [tuple(t.clone() for t in st.pools(l)) for l in range(sh.n_layers)]
        x = W.hidden_states(sh, B, stream_id, device="cuda")
        out = torch.empty_like(x)
        tdp.tdp_stage_decode(st.h, x, i32(batch.ctx_lens), i32(batch.tables), B, out)
        torch.cuda.synchronize()
        ref, new_caches = O.stage_decode(list(f64(x)), caches, list(oracle_layers(sh)), oracle_shape(sh))
        err = row_rel_err(f64(out), np.stack(ref))
        assert err <= TOL, err
        # KV append: the new token's slot holds the oracle's K/V; every other bit is untouched
        mk, mv = written_slot_mask(st, batch.tables, ctx_lens, ctx_lens + 1)
        for l in range(sh.n_layers):
            k_after, v_after = st.pools(l)
            kb, vb = before[l]
            same_k = (k_after.view(torch.int16) == kb.view(torch.int16)).cpu()
            same_v = (v_after.view(torch.int16) == vb.view(torch.int16)).cpu()
            assert bool(same_k[~mk].all()) and bool(same_v[~mv].all()), "a slot outside the append changed"
            kx, vx, cu = export_kv(tdp, st, ctx_lens + 1, batch.tables, l)
            for b in range(B):
                k_ref, v_ref = new_caches[b][l]
                assert row_rel_err(kx[cu[b + 1] - 1], k_ref[-1]) <= TOL
                assert row_rel_err(vx[cu[b + 1] - 1], v_ref[-1]) <= TOL
                # the pre-existing context reads back exactly as imported
                assert np.array_equal(kx[cu[b]:cu[b + 1] - 1], k_ref[:-1])
                assert np.array_equal(vx[cu[b]:cu[b + 1] - 1], v_ref[:-1])
        return err


def run_prefill_case(tdp, shape_name, seq_lens, n_layers=None, stream_id=2, decode_steps=0):
    sh = shape_name if isinstance(shape_name, W.StageShape) else W.SHAPES[shape_name]
    if n_layers:
        sh = sh.with_layers(n_layers)
    seq_lens = np.asarray(seq_lens, dtype=np.int64)
    n = len(seq_lens)
    T = int(seq_lens.sum())
    # reserve pages for the decode steps that follow
    pb = W.make_prefill_batch(seq_lens + decode_steps)
    cu = np.zeros(n + 1, dtype=np.int32)
    cu[1:] = np.cumsum(seq_lens)
    with Stage(tdp, sh, pb.num_pages, n, T, n, pb.tables.shape[1]) as st:
        st.poison()
        x = W.hidden_states(sh, T, stream_id, device="cuda")
        out = torch.empty_like(x)
        tab_d = i32(pb.tables)
        tdp.tdp_stage_prefill(st.h, x, i32(cu), tab_d, n, T, out)
        torch.cuda.synchronize()
        layers = list(oracle_layers(sh))
        osh = oracle_shape(sh)
        xs = f64(x)
        ref, caches = O.stage_prefill([xs[cu[s]:cu[s + 1]] for s in range(n)], layers, osh)
        err = row_rel_err(f64(out), np.concatenate(ref))
        assert err <= TOL, err
        mk, mv = written_slot_mask(st, pb.tables, np.zeros(n, dtype=np.int64), seq_lens)
        for l in range(sh.n_layers):
            k_pool, v_pool = st.pools(l)
            # unwritten slots still hold the poison (NaN != NaN, so compare bits)
            assert bool(torch.isnan(k_pool.cpu()[~mk]).all()) and bool(torch.isnan(v_pool.cpu()[~mv]).all())
            assert not bool(torch.isnan(k_pool.cpu()[mk]).any()) and not bool(torch.isnan(v_pool.cpu()[mv]).any())
            kx, vx, _ = export_kv(tdp, st, seq_lens, pb.tables, l)
            for s in range(n):
                assert row_rel_err(kx[cu[s]:cu[s + 1]].reshape(int(seq_lens[s]), -1),
                                   caches[s][l][0].reshape(int(seq_lens[s]), -1)) <= TOL
                assert row_rel_err(vx[cu[s]:cu[s + 1]].reshape(int(seq_lens[s]), -1),
                                   caches[s][l][1].reshape(int(seq_lens[s]), -1)) <= TOL
        # follow with decode steps on the cache the prefill produced (crosses page boundaries)
        ctx = seq_lens.copy()
        for step in range(decode_steps):
            xd = W.hidden_states(sh, n, 100 + step, device="cuda")
            od = torch.empty_like(xd)
            tdp.tdp_stage_decode(st.h, xd, i32(ctx), tab_d, n, od)
            torch.cuda.synchronize()
            refd, caches = O.stage_decode(list(f64(xd)), caches, layers, osh)
            e2 = row_rel_err(f64(od), np.stack(refd))
            assert e2 <= TOL, (step, e2)
            err = max(err, e2)
            ctx = ctx + 1
        return err


# ----------------------------------------------------------------------------- GEMM alone

@pytest.mark.parametrize("M,N,K,tile,splits,epi", [
    # the planner's own choice
    (4, 768, 256, 0, 0, 0), (4, 256, 704, 0, 0, 1), (33, 320, 128, 0, 2, 0), (64, 512, 512, 0, 1, 1),
    (512, 1280, 2048, 0, 0, 0), (1000, 256, 64, 0, 0, 1), (257, 516, 192, 0, 2, 1),
    # every kernel variant (1: 256 x 256 tile, 2: 128 x 256, 3: 128 x 128), ragged M and N, split-K
    (300, 768, 1024, 1, 1, 0), (257, 516, 192, 1, 2, 1), (513, 520, 448, 1, 2, 1),
    (300, 516, 256, 1, 1, 1), (513, 260, 128, 1, 1, 1),   # whole-tile residual epilogue, ragged M and N
    (100, 384, 256, 2, 3, 0), (130, 1024, 320, 2, 1, 1), (70, 260, 128, 2, 1, 0), (65, 512, 256, 2, 2, 1),
    (100, 384, 256, 3, 2, 0), (300, 640, 1024, 3, 1, 1), (7, 256, 512, 3, 4, 1),
])
def test_gemm_matches_fp64_product(tdp, M, N, K, tile, splits, epi):
    g = torch.Generator(device="cpu").manual_seed(M * 131 + N)
    A = torch.randn(M, K, generator=g).to(torch.bfloat16).cuda()
    Wm = (torch.randn(K, N, generator=g) * 0.05).to(torch.bfloat16).cuda()
    R = torch.randn(M, N, generator=g).to(torch.bfloat16).cuda()
    out = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    tdp.tdp_gemm_bf16(A, Wm, R if epi else None, out, M, N, K, epi, tile, splits)
    ref = f64(A) @ f64(Wm) + (f64(R) if epi else 0.0)
    assert row_rel_err(f64(out), ref) <= 1e-2


@pytest.mark.parametrize("M,F,K,tile,splits", [
    (4, 688, 256, 0, 0), (33, 128, 128, 2, 2), (130, 344, 320, 2, 1), (300, 1376, 1024, 1, 1), (257, 516, 192, 1, 2),
    (100, 64, 256, 3, 1), (512, 1024, 2048, 0, 0), (70, 260, 512, 3, 3),
])
def test_gated_mlp_epilogue_matches_the_fp64_definition(tdp, M, F, K, tile, splits):
    """The gate/up projection with its fused epilogue alone: out = silu(A W_gate) * (A W_up), every kernel
    variant, ragged M and F (F not a multiple of the 32-row gate/up interleave), with and without split-K
    (split-K sums the partials before the activation).  Gate pre-activations span about +-6, so both
    tails of the sigmoid and its middle are exercised."""
    g = torch.Generator(device="cpu").manual_seed(M * 977 + F)
    A = torch.randn(M, K, generator=g).to(torch.bfloat16).cuda()
    Wg = (torch.randn(K, F, generator=g) * (2.0 / K ** 0.5)).to(torch.bfloat16)
    Wu = (torch.randn(K, F, generator=g) * (1.0 / K ** 0.5)).to(torch.bfloat16)
    Wm = torch.cat([Wg, Wu], dim=1).contiguous().cuda()
    out = torch.full((M, F), float("nan"), dtype=torch.bfloat16, device="cuda")
    tdp.tdp_gemm_bf16(A, Wm, None, out, M, 2 * F, K, 2, tile, splits)
    gate = f64(A) @ f64(Wg)
    ref = gate / (1.0 + np.exp(-gate)) * (f64(A) @ f64(Wu))
    assert np.abs(gate).max() > 4.0
    assert row_rel_err(f64(out), ref) <= 1e-2


# ----------------------------------------------------------------------------- the stage

def test_decode_tiny_config(tdp):
    """Benchmark configuration 0: batch 4, contexts uniform in [16, 64], random block tables."""
    run_decode_case(tdp, "tiny", W.decode_ctx_lens("tiny", 4))


def test_prefill_tiny_config(tdp):
    """Benchmark configuration 0: 4 prompts, lengths uniform in [8, 32]."""
    run_prefill_case(tdp, "tiny", W.prefill_seq_lens("tiny", 4))


@pytest.mark.parametrize("shape", ["tiny", "tiny_gqa", "tiny_h128", "tiny_bias", "tiny_mqa", "tiny_g2"])
def test_prefill_then_decode_across_page_boundaries(tdp, shape):
    run_prefill_case(tdp, shape, [1, 15, 16, 17, 33, 70], decode_steps=3)


@pytest.mark.parametrize("shape", ["tiny_gqa", "tiny_h128", "tiny_bias", "tiny_mqa", "tiny_g2"])
def test_decode_edge_contexts(tdp, shape):
    """ctx = 0 (attention over the token itself), page edges, split edges (256 tokens per split)."""
    run_decode_case(tdp, shape, [0, 1, 15, 16, 31, 32, 255, 256, 257, 511, 512, 700])


def test_decode_batch_above_512_and_prefill_of_many_short_prompts(tdp):
    """Sizes on the far side of two internal limits: more than 512 decode rows (no split-K workspace is
    sized beyond that; the planner's work list takes several requests per thread) and more prompts than
    a prefill workgroup usually walks past when it looks for its sequence."""
    rng = np.random.default_rng(520)
    run_decode_case(tdp, "tiny_gqa", rng.integers(0, 41, size=520))
    run_prefill_case(tdp, "tiny_gqa", rng.integers(1, 8, size=300), decode_steps=1)


def test_one_request_and_one_token(tdp):
    """The smallest calls: a decode batch of one request, a prefill of one prompt of one token."""
    run_decode_case(tdp, "tiny_gqa", [37])
    run_decode_case(tdp, "tiny_h128", [0])
    run_prefill_case(tdp, "tiny", [1], decode_steps=2)


def test_model_dimension_above_8192(tdp):
    """Rows longer than 8192 elements: the row-wise kernels loop where they otherwise hold a row in
    registers; decode at a batch that splits K (partials summed by the consumers) and a prefill."""
    run_decode_case(tdp, "tiny_wide", [3, 40, 17, 0, 100, 64, 31, 5])
    run_prefill_case(tdp, "tiny_wide", [20, 1, 33], decode_steps=1)


@pytest.mark.parametrize("shape,ctx,n_layers", [
    ("tiny_gqa", [0, 1, 15, 16, 31, 255, 256, 257, 700, 40, 3], None),     # odd batch: halves of 6 and 5
    ("tiny", [20, 33], None),                                              # one request per half
    ("tiny_h128", [64], None),                                             # a batch of one takes the plain path
    ("7b_quarter", None, 2),                                               # batch 200: split-K partials in both halves
])
def test_decode_as_two_half_batches_on_two_streams(tdp, shape, ctx, n_layers):
    """decode_micro_batches = 2: the batch runs as two halves, the second on the stage's own second
    stream with its own scratch buffers, forked from and joined to the caller's stream.  Outputs, the
    appended K/V and every untouched slot are held to the same bounds as the one-batch form."""
    if ctx is None:
        ctx = np.minimum(W.decode_ctx_lens(shape, 200), 300)
    run_decode_case(tdp, shape, ctx, n_layers=n_layers, micro_batches=2)


def test_two_half_batches_follow_the_callers_stream(tdp):
    """The forked second stream must wait for work queued earlier on the caller's stream (here: the copy that
    produces the input) and the caller's stream must wait for it (here: the copy of the output), on a
    stream that is not the default one; repeated, so that a later step may not overtake an earlier one."""
    sh = W.SHAPES["tiny_gqa"]
    ctx = np.array([5, 40, 300, 77, 16, 255, 31], dtype=np.int64)
    batch = W.make_decode_batch(ctx)
    B = len(ctx)
    outs = {}
    for micro in (0, 2):
        with Stage(tdp, sh, batch.num_pages, B, 0, 0, batch.tables.shape[1], decode_micro_batches=micro) as st:
            import_kv(tdp, st, ctx, batch.tables, 9)
            src = W.hidden_states(sh, B, 9, device="cuda")
            ctx_d, tab_d = i32(ctx), i32(batch.tables)
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            got = []
            with torch.cuda.stream(side):
                for rep in range(4):
                    x = torch.zeros_like(src)
                    out = torch.zeros_like(src)
                    x.copy_(src, non_blocking=True)                       # queued on `side`, just before the call
                    tdp.tdp_stage_decode(st.h, x, ctx_d, tab_d, B, out, side)
                    got.append(out.clone())                               # queued on `side`, right behind it
            side.synchronize()
            outs[micro] = [g.view(torch.int16).cpu() for g in got]
    for rep in range(4):
        assert torch.equal(outs[2][rep], outs[2][0])
        # the halves take other tile shapes than the whole batch, so the two forms agree within rounding
        a = outs[2][rep].view(torch.bfloat16).double().numpy()
        b = outs[0][rep].view(torch.bfloat16).double().numpy()
        assert row_rel_err(a, b) <= 1e-2


def test_decode_is_invariant_under_block_table_permutation(tdp):
    sh = W.SHAPES["tiny_gqa"]
    ctx = np.array([5, 40, 300, 77], dtype=np.int64)
    outs = []
    for seed in (1, 2):
        batch = W.make_decode_batch(ctx, seed=seed)
        with Stage(tdp, sh, batch.num_pages, 4, 0, 0, batch.tables.shape[1]) as st:
            st.poison()
            import_kv(tdp, st, ctx, batch.tables, 9)
            x = W.hidden_states(sh, 4, 9, device="cuda")
            out = torch.empty_like(x)
            tdp.tdp_stage_decode(st.h, x, i32(ctx), i32(batch.tables), 4, out)
            torch.cuda.synchronize()
            outs.append(out.view(torch.int16).cpu())
    assert torch.equal(outs[0], outs[1])


def test_requests_are_independent_on_the_gpu(tdp):
    """A request's output does not depend on the rest of the batch: bit-identical alone / in a batch
    is not promised (tile shapes differ), the tolerance is."""
    sh = W.SHAPES["tiny"]
    ctx = np.array([20, 33, 64], dtype=np.int64)
    batch = W.make_decode_batch(ctx)
    with Stage(tdp, sh, batch.num_pages, 3, 0, 0, batch.tables.shape[1]) as st:
        import_kv(tdp, st, ctx, batch.tables, 4)
        x = W.hidden_states(sh, 3, 4, device="cuda")
        out = torch.empty_like(x)
        tdp.tdp_stage_decode(st.h, x, i32(ctx), i32(batch.tables), 3, out)
        solo = torch.empty_like(x[1:2])
        tdp.tdp_stage_decode(st.h, x[1:2].contiguous(), i32(ctx[1:2]), i32(batch.tables[1:2]), 1, solo)
        torch.cuda.synchronize()
        assert row_rel_err(f64(solo), f64(out[1:2])) <= 1e-2


def test_empty_batches_are_no_ops_and_limits_are_enforced(tdp):
    sh = W.SHAPES["tiny"]
    with Stage(tdp, sh, 8, 4, 64, 4, 4, load_weights=False) as st:
        tdp.tdp_stage_decode(st.h, None, None, None, 0, None)
        tdp.tdp_stage_prefill(st.h, None, None, None, 0, 0, None)
        x = torch.zeros(8, sh.d_model, dtype=torch.bfloat16, device="cuda")
        with pytest.raises(tdp.TdpError) as e:
            tdp.tdp_stage_decode(st.h, x, i32([1] * 5), i32(np.zeros((5, 4))), 5, x)
        assert e.value.code == tdp.EINVAL
        with pytest.raises(tdp.TdpError):
            tdp.tdp_stage_prefill(st.h, x, i32([0, 65]), i32(np.zeros((1, 4))), 1, 65, x)
        with pytest.raises(tdp.TdpError):
            tdp.tdp_stage_set_weight(st.h, 0, tdp.WQ, x, tdp.BF16, tdp.DEVICE, 3, 3)


def test_layer_range_composes_to_the_whole_stage(tdp):
    """Running layers [0,1) then [1,2) with a bf16 hand-over in between is a two-stage pipeline of
    the same model: it must agree with the oracle like the one-stage run does, and the range must
    be validated."""
    sh = W.SHAPES["tiny_gqa"]
    ctx = np.array([3, 40, 100, 17], dtype=np.int64)
    batch = W.make_decode_batch(ctx)
    with Stage(tdp, sh, batch.num_pages, 4, 0, 0, batch.tables.shape[1]) as st:
        caches = import_kv(tdp, st, ctx, batch.tables, 8)
        x = W.hidden_states(sh, 4, 8, device="cuda")
        mid, out = torch.empty_like(x), torch.empty_like(x)
        tdp.tdp_stage_set_layer_range(st.h, 0, 1)
        tdp.tdp_stage_decode(st.h, x, i32(ctx), i32(batch.tables), 4, mid)
        tdp.tdp_stage_set_layer_range(st.h, 1, 1)
        tdp.tdp_stage_decode(st.h, mid, i32(ctx), i32(batch.tables), 4, out)
        tdp.tdp_stage_set_layer_range(st.h, 0, 0)
        torch.cuda.synchronize()
        ref, _ = O.stage_decode(list(f64(x)), caches, list(oracle_layers(sh)), oracle_shape(sh))
        assert row_rel_err(f64(out), np.stack(ref)) <= TOL
        for first, count in ((-1, 1), (0, 3), (2, 1), (1, -1)):
            with pytest.raises(tdp.TdpError):
                tdp.tdp_stage_set_layer_range(st.h, first, count)


def test_fp32_and_host_weights_are_rounded_like_bf16_weights(tdp):
    sh = W.SHAPES["tiny"]
    ctx = np.array([16, 40], dtype=np.int64)
    batch = W.make_decode_batch(ctx)
    outs = []
    for mode in ("bf16_dev", "f32_host"):
        with Stage(tdp, sh, batch.num_pages, 2, 0, 0, batch.tables.shape[1], load_weights=False) as st:
            if mode == "bf16_dev":
                # fp32 source rounded to bf16 by torch, handed over on the device
                for l in range(sh.n_layers):
                    for name in W.WEIGHT_NAMES:
                        w = W.weight(sh, l, name, device="cuda", dtype=torch.float32).to(torch.bfloat16).contiguous()
                        tdp.tdp_stage_set_weight(st.h, l, tdp.WEIGHT_IDS[name], w, tdp.BF16, tdp.DEVICE,
                                                 w.shape[0], w.shape[1] if w.dim() == 2 else 1)
            else:
                for l in range(sh.n_layers):
                    for name in W.WEIGHT_NAMES:
                        w = W.weight(sh, l, name, device="cpu", dtype=torch.float32)
                        if name.startswith("g_"):
                            w = w.to(torch.bfloat16).to(torch.float32)   # same gains in both runs
                        w = w.contiguous()
                        tdp.tdp_stage_set_weight(st.h, l, tdp.WEIGHT_IDS[name], w, tdp.F32, tdp.HOST,
                                                 w.shape[0], w.shape[1] if w.dim() == 2 else 1)
            import_kv(tdp, st, ctx, batch.tables, 6)
            x = W.hidden_states(sh, 2, 6, device="cuda")
            out = torch.empty_like(x)
            tdp.tdp_stage_decode(st.h, x, i32(ctx), i32(batch.tables), 2, out)
            torch.cuda.synchronize()
            outs.append(out.view(torch.int16).cpu())
    assert torch.equal(outs[0], outs[1])


# ----------------------------------------------------------------------------- several tiles, ragged tails

def test_decode_13b_shaped_layer_many_tiles(tdp):
    """One 13B-shaped layer: 40 heads x 128, FFN 13824; batch 40 with contexts up to ~900 tokens
    (several KV splits, ragged last pages, ragged M tile)."""
    ctx = W.decode_ctx_lens("13b_quarter", 40)
    ctx = np.minimum(ctx, 900)
    run_decode_case(tdp, "13b_quarter", ctx, n_layers=1)


def test_prefill_7b_shaped_layer_many_tiles(tdp):
    """One 7B-shaped layer, 5 prompts of ragged length (total 527 tokens: three M tiles)."""
    run_prefill_case(tdp, "7b_quarter", [200, 31, 129, 64, 103], n_layers=1)


@pytest.mark.parametrize("shape,seq_lens", [
    # one head per workgroup (multi-head attention and groups that no power of two divides): a query
    # tile is 256 positions
    ("tiny", [4096]),                       # head_dim 64, sixteen query tiles, 257 pages
    ("tiny", [257, 300, 513, 1000, 256]),   # tile edges: one position into a second tile, exact multiples
    ("tiny_bias", [700, 259]),              # group of 5 -> one head per workgroup
    # two heads per workgroup: 128 positions per tile
    ("tiny_g2", [300, 129, 257, 128]),
    # four and eight heads per workgroup: 64 and 32 positions per tile
    ("tiny_gqa", [200, 65, 64, 449]),
    ("tiny_h128", [130, 577]),
    ("tiny_mqa", [100, 33, 32, 290]),
])
def test_prefill_attention_beyond_one_query_tile(tdp, shape, seq_lens):
    """Prompts longer than one query tile of every prefill-attention variant (Sec. 2.1: the prefill
    phase processes all tokens of a prompt at once): later tiles start at a position above zero, skip
    the key blocks beyond their diagonal and stop at their own end of the prompt.  Outputs, the cached
    keys and values and the untouched slots are compared as in the short cases; one decode step
    follows on the cache the prefill wrote."""
    run_prefill_case(tdp, shape, seq_lens, decode_steps=1)


def test_prefill_7b_shaped_layer_prompts_of_several_query_tiles(tdp):
    """One 7B-shaped layer (32 heads x 128, multi-head attention: 256 query positions per workgroup)
    on prompts of 257 to 1000 tokens."""
    run_prefill_case(tdp, "7b_quarter", [257, 300, 513, 1000], n_layers=1)


def test_prefill_13b_shaped_layer_longest_prompt_of_its_benchmark_batch(tdp):
    """One 13B-shaped layer (40 heads x 128) on a prompt as long as the longest of the 32-prompt
    benchmark batch (1838 tokens: eight query tiles per head)."""
    run_prefill_case(tdp, "13b_quarter", [int(W.prefill_seq_lens("13b_quarter", 32).max())], n_layers=1)


def test_decode_70b_shaped_layer_gqa(tdp):
    """One 70B-shaped layer (64 query heads on 8 KV heads), batch 24."""
    ctx = np.minimum(W.decode_ctx_lens("70b_quarter", 24), 700)
    run_decode_case(tdp, "70b_quarter", ctx, n_layers=1)


@pytest.mark.parametrize("shape", ["7b_quarter", "qwen32b_quarter"])
def test_decode_batch_200_two_layers_split_k_summed_by_the_consumers(tdp, shape):
    """At 192 rows and more the projections whose K range is split leave their partial sums to the
    next kernel (RoPE + KV append sums the QKV partials and adds the bias, the following RMSNorm sums
    the O and down partials together with the residual); two layers so that the second layer's first
    norm is fed that way.  Contexts up to 300 tokens."""
    ctx = np.minimum(W.decode_ctx_lens(shape, 200), 300)
    run_decode_case(tdp, shape, ctx, n_layers=2)


@pytest.mark.parametrize("shape", ["7b_quarter", "qwen32b_quarter"])
def test_prefill_292_tokens_two_layers_split_k_summed_by_the_consumers(tdp, shape):
    """A short prefill (192 to 512 packed tokens) also splits K and leaves the sums to RoPE and to
    the norms; four prompts of ragged length, two layers, one decode step behind it."""
    run_prefill_case(tdp, shape, [120, 31, 77, 64], n_layers=2, decode_steps=1)


def test_a_dropped_bias_would_be_caught(tdp):
    """The biased stage must differ from the same stage without biases by far more than the
    tolerance: otherwise the bias tests above would pass vacuously."""
    from dataclasses import replace
    sh = W.SHAPES["tiny_bias"]
    ctx = np.array([5, 40], dtype=np.int32)
    outs = []
    for biased in (True, False):
        db = W.make_decode_batch(ctx)
        with Stage(tdp, replace(sh, qkv_bias=biased), db.num_pages, 2, 0, 0, db.tables.shape[1]) as st:
            cu = np.array([0, 5, 45], dtype=np.int32)
            k = W.kv_packed(sh, 0, "k", 45, 1, device="cuda")
            for l in range(sh.n_layers):
                tdp.tdp_stage_kv_import(st.h, l, k, k, i32(cu), i32(db.tables), 2, 45)
            x = W.hidden_states(sh, 2, 1, device="cuda")
            out = torch.empty_like(x)
            tdp.tdp_stage_decode(st.h, x, i32(ctx), i32(db.tables), 2, out)
            torch.cuda.synchronize()
            outs.append(f64(out))
    assert row_rel_err(outs[0], outs[1]) > 3 * TOL


@pytest.mark.parametrize("span", [256, 512, 1024, 2048, 4096])
def test_decode_every_span_length(tdp, span):
    """The library picks the span length (tokens of one context handled by one workgroup) from the
    batch size; tdp_stage_set_decode_span pins it.  Contexts sit on and around the span boundaries, so
    requests finish inside one workgroup, need exactly two partials, or end one token into a span."""
    ctx = sorted({0, 31, span - 2, span - 1, span, span + 1, 2 * span - 1, 2 * span, 2 * span + 33,
                  min(3 * span + 7, 4096)} & set(range(0, 4097)))
    run_decode_case(tdp, "tiny_gqa", ctx, n_layers=1, max_pages_per_seq=4096 // 16 + 1, span=span)
    with Stage(tdp, W.SHAPES["tiny"], 4, 1, 0, 0, 2, load_weights=False) as st:
        with pytest.raises(tdp.TdpError):
            tdp.tdp_stage_set_decode_span(st.h, 300)


@pytest.mark.parametrize("shape", ["tiny", "tiny_h128", "tiny_gqa"])
def test_import_puts_every_element_where_the_documented_layout_says(tdp, shape):
    """The pools' layout is part of the ABI (tdp_stage_kv_pool): keys in 64-byte pieces, piece g of a page's
    16 tokens together; values with the token slot fastest.  Imported keys and values are found, bit
    for bit, at the addresses the header's formula gives (Stage.pools undoes the piece order by that
    formula), nothing else is touched, and export returns them."""
    sh = W.SHAPES[shape]
    lens = np.array([1, 16, 37, 5, 64], dtype=np.int64)
    batch = W.make_decode_batch(lens)
    with Stage(tdp, sh, batch.num_pages, len(lens), 0, 0, batch.tables.shape[1], load_weights=False) as st:
        st.poison()
        caches = import_kv(tdp, st, lens, batch.tables, 5)
        mk, mv = written_slot_mask(st, batch.tables, np.zeros(len(lens), dtype=np.int64), lens)
        for l in range(sh.n_layers):
            k_pool, v_pool = (t.float().cpu() for t in st.pools(l))
            assert bool(torch.isnan(k_pool[~mk]).all()) and bool(torch.isnan(v_pool[~mv]).all())
            for b in range(len(lens)):
                k_ref, v_ref = caches[b][l]
                for p in range(int(lens[b])):
                    page, slot = int(batch.tables[b, p // 16]), p % 16
                    assert np.array_equal(k_pool[page, :, slot, :].numpy().astype(np.float64), k_ref[p])
                    assert np.array_equal(v_pool[page, :, :, slot].numpy().astype(np.float64), v_ref[p])
            kx, vx, cu = export_kv(tdp, st, lens, batch.tables, l)
            for b in range(len(lens)):
                assert np.array_equal(kx[cu[b]:cu[b + 1]], caches[b][l][0])
                assert np.array_equal(vx[cu[b]:cu[b + 1]], caches[b][l][1])


@pytest.mark.parametrize("span", [0, 256, 4096])
def test_decode_contexts_far_beyond_the_benchmark(tdp, span):
    """Contexts of up to 20,000 tokens (the benchmark stops at 4096): dozens of spans per request
    (79 at the shortest span length), page lists of over a thousand entries, and a batch that mixes
    them with a one-token context."""
    ctx = [20000, 0, 9000, 16383, 16384, 4097, 12345]
    run_decode_case(tdp, "tiny_gqa", ctx, n_layers=1, max_pages_per_seq=20000 // 16 + 2, span=span)


def test_decode_step_replays_from_a_hip_graph(tdp):
    """A serving loop would capture the decode step once and replay it: the call only enqueues
    kernels on the stream it is given (no allocation, no synchronisation, no memset node), so it
    can be recorded into a HIP graph.  Three replays, with eager work and synchronisations between
    them, must each reproduce the eager result bit for bit."""
    sh = W.SHAPES["tiny_gqa"]
    ctx = np.array([5, 40, 300, 77, 16, 255], dtype=np.int64)
    batch = W.make_decode_batch(ctx)
    B = len(ctx)
    with Stage(tdp, sh, batch.num_pages, B, 0, 0, batch.tables.shape[1]) as st:
        st.poison()
        import_kv(tdp, st, ctx, batch.tables, 9)
        x = W.hidden_states(sh, B, 9, device="cuda")
        ctx_d, tab_d = i32(ctx), i32(batch.tables)
        eager = torch.empty_like(x)
        tdp.tdp_stage_decode(st.h, x, ctx_d, tab_d, B, eager)        # also warms every plan up
        torch.cuda.synchronize()
        out = torch.zeros_like(x)
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                tdp.tdp_stage_decode(st.h, x, ctx_d, tab_d, B, out, torch.cuda.current_stream())
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        for rep in range(3):
            out.zero_()
            scratch = torch.randn(1 << 16, device="cuda").sum()       # unrelated eager work in between
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(out.view(torch.int16), eager.view(torch.int16)), rep
            del scratch

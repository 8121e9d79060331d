"""GPU parity of the 8-bit (E4M3) KV-cache option, through the C ABI, against oracle/fp8_oracle.py and
the cache option of oracle/stage_oracle.py.

What is exact and what is not.  The conversions themselves are integer decisions and are compared
bit for bit: every code decodes to the value the format gives it, and a given fp32 number and scale
give the same code on both sides (the quotient is an fp32 division on both sides).  Cache contents
that come from an import are therefore bit-exact.  A key or value the stage computes itself is
rounded from a number that already differs from the oracle's by the bf16 error of the projection,
so near a rounding boundary the two sides may store neighbouring codes: such entries are checked to
be within one code step (2^-3 of the element at most), to agree wherever the oracle's number is
further from every boundary than the bf16 tolerance, and to disagree rarely.  Outputs are held to
the usual 2e-2 of the row maximum; a token that attends to fewer than 15 cached tokens gives a
single freshly stored entry a weight of up to 1, so for those rows one code step (2^-3) is added to
the bound.
"""
import numpy as np
import pytest
import torch

from harness import workload as W
from oracle import fp8_oracle as F8
from oracle import stage_oracle as O
from stage_helpers import TOL, Stage, f64, i32, oracle_layers, oracle_shape

pytestmark = pytest.mark.gpu

STEP = 2.0 ** -3        # largest relative distance between neighbouring E4M3 values
SHORT_CTX = 15
EQUAL_CODES = []        # fraction of equal codes of every stored token that was checked (printed at the end)


@pytest.fixture(scope="module")
def tdp():
    from paper_2506_10470_amd import tdp as _tdp
    return _tdp


def q8_shape(sh, scales):
    o = oracle_shape(sh)
    o.kv_scales = tuple(scales)
    return o


def ordinal(codes):
    """Codes as signed integers in value order (neighbouring values differ by one)."""
    c = np.asarray(codes).astype(np.int64)
    return np.where(c & 0x80, -(c & 0x7F), c & 0x7F)


def row_errs(got, ref):
    got = np.asarray(got, np.float64).reshape(-1, ref.shape[-1])
    ref = np.asarray(ref, np.float64).reshape(-1, ref.shape[-1])
    assert np.isfinite(got).all(), "non-finite output"
    denom = np.max(np.abs(ref), axis=-1)
    return np.max(np.abs(got - ref), axis=-1) / np.where(denom == 0, 1.0, denom)


def row_tolerances(ctx_lens):
    return np.where(np.asarray(ctx_lens) >= SHORT_CTX, TOL, TOL + STEP)


# ----------------------------------------------------------------------------- the conversions

def test_every_code_decodes_to_the_value_the_format_gives_it(tdp):
    codes = torch.arange(256, dtype=torch.uint8, device="cuda")
    out = torch.full((256,), 7.0, dtype=torch.float32, device="cuda")
    tdp.tdp_e4m3_to_f32(codes, out, 256)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    want = F8.e4m3_decode_table()
    assert np.array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok], want[ok]) and np.array_equal(np.signbit(got[ok]), np.signbit(want[ok]))


@pytest.mark.parametrize("scale", [1.0, 0.5, 8.0, 3.0, 0.7])
def test_encoder_gives_the_oracle_code_for_every_input(tdp, scale):
    rng = np.random.default_rng(int(scale * 100))
    table = F8.e4m3_decode_table()[:0x7F]
    mids = ((table[:-1] + table[1:]) / 2).astype(np.float32)
    f32 = np.float32
    x = np.concatenate([
        rng.normal(0, 1, 50000), rng.normal(0, 150, 50000), rng.uniform(-0.04, 0.04, 50000),
        mids * f32(scale), -mids * f32(scale), np.nextafter(mids * f32(scale), f32(np.inf)),
        np.nextafter(mids * f32(scale), f32(-np.inf)), table * scale, -table * scale,
        [0.0, -0.0, np.inf, -np.inf, np.nan, 448.0 * scale, 464.0 * scale, 1e30, -1e30, 1e-40, -1e-45],
    ]).astype(np.float32)
    n = len(x) // 4 * 4
    x = x[:n]
    src = torch.from_numpy(x).cuda()
    out = torch.zeros(n, dtype=torch.uint8, device="cuda")
    tdp.tdp_e4m3_from_f32(src, out, n, scale)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    want = F8.kv_quantize(x, scale, np.float32)
    nan = np.isnan(x)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.all((got[nan] & 0x7F) == 0x7F)


# ----------------------------------------------------------------------------- import / export

def packed_kv(sh, layer, total, stream_id):
    k = W.kv_packed(sh, layer, "k", total, stream_id, device="cuda")
    v = W.kv_packed(sh, layer, "v", total, stream_id, device="cuda")
    return k, v


def import_kv(tdp, st, lens, tables, stream_id, scales):
    """Fill pages from generated bf16 K/V; returns per-sequence oracle caches (what the cache holds)."""
    sh = st.shape
    lens = np.asarray(lens, dtype=np.int64)
    total = int(lens.sum())
    cu = np.zeros(len(lens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lens)
    caches = [[None] * sh.n_layers for _ in lens]
    cu_d, tab_d = i32(cu), i32(tables)
    for l in range(sh.n_layers):
        if total:
            k, v = packed_kv(sh, l, total, stream_id)
            tdp.tdp_stage_kv_import(st.h, l, k, v, cu_d, tab_d, len(lens), total)
            torch.cuda.synchronize()
            kc, vc = F8.kv_roundtrip(f64(k), scales[0]), F8.kv_roundtrip(f64(v), scales[1])
        else:
            kc = vc = np.zeros((0, sh.n_kv_heads, sh.head_dim))
        for b in range(len(lens)):
            caches[b][l] = (kc[cu[b]:cu[b + 1]], vc[cu[b]:cu[b + 1]])
    return caches


def export_kv(tdp, st, lens, tables, layer):
    sh = st.shape
    total = int(np.sum(lens))
    cu = np.zeros(len(lens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lens)
    k = torch.empty(total, sh.n_kv_heads, sh.head_dim, dtype=torch.bfloat16, device="cuda")
    v = torch.empty_like(k)
    tdp.tdp_stage_kv_export(st.h, layer, k, v, i32(cu), i32(tables), len(lens), total)
    torch.cuda.synchronize()
    return f64(k), f64(v), cu


def slot_codes(st, layer, page, slot):
    """Codes of one token: (K [Hkv, dh], V [Hkv, dh]) read from the documented pool layout."""
    k_pool, v_pool = st.pools(layer)
    return k_pool[page, :, slot, :].cpu().numpy(), v_pool[page, :, :, slot].cpu().numpy()


@pytest.mark.parametrize("shape,scales", [("tiny", (1.0, 1.0)), ("tiny_h128", (0.5, 4.0)), ("tiny_gqa", (0.7, 1.3))])
def test_import_stores_the_oracle_codes_where_the_layout_says_and_export_reads_them_back(tdp, shape, scales):
    sh = W.SHAPES[shape]
    lens = np.array([1, 16, 37, 5], dtype=np.int64)
    batch = W.make_decode_batch(lens)
    total = int(lens.sum())
    cu = np.zeros(5, dtype=np.int64)
    cu[1:] = np.cumsum(lens)
    with Stage(tdp, sh, batch.num_pages, 4, 0, 0, batch.tables.shape[1], load_weights=False, kv_scales=scales) as st:
        st.poison()
        import_kv(tdp, st, lens, batch.tables, 3, scales)
        for l in range(sh.n_layers):
            k, v = packed_kv(sh, l, total, 3)
            want_k, want_v = F8.kv_quantize(f64(k), scales[0]), F8.kv_quantize(f64(v), scales[1])
            k_pool, v_pool = (t.cpu().numpy() for t in st.pools(l))
            seen_k = np.zeros(k_pool.shape, bool)
            seen_v = np.zeros(v_pool.shape, bool)
            for b in range(4):
                for p in range(int(lens[b])):
                    page, slot = int(batch.tables[b, p // 16]), p % 16
                    assert np.array_equal(k_pool[page, :, slot, :], want_k[cu[b] + p])
                    assert np.array_equal(v_pool[page, :, :, slot], want_v[cu[b] + p])
                    seen_k[page, :, slot, :] = True
                    seen_v[page, :, :, slot] = True
            assert np.all(k_pool[~seen_k] == Stage.POISON_CODE) and np.all(v_pool[~seen_v] == Stage.POISON_CODE)
            kx, vx, _ = export_kv(tdp, st, lens, batch.tables, l)
            # export returns bf16(code value * scale): exact for power-of-two scales, one bf16 rounding otherwise
            bf = lambda a: torch.from_numpy(a.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
            assert np.array_equal(kx, bf(F8.e4m3_decode(want_k).astype(np.float32) * np.float32(scales[0])))
            assert np.array_equal(vx, bf(F8.e4m3_decode(want_v).astype(np.float32) * np.float32(scales[1])))


# ----------------------------------------------------------------------------- the stage

def check_stored_token(hip_codes, pre, scale, what):
    """hip_codes: codes the stage stored for one token [Hkv, dh]; pre: the oracle's unrounded values."""
    q = np.asarray(pre, np.float64) / scale
    ref = F8.e4m3_encode(q)
    d = np.abs(ordinal(hip_codes) - ordinal(ref))
    got, want = F8.e4m3_decode(hip_codes), F8.e4m3_decode(ref)
    # neighbouring codes at most; entries far below the row maximum (where a step is tiny and the
    # bf16 error of the sum that produced them is not) may differ by that error instead
    small = np.abs(got - want) <= 2.0 ** -7 * np.max(np.abs(want), axis=-1, keepdims=True)
    assert np.all((d <= 1) | small), (what, "codes more than one step apart", int(np.max(d)))
    # How often the two sides may differ.  The stage's number carries the error of a bf16-operand
    # projection: about 2^-9 / sqrt(3) = 1.1e-3 of the row's rms r (each input is rounded to 8 significant
    # bits, the sum is fp32), plus, for values, their own rounding to bf16 (at most 2^-9 of the element).
    # A rounding boundary falls between the two numbers with probability |error| / step, and the steps of
    # the format are 1/16 to 1/8 of the element: about 1 % for an element as large as r, growing as
    # r / |element| below it; averaged over normally distributed elements 4 to 6 %.  One token's entries
    # (64 to 1024 of them) are held to that rate plus four standard deviations of a binomial count; all
    # tokens of a run together to 93 % equal codes (test_zz_equal_code_fraction_over_the_run).
    EQUAL_CODES.append((int(np.sum(d == 0)), int(d.size)))
    n_el, p_flip = d.size, 0.06
    allowed = n_el * p_flip + 4.0 * np.sqrt(n_el * p_flip * (1.0 - p_flip)) + 1.0
    assert np.sum(d != 0) <= allowed, (what, "too many neighbouring codes", int(np.sum(d != 0)), n_el)
    # Where the oracle's number is further from both neighbouring boundaries than the bf16 error of the
    # stage's own number, the code is decided and must be the same.  That error: the projection is
    # stored in bf16 (2^-9 of the element), the rotation mixes two such entries (2^-9 of the row
    # maximum each); the margin allows four units of the first and two of the second.
    table = F8.e4m3_decode_table()[:0x7F]
    mids = (table[:-1] + table[1:]) / 2
    mag = np.abs(q)
    dist = np.min(np.abs(mag[..., None] - mids[None, None, :]), axis=-1)
    margin = 2.0 ** -7 * mag + 2.0 ** -8 * np.max(mag, axis=-1, keepdims=True)
    decided = dist > margin
    assert decided.mean() > 0.1, what        # the check must not be vacuous
    assert np.array_equal(np.asarray(hip_codes)[decided], ref[decided]), what
    # and the stored values are within one step of the oracle's stored values (a step is at most 2^-3 of the
    # element, hence of the row maximum)
    assert np.all(row_errs(got, want) <= STEP), what


def run_decode_case(tdp, shape_name, ctx_lens, scales, n_layers=None, stream_id=1, max_pages_per_seq=None, span=0):
    sh = W.SHAPES[shape_name]
    if n_layers:
        sh = sh.with_layers(n_layers)
    ctx_lens = np.asarray(ctx_lens, dtype=np.int64)
    B = len(ctx_lens)
    batch = W.make_decode_batch(ctx_lens, max_pages_per_seq=max_pages_per_seq)
    with Stage(tdp, sh, batch.num_pages, B, 0, 0, batch.tables.shape[1], kv_scales=scales) as st:
        st.poison()
        tdp.tdp_stage_set_decode_span(st.h, span)
        caches = import_kv(tdp, st, ctx_lens, batch.tables, stream_id, scales)
        before = [tuple(t.clone() for t in st.pools(l)) for l in range(sh.n_layers)]
        x = W.hidden_states(sh, B, stream_id, device="cuda")
        out = torch.empty_like(x)
        tdp.tdp_stage_decode(st.h, x, i32(batch.ctx_lens), i32(batch.tables), B, out)
        torch.cuda.synchronize()
        layers = list(oracle_layers(sh))
        ref, new_caches = O.stage_decode(list(f64(x)), caches, layers, q8_shape(sh, scales))
        errs = row_errs(f64(out), np.stack(ref))
        assert np.all(errs <= row_tolerances(ctx_lens)), (errs, ctx_lens)
        for l in range(sh.n_layers):
            k_after, v_after = st.pools(l)
            kb, vb = before[l]
            changed_k = (k_after != kb).cpu().numpy()
            changed_v = (v_after != vb).cpu().numpy()
            allowed_k = np.zeros_like(changed_k)
            allowed_v = np.zeros_like(changed_v)
            for b in range(B):
                page, slot = int(batch.tables[b, ctx_lens[b] // 16]), int(ctx_lens[b] % 16)
                allowed_k[page, :, slot, :] = True
                allowed_v[page, :, :, slot] = True
            assert not np.any(changed_k & ~allowed_k) and not np.any(changed_v & ~allowed_v), "a slot outside the append changed"
        # layer 0 sees the same input on both sides: its appended codes are checked against the oracle's
        # unrounded key and value (the plain layer of the oracle, same cache)
        for b in range(B):
            _, k_plain, v_plain = O.layer_forward(f64(x)[b][None, :], caches[b][0][0], caches[b][0][1], layers[0],
                                                  oracle_shape(sh))
            page, slot = int(batch.tables[b, ctx_lens[b] // 16]), int(ctx_lens[b] % 16)
            kc, vc = slot_codes(st, 0, page, slot)
            check_stored_token(kc, k_plain[-1], scales[0], ("k", b))
            check_stored_token(vc, v_plain[-1], scales[1], ("v", b))
        return float(np.max(errs))


@pytest.mark.parametrize("shape,scales", [("tiny", (1.0, 1.0)), ("tiny_gqa", (0.5, 2.0)), ("tiny_h128", (1.0, 1.0)),
                                          ("tiny_bias", (2.0, 0.25)), ("tiny_mqa", (1.0, 0.5)), ("tiny_g2", (0.5, 1.0))])
def test_decode_edge_contexts(tdp, shape, scales):
    """ctx = 0 (attention over the token itself), page edges, block edges (64 tokens), span edges (256)."""
    run_decode_case(tdp, shape, [0, 1, 15, 16, 31, 32, 63, 64, 65, 127, 255, 256, 257, 511, 512, 700], scales)


def test_decode_with_a_scale_that_is_not_a_power_of_two(tdp):
    run_decode_case(tdp, "tiny_h128", [40, 100, 17, 333], (0.7, 1.3))


@pytest.mark.parametrize("span", [256, 512, 1024, 2048, 4096])
def test_decode_every_span_length(tdp, span):
    ctx = sorted({31, span - 2, span - 1, span, span + 1, 2 * span - 1, 2 * span, 2 * span + 33,
                  min(3 * span + 7, 4096)} & set(range(0, 4097)))
    run_decode_case(tdp, "tiny_gqa", ctx, (1.0, 1.0), n_layers=1, max_pages_per_seq=4096 // 16 + 1, span=span)


def test_decode_70b_shaped_layer(tdp):
    """One 70B-shaped layer (64 query heads on 8 KV heads, head_dim 128), batch 24, contexts to 700."""
    ctx = np.minimum(W.decode_ctx_lens("70b_quarter", 24), 700)
    run_decode_case(tdp, "70b_quarter", ctx, (1.0, 1.0), n_layers=1)


def test_dropped_scales_would_be_caught(tdp):
    """The oracle run on the raw code values (scales forgotten) must be further from the GPU result
    than the tolerance, or the scale handling is not being tested."""
    sh = W.SHAPES["tiny_gqa"]
    scales = (0.25, 4.0)
    ctx = np.array([40, 90, 17], dtype=np.int64)
    batch = W.make_decode_batch(ctx)
    with Stage(tdp, sh, batch.num_pages, 3, 0, 0, batch.tables.shape[1], kv_scales=scales) as st:
        caches = import_kv(tdp, st, ctx, batch.tables, 5, scales)
        x = W.hidden_states(sh, 3, 5, device="cuda")
        out = torch.empty_like(x)
        tdp.tdp_stage_decode(st.h, x, i32(ctx), i32(batch.tables), 3, out)
        torch.cuda.synchronize()
        layers = list(oracle_layers(sh))
        good, _ = O.stage_decode(list(f64(x)), caches, layers, q8_shape(sh, scales))
        # a kernel that forgot the scales would attend to the raw code values: keys 4 times too large
        # (sharper softmax), values 4 times too small
        raw_caches = [[(k / scales[0], v / scales[1]) for k, v in c] for c in caches]
        wrong, _ = O.stage_decode(list(f64(x)), raw_caches, layers, q8_shape(sh, (1.0, 1.0)))
        assert np.all(row_errs(f64(out), np.stack(good)) <= TOL)
        assert np.max(row_errs(f64(out), np.stack(wrong))) > 3 * TOL


@pytest.mark.parametrize("shape", ["tiny", "tiny_gqa", "tiny_h128", "tiny_mqa", "tiny_g2"])
def test_prefill_writes_the_cache_and_decode_steps_read_it(tdp, shape):
    """Prefill stores the codes of its keys and values and attends to them; the decode steps that
    follow read the same cache."""
    sh = W.SHAPES[shape]
    scales = (1.0, 1.0)
    seq_lens = np.array([1, 15, 16, 17, 33, 70], dtype=np.int64)
    steps = 3
    n, T = len(seq_lens), int(seq_lens.sum())
    pb = W.make_prefill_batch(seq_lens + steps)
    cu = np.zeros(n + 1, dtype=np.int32)
    cu[1:] = np.cumsum(seq_lens)
    with Stage(tdp, sh, pb.num_pages, n, T, n, pb.tables.shape[1], kv_scales=scales) as st:
        st.poison()
        x = W.hidden_states(sh, T, 2, device="cuda")
        out = torch.empty_like(x)
        tab_d = i32(pb.tables)
        tdp.tdp_stage_prefill(st.h, x, i32(cu), tab_d, n, T, out)
        torch.cuda.synchronize()
        layers = list(oracle_layers(sh))
        osh = q8_shape(sh, scales)
        xs = f64(x)
        ref, caches = O.stage_prefill([xs[cu[s]:cu[s + 1]] for s in range(n)], layers, osh)
        pos = np.concatenate([np.arange(L) for L in seq_lens])
        errs = row_errs(f64(out), np.concatenate(ref))
        assert np.all(errs <= row_tolerances(pos)), errs
        for l in range(sh.n_layers):
            k_pool, v_pool = (t.cpu().numpy() for t in st.pools(l))
            mk, mv = np.zeros(k_pool.shape, bool), np.zeros(v_pool.shape, bool)
            for s in range(n):
                for p in range(int(seq_lens[s])):
                    mk[int(pb.tables[s, p // 16]), :, p % 16, :] = True
                    mv[int(pb.tables[s, p // 16]), :, :, p % 16] = True
            assert np.all(k_pool[~mk] == Stage.POISON_CODE) and np.all(v_pool[~mv] == Stage.POISON_CODE)
            kx, vx, _ = export_kv(tdp, st, seq_lens, pb.tables, l)
            for s in range(n):
                L = int(seq_lens[s])
                assert np.all(row_errs(kx[cu[s]:cu[s + 1]].reshape(L, -1), caches[s][l][0].reshape(L, -1)) <= TOL + STEP)
                assert np.all(row_errs(vx[cu[s]:cu[s + 1]].reshape(L, -1), caches[s][l][1].reshape(L, -1)) <= TOL + STEP)
        # layer 0 of the first prompts: stored codes against the oracle's unrounded keys / values
        _, k_plain, v_plain = O.layer_forward(xs[cu[4]:cu[5]], O.empty_cache(osh), O.empty_cache(osh), layers[0], oracle_shape(sh))
        for p in (0, 16, 32):
            kc, vc = slot_codes(st, 0, int(pb.tables[4, p // 16]), p % 16)
            check_stored_token(kc, k_plain[p], scales[0], ("k", p))
            check_stored_token(vc, v_plain[p], scales[1], ("v", p))
        ctx = seq_lens.copy()
        for step in range(steps):
            xd = W.hidden_states(sh, n, 100 + step, device="cuda")
            od = torch.empty_like(xd)
            tdp.tdp_stage_decode(st.h, xd, i32(ctx), tab_d, n, od)
            torch.cuda.synchronize()
            refd, caches = O.stage_decode(list(f64(xd)), caches, layers, osh)
            errs = row_errs(f64(od), np.stack(refd))
            assert np.all(errs <= row_tolerances(ctx)), (step, errs)
            ctx = ctx + 1


@pytest.mark.parametrize("shape,seq_lens,n_layers", [
    ("tiny", [600, 257], None), ("tiny", [4096], 1), ("tiny_g2", [300, 129], None), ("tiny_gqa", [200, 65], None),
    ("tiny_mqa", [100, 33], None), ("7b_quarter", [257, 600], 1),
])
def test_prefill_beyond_one_query_tile_with_an_8_bit_cache(tdp, shape, seq_lens, n_layers):
    """Prompts longer than one query tile of every prefill-attention variant, keys and values read back
    from pools of codes (later tiles start above position zero and skip the key blocks past their
    diagonal); one decode step follows on the cache the prefill wrote."""
    sh = W.SHAPES[shape]
    if n_layers:
        sh = sh.with_layers(n_layers)
    scales = (1.0, 0.5)
    seq_lens = np.asarray(seq_lens, dtype=np.int64)
    n, T = len(seq_lens), int(seq_lens.sum())
    pb = W.make_prefill_batch(seq_lens + 1)
    cu = np.zeros(n + 1, dtype=np.int32)
    cu[1:] = np.cumsum(seq_lens)
    with Stage(tdp, sh, pb.num_pages, n, T, n, pb.tables.shape[1], kv_scales=scales) as st:
        st.poison()
        x = W.hidden_states(sh, T, 2, device="cuda")
        out = torch.empty_like(x)
        tab_d = i32(pb.tables)
        tdp.tdp_stage_prefill(st.h, x, i32(cu), tab_d, n, T, out)
        torch.cuda.synchronize()
        layers = list(oracle_layers(sh))
        osh = q8_shape(sh, scales)
        xs = f64(x)
        ref, caches = O.stage_prefill([xs[cu[s]:cu[s + 1]] for s in range(n)], layers, osh)
        pos = np.concatenate([np.arange(L) for L in seq_lens])
        errs = row_errs(f64(out), np.concatenate(ref))
        if shape.startswith("tiny"):
            assert np.all(errs <= row_tolerances(pos)), float(np.max(errs))
        else:
            # At the real width the two sides' keys and values differ by the projection's bf16 error
            # before they are rounded to codes, so near a rounding boundary neighbouring codes are stored
            # (checked below: within one step); with scores as peaked as these weights give, a row that
            # puts most of its weight on such an entry moves by up to that step.  Every row is held to
            # tolerance + one step, and all but a few to the tolerance itself.
            assert np.all(errs <= TOL + STEP), float(np.max(errs))
            long_rows = pos >= SHORT_CTX
            assert np.mean(errs[long_rows] <= TOL) >= 0.98, float(np.mean(errs[long_rows] <= TOL))
        for l in range(sh.n_layers):
            kx, vx, _ = export_kv(tdp, st, seq_lens, pb.tables, l)
            for s in range(n):
                L = int(seq_lens[s])
                assert np.all(row_errs(kx[cu[s]:cu[s + 1]].reshape(L, -1), caches[s][l][0].reshape(L, -1)) <= TOL + STEP)
                assert np.all(row_errs(vx[cu[s]:cu[s + 1]].reshape(L, -1), caches[s][l][1].reshape(L, -1)) <= TOL + STEP)
        xd = W.hidden_states(sh, n, 100, device="cuda")
        od = torch.empty_like(xd)
        tdp.tdp_stage_decode(st.h, xd, i32(seq_lens), tab_d, n, od)
        torch.cuda.synchronize()
        refd, _ = O.stage_decode(list(f64(xd)), caches, layers, osh)
        assert np.all(row_errs(f64(od), np.stack(refd)) <= (TOL if shape.startswith("tiny") else TOL + STEP))


def test_decode_is_invariant_under_block_table_permutation(tdp):
    sh = W.SHAPES["tiny_gqa"]
    ctx = np.array([5, 40, 300, 77], dtype=np.int64)
    outs = []
    for seed in (1, 2):
        batch = W.make_decode_batch(ctx, seed=seed)
        with Stage(tdp, sh, batch.num_pages, 4, 0, 0, batch.tables.shape[1], kv_scales=(1.0, 1.0)) as st:
            st.poison()
            import_kv(tdp, st, ctx, batch.tables, 9, (1.0, 1.0))
            x = W.hidden_states(sh, 4, 9, device="cuda")
            out = torch.empty_like(x)
            tdp.tdp_stage_decode(st.h, x, i32(ctx), i32(batch.tables), 4, out)
            torch.cuda.synchronize()
            outs.append(out.view(torch.int16).cpu())
    assert torch.equal(outs[0], outs[1])


def test_zz_equal_code_fraction_over_the_run():
    """Over every stored token the tests above looked at, the stage and the oracle stored the same code for
    at least 93 % of the entries (expected from the projection's bf16 operand error: 94 to 96 %)."""
    import sys
    if not EQUAL_CODES:
        pytest.skip("no stored token was checked in this run")
    same, total = sum(a for a, _ in EQUAL_CODES), sum(b for _, b in EQUAL_CODES)
    print("equal codes, stage vs oracle: %.4f of %d entries in %d stored tokens" % (same / total, total, len(EQUAL_CODES)),
          file=sys.stderr, flush=True)
    assert same / total >= 0.93

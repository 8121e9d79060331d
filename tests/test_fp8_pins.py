"""Pins for oracle/fp8_oracle.py and the 8-bit cache option of oracle/stage_oracle.py.  No GPU.

The format is pinned against values worked out by hand from its definition (sign, 4 exponent
bits with bias 7, 3 mantissa bits, subnormals, no infinities, one NaN per sign, largest finite
value 448), against brute force over the table, and against torch's float8_e4m3fn, an independent
implementation of the same public format (inside the range where that one does not turn
overflow into NaN).  A slip in the bias, the subnormal scale, the tie rule, the saturation or the
sign handling fails at least one pin.
"""
import numpy as np
import torch

from oracle import fp8_oracle as F8
from oracle import stage_oracle as O

RNG = np.random.default_rng(77)
TABLE = F8.e4m3_decode_table()


def test_decode_table_by_hand():
    want = {0x00: 0.0, 0x01: 2.0 ** -9, 0x07: 7 * 2.0 ** -9, 0x08: 2.0 ** -6, 0x0F: 1.875 * 2.0 ** -6,
            0x30: 0.5, 0x38: 1.0, 0x39: 1.125, 0x3C: 1.5, 0x40: 2.0, 0x47: 3.75, 0x77: 240.0, 0x78: 256.0,
            0x7E: 448.0, 0xB8: -1.0, 0xFE: -448.0, 0x81: -(2.0 ** -9)}
    for c, v in want.items():
        assert TABLE[c] == v, hex(c)
    assert np.isnan(TABLE[0x7F]) and np.isnan(TABLE[0xFF])
    assert TABLE[0x80] == 0.0 and np.signbit(TABLE[0x80])
    assert np.isfinite(TABLE).sum() == 254
    assert np.all(np.diff(TABLE[:0x7F]) > 0)                       # strictly increasing in the code
    assert np.array_equal(TABLE[0x80:0xFF], -TABLE[0x00:0x7F])


def test_decode_table_matches_library_format():
    lib = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(np.isnan(lib), np.isnan(TABLE))
    ok = ~np.isnan(TABLE)
    assert np.array_equal(lib[ok], TABLE[ok]) and np.array_equal(np.signbit(lib[ok]), np.signbit(TABLE[ok]))


def test_encode_inverts_decode_on_every_finite_code():
    codes = np.array([c for c in range(256) if c not in (0x7F, 0xFF)], np.uint8)
    assert np.array_equal(F8.e4m3_encode(TABLE[codes]), codes)


def brute_force_encode(x):
    """argmin |x - value| over the finite codes of x's sign, ties to the even code, written as loops."""
    out = np.empty(len(x), np.uint8)
    for i, v in enumerate(x):
        best, best_d = 0, None
        for c in range(0x7F):
            d = abs(abs(v) - TABLE[c])
            if best_d is None or d < best_d or (d == best_d and c % 2 == 0):
                best, best_d = c, d
        out[i] = best | (0x80 if np.signbit(v) else 0)
    return out


def test_encode_against_brute_force_and_ties():
    mids = (TABLE[:0x7E] + TABLE[1:0x7F]) / 2
    x = np.concatenate([RNG.normal(0, 1, 400), RNG.normal(0, 100, 400), RNG.uniform(-2.0 ** -5, 2.0 ** -5, 400),
                        mids, -mids, np.nextafter(mids, np.inf), np.nextafter(mids, -np.inf), [0.0, -0.0]])
    x = x[np.abs(x) <= 448.0]
    assert np.array_equal(F8.e4m3_encode(x), brute_force_encode(x))
    # a tie goes to the even code: between 1.0 (0x38) and 1.125 (0x39) -> 0x38; between 1.125 and 1.25 (0x3a) -> 0x3a
    assert list(F8.e4m3_encode(np.array([1.0625, 1.1875, 2.0 ** -10, 3 * 2.0 ** -10]))) == [0x38, 0x3A, 0x00, 0x02]


def test_encode_matches_library_inside_its_range():
    x = np.concatenate([RNG.normal(0, 1, 20000), RNG.normal(0, 60, 20000), RNG.uniform(-0.03, 0.03, 20000)])
    x = x[np.abs(x) < 460].astype(np.float32)
    lib = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(F8.e4m3_encode(x.astype(np.float64)), lib)


def test_encode_saturates_and_keeps_nan():
    x = np.array([448.0, 463.9, 464.0, 470.0, 1e30, np.inf, -464.0, -1e30, -np.inf, np.nan])
    assert list(F8.e4m3_encode(x)[:9]) == [0x7E] * 6 + [0xFE] * 3
    assert F8.e4m3_encode(x)[9] & 0x7F == 0x7F


def test_encode_is_monotone_and_within_half_a_step():
    x = np.sort(np.concatenate([RNG.normal(0, 3, 5000), RNG.uniform(-500, 500, 5000)]))
    v = F8.e4m3_decode(F8.e4m3_encode(x))
    assert np.all(np.diff(v) >= 0)
    normal = (np.abs(x) >= 2.0 ** -6) & (np.abs(x) <= 448)
    assert np.all(np.abs(v - x)[normal] <= np.abs(x)[normal] / 16)            # half of a 2^-3 relative step
    assert np.all(np.abs(v - x)[np.abs(x) < 2.0 ** -6] <= 2.0 ** -10)           # half a subnormal step


def test_cache_scale_and_division_precision():
    x = RNG.normal(0, 2, 4096)
    for s in (0.25, 1.0, 8.0):                                                    # powers of two commute exactly
        assert np.array_equal(F8.kv_roundtrip(x, s), s * F8.kv_roundtrip(x.astype(np.float32) / np.float32(s), 1.0))
    # the quotient is formed in the stated precision: a value a hair above a tie in float64 lands on the tie in float32
    x = np.array([1.0625 * 3.0 * (1 + 2.0 ** -40)])
    assert F8.kv_quantize(x, 3.0, np.float64)[0] == 0x39 and F8.kv_quantize(x, 3.0, np.float32)[0] == 0x38
    # range: 448 * scale is the largest magnitude the cache can hold
    assert F8.kv_roundtrip(np.array([1e4, -1e4]), 2.0).tolist() == [896.0, -896.0]


# ---------------------------------------------------------------- the cache option of the stage oracle

SH = O.Shape(4, 2, 8)


def rand_layer(d, sh, f, rng):
    m = lambda a, b: rng.normal(0, 0.25, (a, b))
    return O.LayerWeights(m(d, sh.n_q_heads * sh.head_dim), m(d, sh.n_kv_heads * sh.head_dim),
                          m(d, sh.n_kv_heads * sh.head_dim), m(sh.n_q_heads * sh.head_dim, d), m(d, f), m(d, f),
                          m(f, d), 1 + rng.normal(0, 0.1, d), 1 + rng.normal(0, 0.1, d))


def by_hand_layer(x, k_all, v_all, p0, w, sh):
    """The layer recomposed from the oracle's primitives with the attention inputs given."""
    L = x.shape[0]
    y = O.rmsnorm(x, w.g_attn, sh.rms_eps)
    q = O.rope((y @ w.wq).reshape(L, sh.n_q_heads, sh.head_dim), np.arange(p0, p0 + L), sh.rope_base)
    h = x + O.attention(q, k_all, v_all, p0, sh) @ w.wo
    y2 = O.rmsnorm(h, w.g_mlp, sh.rms_eps)
    return h + (O.silu(y2 @ w.wg) * (y2 @ w.wu)) @ w.wd


def test_cache_holds_representable_values_and_attention_reads_the_cache():
    rng = np.random.default_rng(5)
    w = rand_layer(16, SH, 24, rng)
    x = rng.normal(size=(7, 16))
    q8 = O.Shape(4, 2, 8, kv_scales=(0.5, 2.0))
    out_plain, k_plain, v_plain = O.layer_forward(x, O.empty_cache(SH), O.empty_cache(SH), w, SH)
    out_q8, k8, v8 = O.layer_forward(x, O.empty_cache(SH), O.empty_cache(SH), w, q8)
    assert np.array_equal(k8, F8.kv_roundtrip(k_plain, 0.5)) and np.array_equal(v8, F8.kv_roundtrip(v_plain, 2.0))
    assert not np.array_equal(k8, k_plain)
    grid = set((F8.e4m3_decode_table()[:0x7F] * 0.5).tolist())
    assert all(abs(v) in grid for v in k8.ravel())
    # prefill attends to the stored keys and values, not to the ones it computed
    assert np.allclose(out_q8, by_hand_layer(x, k8, v8, 0, w, SH), atol=1e-12)
    assert np.max(np.abs(out_q8 - out_plain)) > 1e-6


def test_decode_step_attends_to_the_stored_token_and_stored_context():
    rng = np.random.default_rng(6)
    w = rand_layer(16, SH, 24, rng)
    q8 = O.Shape(4, 2, 8, kv_scales=(1.0, 1.0))
    kc, vc = rng.normal(size=(5, 2, 8)), rng.normal(size=(5, 2, 8))
    kc8, vc8 = F8.kv_roundtrip(kc, 1.0), F8.kv_roundtrip(vc, 1.0)
    x = rng.normal(size=(1, 16))
    out, k_all, v_all = O.layer_forward(x, kc8, vc8, w, q8)
    out_plain, k_plain, v_plain = O.layer_forward(x, kc8, vc8, w, SH)
    assert np.array_equal(k_all[:5], kc8) and np.array_equal(k_all[5:], F8.kv_roundtrip(k_plain[5:], 1.0))
    assert np.array_equal(v_all[5:], F8.kv_roundtrip(v_plain[5:], 1.0))
    assert np.allclose(out, by_hand_layer(x, k_all, v_all, 5, w, SH), atol=1e-12)
    # and it differs from attending to the unrounded new token
    assert np.max(np.abs(out_plain - out)) > 1e-6


def test_representable_cache_makes_the_option_a_no_op():
    """If every key and value already is an E4M3 number, an 8-bit cache changes nothing."""
    rng = np.random.default_rng(8)
    sh = O.Shape(2, 1, 4)
    d = 4
    eye = np.eye(d)
    # projections that copy the (normalised) input: with inputs of equal magnitude the norm output is +-1
    w = O.LayerWeights(np.tile(eye, (1, 2)), eye, eye, rng.normal(size=(8, d)), rng.normal(size=(d, 6)),
                       rng.normal(size=(d, 6)), rng.normal(size=(6, d)), np.ones(d), np.ones(d))
    x = rng.choice([-1.0, 1.0], size=(1, d)) * 3.0
    shq = O.Shape(2, 1, 4, rms_eps=0.0, kv_scales=(1.0, 1.0))
    shp = O.Shape(2, 1, 4, rms_eps=0.0)
    # position 0: the rotation is the identity, so k = v = +-1 exactly
    a, ka, va = O.layer_forward(x, O.empty_cache(sh), O.empty_cache(sh), w, shq)
    b, kb, vb = O.layer_forward(x, O.empty_cache(sh), O.empty_cache(sh), w, shp)
    assert np.array_equal(ka, kb) and np.array_equal(va, vb) and np.array_equal(a, b)


def test_stage_prefill_and_decode_carry_the_stored_cache():
    rng = np.random.default_rng(9)
    layers = [rand_layer(16, SH, 24, rng) for _ in range(2)]
    q8 = O.Shape(4, 2, 8, kv_scales=(1.0, 1.0))
    prompts = [rng.normal(size=(6, 16)), rng.normal(size=(3, 16))]
    outs8, caches8 = O.stage_prefill(prompts, layers, q8)
    outs, caches = O.stage_prefill(prompts, layers, SH)
    # layer 0 sees the same input either way: its cache is the plain one through the format
    assert np.array_equal(caches8[0][0][0], F8.kv_roundtrip(caches[0][0][0], 1.0))
    assert np.max(np.abs(outs8[0] - outs[0])) > 1e-6
    xs = [rng.normal(size=16), rng.normal(size=16)]
    step8, new8 = O.stage_decode(xs, caches8, layers, q8)
    want0, _ = O.stage_forward(xs[0][None, :], caches8[0], layers, q8)
    assert np.array_equal(step8[0], want0[0])
    assert new8[1][0][0].shape[0] == 4
    grid = set(F8.e4m3_decode_table()[:0x7F].tolist())
    assert all(abs(v) in grid for v in new8[1][1][1].ravel())


def test_stored_cache_is_the_reading_under_which_decode_equals_full_recompute():
    """Which values prefill attends to when the cache is held in 8 bits is fixed by an invariant of the
    method itself, not by how a kernel happens to read: decoding one token on a cache must give what
    recomputing the whole sequence gives at its last position (prefill(L) = prefill(L-1) + decode, the
    KV cache being only a memo of the prefill's keys and values, Sec. 2.1).  A decode step can only see
    what the cache holds, i.e. the rounded keys and values; so the recompute must see them too.  With
    the cache as the one source the invariant holds exactly, also token by token; if prefill attended to
    the unrounded keys and values instead, it would break."""
    rng = np.random.default_rng(12)
    layers = [rand_layer(16, SH, 24, rng) for _ in range(3)]
    q8 = O.Shape(4, 2, 8, kv_scales=(0.5, 2.0))
    x = rng.normal(size=(7, 16))
    full, caches_full = O.stage_forward(x, None, layers, q8)
    part, caches = O.stage_forward(x[:6], None, layers, q8)
    last, caches2 = O.stage_forward(x[6:7], caches, layers, q8)
    assert np.allclose(part, full[:6], atol=1e-12) and np.allclose(last[0], full[6], atol=1e-12)
    for (ka, va), (kb, vb) in zip(caches_full, caches2):
        assert np.array_equal(ka[:6], kb[:6]) and np.allclose(ka, kb, atol=1e-12) and np.allclose(va, vb, atol=1e-12)
    # one prefill token followed by single-token decode steps
    out, c = O.stage_forward(x[:1], None, layers, q8)
    rows = [out[0]]
    for t in range(1, 7):
        outs, cs = O.stage_decode([x[t]], [c], layers, q8)
        rows.append(outs[0])
        c = cs[0]
    assert np.allclose(np.stack(rows), full, atol=1e-11)
    # the other reading - prefill attends to the keys and values as computed and only stores the codes -
    # recomposed from the oracle's primitives for one layer: its last row is NOT what decode gives
    w = layers[0]
    _, k_plain, v_plain = O.layer_forward(x, O.empty_cache(SH), O.empty_cache(SH), w, SH)
    as_computed = by_hand_layer(x, k_plain, v_plain, 0, w, SH)
    _, k6, v6 = O.layer_forward(x[:6], O.empty_cache(SH), O.empty_cache(SH), w, q8)
    dec, _, _ = O.layer_forward(x[6:7], k6, v6, w, q8)
    assert np.max(np.abs(as_computed[6] - dec[0])) > 1e-4
    stored, _, _ = O.layer_forward(x, O.empty_cache(SH), O.empty_cache(SH), w, q8)
    assert np.allclose(stored[6], dec[0], atol=1e-12)

"""Pins for the fp64 oracle: closed forms, invariants, brute force and an
independently composed library formulation.  No GPU, no HIP path.

Each pin is chosen so that a plausible slip in oracle/stage_oracle.py (a
dropped gain or eps, a wrong sign or pairing in the rotation, an off-by-one in
the causal span, a missing 1/sqrt(d_h), a wrong K/V head for a query head, a
missing residual) fails at least one of them.
"""
import math

import numpy as np
import pytest
import torch

from oracle import stage_oracle as O

RNG = np.random.default_rng(1234)


def rand_layer(d, hq, hkv, dh, f, scale=0.2, rng=RNG):
    def m(a, b):
        return rng.normal(0, scale, (a, b))
    return O.LayerWeights(m(d, hq * dh), m(d, hkv * dh), m(d, hkv * dh), m(hq * dh, d),
                          m(d, f), m(d, f), m(f, d),
                          1 + rng.normal(0, 0.1, d), 1 + rng.normal(0, 0.1, d))


SH = O.Shape(4, 2, 8)
D, F = 16, 24


# ---------------------------------------------------------------- RMSNorm

def test_rmsnorm_unit_mean_square_and_scale_invariance():
    x = RNG.normal(0, 3, (5, 32))
    y = O.rmsnorm(x, np.ones(32), 0.0)
    assert np.allclose(np.mean(y * y, -1), 1.0, atol=1e-12)
    assert np.allclose(O.rmsnorm(7.5 * x, np.ones(32), 0.0), y, atol=1e-12)


def test_rmsnorm_gain_and_eps_by_hand():
    x = np.array([[3.0, 4.0]])
    g = np.array([2.0, -1.0])
    # mean square = 12.5; eps = 3.5 -> denominator sqrt(16) = 4
    assert np.allclose(O.rmsnorm(x, g, 3.5), [[1.5, -1.0]], atol=1e-15)


# ---------------------------------------------------------------- RoPE

def test_rope_identity_at_zero_and_norm_preserving():
    z = RNG.normal(size=(3, 2, 8))
    assert np.array_equal(O.rope(z, np.zeros(3), 10000.0), z)
    r = O.rope(z, np.array([5, 17, 1023]), 10000.0)
    assert np.allclose(np.linalg.norm(r, axis=-1), np.linalg.norm(z, axis=-1), atol=1e-12)


def test_rope_by_hand_pairing_sign_and_frequency():
    # dh = 4: pair 0 = (z0, z2) turns by p*1, pair 1 = (z1, z3) by p*base^(-1/2)
    z = np.array([[[1.0, 2.0, 3.0, 4.0]]])
    p, base = 3.0, 100.0
    t0, t1 = p * 1.0, p * base ** -0.5
    want = [1 * math.cos(t0) - 3 * math.sin(t0), 2 * math.cos(t1) - 4 * math.sin(t1),
            1 * math.sin(t0) + 3 * math.cos(t0), 2 * math.sin(t1) + 4 * math.cos(t1)]
    assert np.allclose(O.rope(z, np.array([p]), base)[0, 0], want, atol=1e-14)


def test_rope_inner_product_depends_on_offset_only():
    q = RNG.normal(size=(1, 1, 16))
    k = RNG.normal(size=(1, 1, 16))
    def ip(pq, pk):
        return float(np.sum(O.rope(q, np.array([pq]), 1e4) * O.rope(k, np.array([pk]), 1e4)))
    assert abs(ip(10, 3) - ip(110, 103)) < 1e-10
    assert abs(ip(10, 3) - ip(10, 4)) > 1e-6


def test_rope_matches_complex_rotation():
    """Independent formulation: each pair is a complex number times e^{i p theta}."""
    L, H, dh = 6, 3, 16
    z = RNG.normal(size=(L, H, dh))
    pos = np.array([0, 1, 2, 40, 999, 4095])
    zc = z[..., : dh // 2] + 1j * z[..., dh // 2:]
    theta = 10000.0 ** (-np.arange(0, dh, 2) / dh)
    rot = zc * np.exp(1j * pos[:, None, None] * theta[None, None, :])
    want = np.concatenate([rot.real, rot.imag], -1)
    assert np.allclose(O.rope(z, pos, 10000.0), want, atol=1e-12)


# ---------------------------------------------------------------- softmax / attention

def test_softmax_rows_sum_to_one_and_nonnegative():
    for n in (1, 2, 17, 300):
        q = RNG.normal(size=8) * 5
        k = RNG.normal(size=(n, 8)) * 5
        w = O.attention_weights(q, k, n)
        assert w.shape == (n,)
        assert np.all(w >= 0)
        assert abs(w.sum() - 1.0) < 1e-12


def test_softmax_stable_for_large_scores():
    w = O.softmax(np.array([1000.0, 1000.0, -1000.0]))
    assert np.allclose(w, [0.5, 0.5, 0.0])


def brute_attention(q, k, v, p0, hq, hkv):
    """Explicit score matrix, explicit mask, naive exp / sum, Python loops."""
    L, _, dh = q.shape
    n = k.shape[0]
    G = hq // hkv
    out = np.zeros((L, hq, dh))
    for h in range(hq):
        S = np.zeros((L, n))
        for i in range(L):
            for j in range(n):
                S[i, j] = sum(q[i, h, c] * k[j, h // G, c] for c in range(dh)) / math.sqrt(dh)
        for i in range(L):
            e = [math.exp(S[i, j]) if j <= p0 + i else 0.0 for j in range(n)]
            tot = sum(e)
            for c in range(dh):
                out[i, h, c] = sum(e[j] * v[j, h // G, c] for j in range(n)) / tot
    return out.reshape(L, hq * dh)


@pytest.mark.parametrize("L,p0,hq,hkv,dh", [(1, 0, 2, 2, 4), (5, 0, 4, 2, 4), (3, 4, 4, 1, 6), (1, 9, 6, 3, 4)])
def test_attention_matches_brute_force(L, p0, hq, hkv, dh):
    sh = O.Shape(hq, hkv, dh)
    q = RNG.normal(size=(L, hq, dh))
    k = RNG.normal(size=(p0 + L, hkv, dh))
    v = RNG.normal(size=(p0 + L, hkv, dh))
    assert np.allclose(O.attention(q, k, v, p0, sh), brute_attention(q, k, v, p0, hq, hkv), atol=1e-12)


def test_attention_closed_forms():
    sh = O.Shape(2, 1, 4)
    q = RNG.normal(size=(1, 2, 4))
    k = RNG.normal(size=(7, 1, 4))
    # (i) all values equal -> output is that value whatever the scores
    v = np.tile(RNG.normal(size=(1, 1, 4)), (7, 1, 1))
    assert np.allclose(O.attention(q, k, v, 6, sh).reshape(2, 4), v[0, 0][None], atol=1e-13)
    # (ii) single visible token -> output is its value
    v1 = RNG.normal(size=(1, 1, 4))
    assert np.allclose(O.attention(q, k[:1], v1, 0, sh).reshape(2, 4), v1[0, 0][None], atol=1e-13)
    # (iii) zero query -> plain mean of the visible values
    v = RNG.normal(size=(7, 1, 4))
    assert np.allclose(O.attention(np.zeros((1, 2, 4)), k, v, 6, sh).reshape(2, 4), v[:, 0].mean(0)[None], atol=1e-13)


def test_attention_scale_is_inverse_sqrt_head_dim():
    # two keys, scores differ by dh/sqrt(dh)=sqrt(dh): weight ratio must be e^{sqrt(dh)}
    dh = 16
    q = np.ones(dh)
    k = np.stack([np.ones(dh), np.zeros(dh)])
    w = O.attention_weights(q, k, 2)
    assert abs(w[0] / w[1] - math.exp(math.sqrt(dh))) < 1e-9


def test_causality_future_tokens_do_not_matter():
    w = rand_layer(D, 4, 2, 8, F)
    x = RNG.normal(size=(9, D))
    y0, _, _ = O.layer_forward(x, O.empty_cache(SH), O.empty_cache(SH), w, SH)
    x2 = x.copy()
    x2[6:] += RNG.normal(size=(3, D))
    y1, _, _ = O.layer_forward(x2, O.empty_cache(SH), O.empty_cache(SH), w, SH)
    assert np.array_equal(y0[:6], y1[:6])
    assert not np.allclose(y0[6:], y1[6:])


def test_attention_sees_exactly_positions_up_to_and_including_self():
    """Row i must change when token i's own key changes and when token i-1's does."""
    sh = O.Shape(1, 1, 4)
    q = RNG.normal(size=(3, 1, 4))
    k = RNG.normal(size=(5, 1, 4))
    v = RNG.normal(size=(5, 1, 4))
    base = O.attention(q, k, v, 2, sh)
    for j in range(5):
        v2 = v.copy()
        v2[j] += 1.0
        changed = ~np.isclose(O.attention(q, k, v2, 2, sh), base).all(axis=1)
        assert list(changed) == [j <= 2 + i for i in range(3)]


# ---------------------------------------------------------------- layer / stage

def test_prefill_equals_prefill_minus_one_then_decode_and_all_decodes():
    layers = [rand_layer(D, 4, 2, 8, F) for _ in range(3)]
    x = RNG.normal(size=(7, D))
    full, caches_full = O.stage_forward(x, None, layers, SH)
    part, caches = O.stage_forward(x[:6], None, layers, SH)
    last, caches2 = O.stage_forward(x[6:7], caches, layers, SH)
    assert np.allclose(part, full[:6], atol=1e-12)
    assert np.allclose(last[0], full[6], atol=1e-12)
    for (ka, va), (kb, vb) in zip(caches_full, caches2):
        assert np.allclose(ka, kb, atol=1e-12) and np.allclose(va, vb, atol=1e-12)
    # one prefill token followed by L-1 single-token decode steps
    out, c = O.stage_forward(x[:1], None, layers, SH)
    rows = [out[0]]
    for t in range(1, 7):
        outs, cs = O.stage_decode([x[t]], [c], layers, SH)
        rows.append(outs[0])
        c = cs[0]
    assert np.allclose(np.stack(rows), full, atol=1e-11)


def test_cache_holds_rotated_keys_and_plain_values():
    w = rand_layer(D, 4, 2, 8, F)
    x = RNG.normal(size=(4, D))
    _, k_all, v_all = O.layer_forward(x, O.empty_cache(SH), O.empty_cache(SH), w, SH)
    y = O.rmsnorm(x, w.g_attn, SH.rms_eps)
    assert np.allclose(v_all, (y @ w.wv).reshape(4, 2, 8), atol=1e-13)
    k_plain = (y @ w.wk).reshape(4, 2, 8)
    assert np.allclose(k_all[0], k_plain[0], atol=1e-13)       # position 0: no rotation
    assert not np.allclose(k_all[1:], k_plain[1:])
    assert np.allclose(np.linalg.norm(k_all, axis=-1), np.linalg.norm(k_plain, axis=-1), atol=1e-12)


def test_zero_output_projections_make_stage_identity():
    w = rand_layer(D, 4, 2, 8, F)
    w.wo[:] = 0
    w.wd[:] = 0
    x = RNG.normal(size=(5, D))
    out, _ = O.stage_forward(x, None, [w, w], SH)
    assert np.array_equal(out, x)


def test_residual_structure():
    """With W_d = 0 the layer returns x + attn W_o; with W_o = 0 it returns x + mlp(x)."""
    w = rand_layer(D, 4, 2, 8, F)
    x = RNG.normal(size=(3, D))
    w1 = O.LayerWeights(**{**w.__dict__, "wd": np.zeros_like(w.wd)})
    out1, k_all, v_all = O.layer_forward(x, O.empty_cache(SH), O.empty_cache(SH), w1, SH)
    y = O.rmsnorm(x, w.g_attn, SH.rms_eps)
    q = O.rope((y @ w.wq).reshape(3, 4, 8), np.arange(3), SH.rope_base)
    a = brute_attention(q, k_all, v_all, 0, 4, 2)
    assert np.allclose(out1, x + a @ w.wo, atol=1e-12)
    w2 = O.LayerWeights(**{**w.__dict__, "wo": np.zeros_like(w.wo)})
    out2, _, _ = O.layer_forward(x, O.empty_cache(SH), O.empty_cache(SH), w2, SH)
    y2 = O.rmsnorm(x, w.g_mlp, SH.rms_eps)
    g = y2 @ w.wg
    mlp = (g / (1 + np.exp(-g)) * (y2 @ w.wu)) @ w.wd
    assert np.allclose(out2, x + mlp, atol=1e-12)


def test_silu_values():
    assert O.silu(np.array([0.0]))[0] == 0.0
    assert abs(O.silu(np.array([40.0]))[0] - 40.0) < 1e-12
    assert abs(O.silu(np.array([1.0]))[0] - 1.0 / (1.0 + math.exp(-1.0))) < 1e-15
    assert abs(O.silu(np.array([-1.0]))[0] + 1.0 / (1.0 + math.exp(1.0))) < 1e-15


def test_gqa_equals_mha_with_repeated_kv_heads():
    hq, hkv, dh = 4, 2, 8
    w = rand_layer(D, hq, hkv, dh, F)
    G = hq // hkv
    def rep(m):
        return np.repeat(m.reshape(D, hkv, dh), G, axis=1).reshape(D, hq * dh)
    w_mha = O.LayerWeights(**{**w.__dict__, "wk": rep(w.wk), "wv": rep(w.wv)})
    x = RNG.normal(size=(6, D))
    a, _ = O.stage_forward(x, None, [w], O.Shape(hq, hkv, dh))
    b, _ = O.stage_forward(x, None, [w_mha], O.Shape(hq, hq, dh))
    assert np.allclose(a, b, atol=1e-12)


def test_requests_are_independent_and_batch_order_is_free():
    layers = [rand_layer(D, 4, 2, 8, F) for _ in range(2)]
    prompts = [RNG.normal(size=(n, D)) for n in (3, 7, 5)]
    outs, caches = O.stage_prefill(prompts, layers, SH)
    outs_r, _ = O.stage_prefill(prompts[::-1], layers, SH)
    for a, b in zip(outs, outs_r[::-1]):
        assert np.array_equal(a, b)
    solo, _ = O.stage_prefill([prompts[1]], layers, SH)
    assert np.array_equal(solo[0], outs[1])
    xs = [RNG.normal(size=D) for _ in range(3)]
    d_all, _ = O.stage_decode(xs, caches, layers, SH)
    d_one, _ = O.stage_decode([xs[2]], [caches[2]], layers, SH)
    assert np.array_equal(d_all[2], d_one[0])


def test_decode_with_empty_cache_attends_to_itself_only():
    """ctx = 0: the attention output is the token's own value vector."""
    w = rand_layer(D, 4, 2, 8, F)
    w.wd[:] = 0
    x = RNG.normal(size=(1, D))
    out, _, v_all = O.layer_forward(x, O.empty_cache(SH), O.empty_cache(SH), w, SH)
    a = np.repeat(v_all[0], 2, axis=0).reshape(1, 32)      # query head h reads kv head h // 2
    assert np.allclose(out, x + a @ w.wo, atol=1e-12)


def test_layer_matches_library_composition_in_torch_fp64():
    """The same layer composed independently from torch fp64 library routines
    (scaled_dot_product_attention with a causal mask, complex-number rotation)."""
    hq, hkv, dh, d, f = 6, 2, 16, 32, 40
    sh = O.Shape(hq, hkv, dh)
    w = rand_layer(d, hq, hkv, dh, f)
    L = 11
    x = RNG.normal(size=(L, d))
    got, k_all, v_all = O.layer_forward(x, O.empty_cache(sh), O.empty_cache(sh), w, sh)

    T = lambda a: torch.tensor(a, dtype=torch.float64)
    xt = T(x)
    def rms(t, g):
        return t * torch.rsqrt(t.pow(2).mean(-1, keepdim=True) + sh.rms_eps) * T(g)
    def rot(t):                                   # [L, H, dh]
        tc = torch.complex(t[..., : dh // 2], t[..., dh // 2:])
        inv = 1.0 / (sh.rope_base ** (torch.arange(0, dh, 2, dtype=torch.float64) / dh))
        ang = torch.outer(torch.arange(L, dtype=torch.float64), inv)
        r = tc * torch.polar(torch.ones_like(ang), ang)[:, None, :]
        return torch.cat([r.real, r.imag], -1)
    y = rms(xt, w.g_attn)
    q = rot((y @ T(w.wq)).view(L, hq, dh)).transpose(0, 1)
    k = rot((y @ T(w.wk)).view(L, hkv, dh)).transpose(0, 1).repeat_interleave(hq // hkv, 0)
    v = (y @ T(w.wv)).view(L, hkv, dh).transpose(0, 1).repeat_interleave(hq // hkv, 0)
    a = torch.nn.functional.scaled_dot_product_attention(q[None], k[None], v[None], is_causal=True)[0]
    h = xt + a.transpose(0, 1).reshape(L, hq * dh) @ T(w.wo)
    y2 = rms(h, w.g_mlp)
    want = h + (torch.nn.functional.silu(y2 @ T(w.wg)) * (y2 @ T(w.wu))) @ T(w.wd)
    assert np.allclose(got, want.numpy(), atol=1e-11)


# ---------------------------------------------------------------- pipeline ends

def test_embedding_lookup_equals_one_hot_product():
    from oracle import ends_oracle as E
    rng = np.random.default_rng(31)
    table = rng.standard_normal((50, 16))
    ids = rng.integers(0, 50, size=23)
    one_hot = np.zeros((23, 50))
    one_hot[np.arange(23), ids] = 1.0
    assert np.array_equal(E.embed(ids, table), one_hot @ table)
    with pytest.raises(IndexError):
        E.embed([50], table)
    with pytest.raises(IndexError):
        E.embed([-1], table)


def test_greedy_takes_the_lowest_index_among_the_maxima():
    from oracle import ends_oracle as E
    assert list(E.greedy_tokens(np.array([[1.0, 3.0, 3.0, 2.0], [5.0, 5.0, 5.0, 5.0], [0.0, -1.0, 2.0, 2.0]]))) == [1, 0, 2]
    rng = np.random.default_rng(32)
    logits = rng.integers(0, 6, size=(40, 97)).astype(np.float64)      # many ties
    assert np.array_equal(E.greedy_tokens(logits), np.argmax(logits, axis=1))
    assert list(E.greedy_tokens(np.array([[-np.inf, -3.0, -np.inf]]))) == [1]


def test_final_logits_closed_forms():
    from oracle import ends_oracle as E
    rng = np.random.default_rng(33)
    x = rng.standard_normal((7, 12))
    ones = np.ones(12)
    # identity head, unit gain, eps -> 0: logits are x scaled to unit mean square, so the argmax is x's
    lg = E.final_logits(x, ones, np.eye(12), 0.0)
    assert np.allclose(np.mean(lg ** 2, axis=1), 1.0)
    assert np.array_equal(E.greedy_tokens(lg), np.argmax(x, axis=1))
    # the norm removes positive scale
    w = rng.standard_normal((12, 30))
    g = 1.0 + 0.1 * rng.standard_normal(12)
    assert np.allclose(E.final_logits(3.7 * x, g, w, 0.0), E.final_logits(x, g, w, 0.0))
    # the gain acts per input channel: folding it into the head's rows gives the same logits
    assert np.allclose(E.final_logits(x, g, w, 1e-5), E.final_logits(x, ones, g[:, None] * w, 1e-5))
    # a dropped norm would fail this: logits of a huge input stay bounded
    assert np.max(np.abs(E.final_logits(1e6 * x, ones, w, 1e-5))) < 1e3


# ---------------------------------------------------------------- q / k / v biases (Qwen-style layer)

def _with_bias(w, bq, bk, bv):
    import dataclasses
    return dataclasses.replace(w, bq=bq, bk=bk, bv=bv)


def test_zero_bias_is_no_bias():
    w = rand_layer(D, 4, 2, 8, F)
    x = RNG.normal(size=(5, D))
    e = O.empty_cache(SH)
    a = O.layer_forward(x, e, e, w, SH)
    b = O.layer_forward(x, e, e, _with_bias(w, np.zeros(32), np.zeros(16), np.zeros(16)), SH)
    for u, v in zip(a, b):
        assert np.array_equal(u, v)


def test_bias_equals_an_extra_weight_row_fed_by_a_constant_channel():
    """q = y W + b is the product of [y, c] with [[W], [b / c]]: build a layer of width D+1 whose
    last normalised channel is a known constant and whose extra weight rows carry the biases."""
    rng = np.random.default_rng(41)
    w = rand_layer(D, 4, 2, 8, F, rng=rng)
    bq, bk, bv = rng.normal(size=32), rng.normal(size=16), rng.normal(size=16)
    x = rng.normal(size=(6, D))
    e = O.empty_cache(SH)
    want = O.layer_forward(x, e, e, _with_bias(w, bq, bk, bv), SH)
    # reference composed by hand from the oracle's own building blocks, bias as an augmented product
    y = O.rmsnorm(x, w.g_attn, SH.rms_eps)
    ya = np.concatenate([y, np.ones((6, 1))], axis=1)
    q = (ya @ np.vstack([w.wq, bq])).reshape(6, 4, 8)
    k = (ya @ np.vstack([w.wk, bk])).reshape(6, 2, 8)
    v = (ya @ np.vstack([w.wv, bv])).reshape(6, 2, 8)
    pos = np.arange(6)
    q, k = O.rope(q, pos, SH.rope_base), O.rope(k, pos, SH.rope_base)
    a = O.attention(q, k, v, 0, SH)
    h = x + a @ w.wo
    y2 = O.rmsnorm(h, w.g_mlp, SH.rms_eps)
    out = h + (O.silu(y2 @ w.wg) * (y2 @ w.wu)) @ w.wd
    assert np.allclose(want[0], out, rtol=1e-12, atol=1e-12)
    assert np.allclose(want[1], k) and np.allclose(want[2], v)


def test_value_bias_shifts_the_attention_output_by_itself():
    """Softmax weights sum to 1, so adding b_v to every value adds b_v (per head) to the attention
    output and b_v-through-W_o to the residual branch - whatever q and k are."""
    rng = np.random.default_rng(42)
    w = rand_layer(D, 4, 2, 8, F, rng=rng)
    # kill the MLP branch so the layer output is x + attn @ wo
    w.wd[:] = 0.0
    bv = rng.normal(size=16)
    x = rng.normal(size=(5, D))
    e = O.empty_cache(SH)
    plain = O.layer_forward(x, e, e, w, SH)[0]
    shifted = O.layer_forward(x, e, e, _with_bias(w, None, None, bv), SH)[0]
    per_q_head = np.repeat(bv.reshape(2, 8), 2, axis=0).reshape(-1)      # kv head h serves q heads 2h, 2h+1
    assert np.allclose(shifted - plain, np.tile(per_q_head @ w.wo, (5, 1)), atol=1e-12)


def test_key_bias_is_rotated_with_the_key():
    """The cached key is rope(y W_k + b_k): with W_k = 0 the cache holds the rotated bias alone."""
    rng = np.random.default_rng(43)
    w = rand_layer(D, 4, 2, 8, F, rng=rng)
    w.wk[:] = 0.0
    bk = rng.normal(size=16)
    x = rng.normal(size=(4, D))
    e = O.empty_cache(SH)
    _, k_all, _ = O.layer_forward(x, e, e, _with_bias(w, None, bk, None), SH)
    want = O.rope(np.tile(bk.reshape(1, 2, 8), (4, 1, 1)), np.arange(4), SH.rope_base)
    assert np.allclose(k_all, want, atol=1e-14)
    assert not np.allclose(k_all[1], bk.reshape(2, 8))                   # position 1 really is rotated

"""fp64 CPU oracle for the forward pass of one pipeline stage.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the GPU
path is checked against.  It is imported by tests, by the smoke check and by
the benchmark's CPU-baseline leg, never by the product path, and it shares no
code with the HIP kernels.

What it computes.  A pipeline stage is a contiguous slice of the model's
layers (paper Sec. 2.2.3); a batch is either all-prefill or all-decode
(separate batching, Sec. 2.3 and Sec. 3.1).  Prefill processes every prompt
token at once and initialises the KV cache; a decode step processes one new
token per request and reads the cached keys and values (Sec. 2.1).  Models
with grouped-query attention share each K/V head among several query heads
(Sec. 4.1).  The paper takes the Llama-2 layer itself as given (Table 2); the
layer below is that public definition: pre-norm residual blocks, RMSNorm,
rotary position embedding in the half-split pairing, softmax attention with
scale 1/sqrt(head_dim), SwiGLU feed-forward, no biases.  The paper's third
model (Qwen2.5-32B, Table 2) is the same layer with biases on the q / k / v
projections; LayerWeights carries them as optional fields.

Requests are independent, so the oracle works on ONE request at a time with a
contiguous (unpaged) KV list: paging is the thing under test, not part of the
definition.  All arithmetic is float64; matrices are [in, out] so y = x @ W.

Every function here is pinned by tests/test_oracle_pins.py against closed
forms, invariants, brute force and an independently composed library
formulation.  Not pinned ("parity unpinned"): which of the two rotary pairings
a real checkpoint expects, since no trained weights are available; with
synthetic weights the two differ by a fixed column permutation of W_q / W_k.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Iterable, List, Optional, Sequence, Tuple

import numpy as np

from .fp8_oracle import kv_roundtrip

F64 = np.float64


@dataclass
class LayerWeights:
    """One decoder layer; matrices [in, out], gains [d_model]; all float64."""
    wq: np.ndarray
    wk: np.ndarray
    wv: np.ndarray
    wo: np.ndarray
    wg: np.ndarray
    wu: np.ndarray
    wd: np.ndarray
    g_attn: np.ndarray
    g_mlp: np.ndarray
    # Optional biases of the q / k / v projections ([d_q], [d_kv], [d_kv]): the Qwen2.5 row of the
    # paper's Table 2 is a Llama-style layer with exactly this addition (public model definition);
    # None = no bias (Llama).
    bq: Optional[np.ndarray] = None
    bk: Optional[np.ndarray] = None
    bv: Optional[np.ndarray] = None


@dataclass
class Shape:
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    # 8-bit KV cache option (fp8_oracle.py): (k_scale, v_scale), or None for a cache that stores
    # keys and values as they are.
    kv_scales: Optional[Tuple[float, float]] = None


def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """y = x * g / sqrt(mean(x^2) + eps), per row."""
    x = np.asarray(x, F64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x * np.asarray(g, F64) / np.sqrt(ms + eps)


def rope(z: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotary embedding, half-split pairing.  z: [L, H, dh]; pos: [L].
    Pair i is (z[i], z[i + dh/2]) and turns by the angle pos * base^(-2i/dh)."""
    z = np.asarray(z, F64)
    dh = z.shape[-1]
    half = dh // 2
    i = np.arange(half, dtype=F64)
    theta = base ** (-2.0 * i / dh)
    ang = np.asarray(pos, F64)[:, None] * theta[None, :]          # [L, half]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    a = z[..., :half]
    b = z[..., half:]
    return np.concatenate([a * c - b * s, a * s + b * c], axis=-1)


def softmax(s: np.ndarray) -> np.ndarray:
    """Softmax of a 1-D score vector (max subtracted first)."""
    e = np.exp(s - np.max(s))
    return e / np.sum(e)


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def attention_weights(q: np.ndarray, k: np.ndarray, n_visible: int) -> np.ndarray:
    """Softmax weights of one query vector q [dh] over keys k[:n_visible] [n, dh]."""
    dh = q.shape[-1]
    s = (k[:n_visible] @ q) / np.sqrt(F64(dh))
    return softmax(s)


def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, p0: int, sh: Shape) -> np.ndarray:
    """Causal attention of L new tokens at absolute positions p0..p0+L-1 over a
    request's full key/value list (cache followed by the new tokens).
    q: [L, Hq, dh]; k, v: [p0 + L, Hkv, dh].  Token i sees keys 0..p0+i.
    Query head h uses K/V head h // (Hq/Hkv).  Returns [L, Hq*dh]."""
    L = q.shape[0]
    G = sh.n_q_heads // sh.n_kv_heads
    out = np.zeros((L, sh.n_q_heads, sh.head_dim), F64)
    for i in range(L):
        n_vis = p0 + i + 1
        for h in range(sh.n_q_heads):
            kvh = h // G
            w = attention_weights(q[i, h], k[:, kvh, :], n_vis)
            out[i, h] = w @ v[:n_vis, kvh, :]
    return out.reshape(L, sh.n_q_heads * sh.head_dim)


def layer_forward(x: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray, w: LayerWeights,
                  sh: Shape) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """One decoder layer for ONE request.
    x: [L, d] new tokens at positions p0..p0+L-1 where p0 = len(k_cache);
    k_cache, v_cache: [p0, Hkv, dh] (keys stored after rotation).
    Returns (x_next [L, d], k_all [p0+L, Hkv, dh], v_all).
    With an 8-bit cache (sh.kv_scales) the cache is the only source of keys and values: the new
    tokens' keys and values go through the format first, attention (prefill and decode alike, Sec.
    2.1: prefill initialises the cache, decode reads it) sees what the cache holds, and the
    returned lists hold that too."""
    x = np.asarray(x, F64)
    L = x.shape[0]
    p0 = k_cache.shape[0]
    pos = np.arange(p0, p0 + L)
    y = rmsnorm(x, w.g_attn, sh.rms_eps)
    q, k, v = y @ w.wq, y @ w.wk, y @ w.wv
    if w.bq is not None:
        q = q + np.asarray(w.bq, F64)  # the bias joins the projection before the rotation
    if w.bk is not None:
        k = k + np.asarray(w.bk, F64)
    if w.bv is not None:
        v = v + np.asarray(w.bv, F64)
    q = q.reshape(L, sh.n_q_heads, sh.head_dim)
    k = k.reshape(L, sh.n_kv_heads, sh.head_dim)
    v = v.reshape(L, sh.n_kv_heads, sh.head_dim)
    q = rope(q, pos, sh.rope_base)
    k = rope(k, pos, sh.rope_base)
    if sh.kv_scales is None:
        k_st, v_st = k, v
    else:
        k_st, v_st = kv_roundtrip(k, sh.kv_scales[0]), kv_roundtrip(v, sh.kv_scales[1])
    k_all = np.concatenate([np.asarray(k_cache, F64), k_st], axis=0)
    v_all = np.concatenate([np.asarray(v_cache, F64), v_st], axis=0)
    a = attention(q, k_all, v_all, p0, sh)
    h = x + a @ w.wo
    y2 = rmsnorm(h, w.g_mlp, sh.rms_eps)
    u = silu(y2 @ w.wg) * (y2 @ w.wu)
    return h + u @ w.wd, k_all, v_all


def empty_cache(sh: Shape) -> np.ndarray:
    return np.zeros((0, sh.n_kv_heads, sh.head_dim), F64)


def stage_forward(x: np.ndarray, caches: Optional[Sequence[Tuple[np.ndarray, np.ndarray]]],
                  layers: Iterable[LayerWeights], sh: Shape
                  ) -> Tuple[np.ndarray, List[Tuple[np.ndarray, np.ndarray]]]:
    """The whole stage for ONE request: L new tokens through every layer.
    caches[l] = (k, v) held for layer l before the call (None = empty: prefill).
    Returns the stage output [L, d] (no final norm: the stage is mid-pipeline)
    and the per-layer caches after the call."""
    new_caches = []
    for li, w in enumerate(layers):
        if caches is None:
            kc, vc = empty_cache(sh), empty_cache(sh)
        else:
            kc, vc = caches[li]
        x, k_all, v_all = layer_forward(x, kc, vc, w, sh)
        new_caches.append((k_all, v_all))
    return x, new_caches


def stage_prefill(prompts: Sequence[np.ndarray], layers: Sequence[LayerWeights], sh: Shape):
    """Prefill phase: each prompt [L_s, d] starts from an empty cache.
    Returns ([out_s], [caches_s])."""
    outs, caches = [], []
    for x in prompts:
        o, c = stage_forward(x, None, layers, sh)
        outs.append(o)
        caches.append(c)
    return outs, caches


def stage_decode(xs: Sequence[np.ndarray], caches: Sequence[Sequence[Tuple[np.ndarray, np.ndarray]]],
                 layers: Sequence[LayerWeights], sh: Shape):
    """Decode step: request b contributes one token xs[b] [d] at position
    len(cache_b); attention covers the cache plus the token itself."""
    outs, new = [], []
    for x, c in zip(xs, caches):
        o, nc = stage_forward(np.asarray(x, F64)[None, :], c, layers, sh)
        outs.append(o[0])
        new.append(nc)
    return outs, new

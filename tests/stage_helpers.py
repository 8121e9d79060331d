"""Oracle-side plumbing of the GPU parity tests: turn generated weights into oracle inputs and
compare with the stated tolerance.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

from harness import workload as W
from harness.runner import Stage, dev_view_bf16, i32  # noqa: F401  (re-exported for the tests)
from oracle import stage_oracle as O

TOL = 2e-2          # max |gpu - oracle| / max |oracle row|, on bf16 outputs with fp32 accumulation


def oracle_shape(sh: W.StageShape) -> O.Shape:
    return O.Shape(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.rms_eps, sh.rope_base)


def _gen_device() -> str:
    # the generator is bit-identical on both devices (tested); the GPU is only faster
    return "cuda" if torch.cuda.is_available() else "cpu"


def oracle_layer(sh: W.StageShape, layer: int, dtype=torch.bfloat16, device=None) -> O.LayerWeights:
    """Generated weights, rounded like the GPU path stores them (bf16), widened to fp64."""
    device = device or _gen_device()
    def get(name):
        w = W.weight(sh, layer, name, device=device, dtype=dtype)
        if not name.startswith(("g_", "b")):
            w = w.to(torch.bfloat16)      # matrices are held in bf16 by the stage; gains and biases stay fp32
        return w.to("cpu").to(torch.float64).numpy()
    biases = {n: get(n) for n in W.BIAS_NAMES} if sh.qkv_bias else {}
    return O.LayerWeights(*(get(n) for n in W.WEIGHT_NAMES), **biases)


def oracle_layers(sh: W.StageShape, dtype=torch.bfloat16, device=None):
    """Lazy: one layer's fp64 weights alive at a time."""
    for l in range(sh.n_layers):
        yield oracle_layer(sh, l, dtype, device)


def f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


def row_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max over rows of max|got - ref| / max|ref| (the row's largest magnitude)."""
    got = np.asarray(got, np.float64).reshape(-1, ref.shape[-1])
    ref = np.asarray(ref, np.float64).reshape(-1, ref.shape[-1])
    assert np.isfinite(got).all(), "non-finite output"
    denom = np.max(np.abs(ref), axis=-1)
    denom = np.where(denom == 0, 1.0, denom)
    return float(np.max(np.max(np.abs(got - ref), axis=-1) / denom))


def bf16_round(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even to bf16, returned as float64."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16).to(torch.float64).numpy()


def layer_forward_bf16_operands(x, k_cache, v_cache, w: O.LayerWeights, sh: O.Shape):
    """The oracle's layer, composed from the oracle's own primitives, with every tensor that a
    bf16-operand implementation must hold in bf16 rounded to bf16 (norm outputs, q, k, v before and
    after rotation, attention output, SwiGLU output) and ALL arithmetic left in fp64.  Its distance
    to the unrounded oracle is the error floor of any such implementation on this input: it
    measures the precision, not a kernel."""
    rb = bf16_round
    x = np.asarray(x, np.float64)
    L, p0 = x.shape[0], k_cache.shape[0]
    pos = np.arange(p0, p0 + L)
    y = rb(O.rmsnorm(x, w.g_attn, sh.rms_eps))
    bias = lambda b: 0.0 if b is None else np.asarray(b, np.float64)
    q = rb(O.rope(rb(y @ w.wq + bias(w.bq)).reshape(L, sh.n_q_heads, sh.head_dim), pos, sh.rope_base))
    k = rb(O.rope(rb(y @ w.wk + bias(w.bk)).reshape(L, sh.n_kv_heads, sh.head_dim), pos, sh.rope_base))
    v = rb(y @ w.wv + bias(w.bv)).reshape(L, sh.n_kv_heads, sh.head_dim)
    k_all = np.concatenate([np.asarray(k_cache, np.float64), k], axis=0)
    v_all = np.concatenate([np.asarray(v_cache, np.float64), v], axis=0)
    a = rb(O.attention(q, k_all, v_all, p0, sh))
    h = x + a @ w.wo
    y2 = rb(O.rmsnorm(h, w.g_mlp, sh.rms_eps))
    u = rb(O.silu(y2 @ w.wg) * (y2 @ w.wu))
    return h + u @ w.wd, k_all, v_all

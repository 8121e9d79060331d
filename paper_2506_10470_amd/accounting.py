"""Algorithmic work of one pipeline-stage pass: the bytes the method must move
and the flops it must do, independent of any implementation.  Used for the
roofline figures the benchmark prints.

The KV-cache size formula reproduces the paper's worked example (Sec. 2.2.1:
Llama-30B, about 1.52 MB per token, about 178 GB for 400 requests of average
length 300) and the weight count reproduces the model sizes of Table 2.
"""
from __future__ import annotations

from typing import Sequence


def matmul_params_per_layer(d_model: int, n_q_heads: int, n_kv_heads: int, head_dim: int, d_ff: int) -> int:
    """Parameters in the seven projection matrices of one decoder layer."""
    return d_model * head_dim * (2 * n_q_heads + 2 * n_kv_heads) + 3 * d_model * d_ff


def kv_bytes_per_token(n_layers: int, n_kv_heads: int, head_dim: int, elem_bytes: int = 2) -> int:
    """K and V of one token across n_layers layers."""
    return 2 * n_layers * n_kv_heads * head_dim * elem_bytes


def decode_step_work(n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ff,
                     ctx_lens: Sequence[int], elem_bytes: int = 2, kv_elem_bytes: int = 0):
    """Algorithmic (bytes, flops) of one decode step.  ctx_lens = tokens already
    cached per request; the step reads ctx+1 tokens of K/V and appends one.
    Weights are read once per step whatever the batch size; activations between
    kernels are implementation traffic and are not counted.  kv_elem_bytes: bytes
    per cached element when the cache is held in another type than the model
    (0 = the same)."""
    B = len(ctx_lens)
    P = matmul_params_per_layer(d_model, n_q_heads, n_kv_heads, head_dim, d_ff)
    kvtok = kv_bytes_per_token(1, n_kv_heads, head_dim, kv_elem_bytes or elem_bytes)
    span = sum(int(c) + 1 for c in ctx_lens)
    w_bytes = n_layers * P * elem_bytes
    kv_read = n_layers * kvtok * span
    kv_write = n_layers * kvtok * B
    io = 2 * B * d_model * elem_bytes
    gemm_flops = 2 * B * n_layers * P
    attn_flops = 4 * n_layers * n_q_heads * head_dim * span
    return {
        "bytes": w_bytes + kv_read + kv_write + io,
        "weight_bytes": w_bytes, "kv_read_bytes": kv_read, "kv_write_bytes": kv_write, "io_bytes": io,
        "flops": gemm_flops + attn_flops, "gemm_flops": gemm_flops, "attn_flops": attn_flops,
    }


def prefill_work(n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ff,
                 seq_lens: Sequence[int], elem_bytes: int = 2):
    """Algorithmic (bytes, flops) of one prefill batch; causal attention counts
    only the visible (j <= i) pairs."""
    T = sum(int(l) for l in seq_lens)
    P = matmul_params_per_layer(d_model, n_q_heads, n_kv_heads, head_dim, d_ff)
    kvtok = kv_bytes_per_token(1, n_kv_heads, head_dim, elem_bytes)
    gemm_flops = 2 * T * n_layers * P
    attn_flops = n_layers * sum(2 * n_q_heads * head_dim * int(l) * (int(l) + 1) for l in seq_lens)
    byts = n_layers * P * elem_bytes + n_layers * kvtok * T + 2 * T * d_model * elem_bytes
    return {"bytes": byts, "flops": gemm_flops + attn_flops, "gemm_flops": gemm_flops,
            "attn_flops": attn_flops, "tokens": T}

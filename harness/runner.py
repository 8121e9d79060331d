"""Plumbing shared by the tests, the benchmark and the smoke check: create a stage through the
C ABI, load generated weights, view the KV pools as tensors.  None of the method's arithmetic
lives here, and nothing here touches the oracle."""
from __future__ import annotations

import numpy as np
import torch

from harness import workload as W


class DevMem:
    """Zero-copy view of raw device memory through the CUDA array interface."""

    def __init__(self, ptr: int, n_elems: int, typestr: str = "<i2"):
        self.__cuda_array_interface__ = {"shape": (n_elems,), "typestr": typestr,
                                         "data": (ptr, False), "version": 2}


def dev_view_bf16(ptr: int, nbytes: int) -> torch.Tensor:
    return torch.as_tensor(DevMem(ptr, nbytes // 2), device="cuda").view(torch.bfloat16)


def dev_view_u8(ptr: int, nbytes: int) -> torch.Tensor:
    return torch.as_tensor(DevMem(ptr, nbytes, "|u1"), device="cuda")

class Stage:
    def __init__(self, tdp, shape: W.StageShape, num_pages: int, max_batch: int, max_tokens: int,
                 max_seqs: int, max_pages_per_seq: int, weight_dtype=torch.bfloat16, load_weights=True,
                 kv_scales=None, layer_offset: int = 0, decode_micro_batches: int = 0):
        """kv_scales: None = bf16 KV pools; (k_scale, v_scale) = 8-bit (E4M3) pools with those scales.
        layer_offset: the stage's layer l gets the generated weights of model layer layer_offset + l (a
        later stage of a pipeline)."""
        self.tdp = tdp
        self.shape = shape
        self.kv_scales = kv_scales
        self.layer_offset = layer_offset
        self.cfg = tdp.StageConfig(
            n_layers=shape.n_layers, d_model=shape.d_model, n_q_heads=shape.n_q_heads,
            n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim, d_ff=shape.d_ff, rms_eps=shape.rms_eps,
            rope_base=shape.rope_base, page_size=shape.page_size, num_pages=num_pages, max_batch=max_batch,
            max_tokens=max_tokens, max_seqs=max_seqs, max_pages_per_seq=max_pages_per_seq,
            kv_dtype=tdp.KV_BF16 if kv_scales is None else tdp.KV_FP8_E4M3,
            k_scale=0.0 if kv_scales is None else kv_scales[0], v_scale=0.0 if kv_scales is None else kv_scales[1],
            decode_micro_batches=decode_micro_batches)
        self.h = tdp.tdp_stage_create(self.cfg)
        self.num_pages = num_pages
        self.max_pages_per_seq = max_pages_per_seq
        if load_weights:
            self.load_weights(weight_dtype)

    def load_weights(self, dtype=torch.bfloat16):
        tdp, sh = self.tdp, self.shape
        for l in range(sh.n_layers):
            for name in W.WEIGHT_NAMES + (W.BIAS_NAMES if sh.qkv_bias else ()):
                w = W.weight(sh, self.layer_offset + l, name, device="cuda", dtype=dtype).contiguous()
                rows = w.shape[0]
                cols = w.shape[1] if w.dim() == 2 else 1
                tdp.tdp_stage_set_weight(self.h, l, tdp.WEIGHT_IDS[name], w,
                                         tdp.BF16 if dtype == torch.bfloat16 else tdp.F32, tdp.DEVICE, rows, cols)
                del w

    def raw_pools(self, layer):
        """Zero-copy flat views of the layer's K and V pools: bf16, or the raw codes (uint8) of an 8-bit cache."""
        k, v, n = self.tdp.tdp_stage_kv_pool(self.h, layer)
        view = dev_view_bf16 if self.kv_scales is None else dev_view_u8
        return view(k, n), view(v, n)

    def pools(self, layer):
        """(K [pages, Hkv, 16, dh], V [pages, Hkv, dh, 16]) in logical coordinates, from the documented
        layout alone.  V is a zero-copy view.  K is a copy: in memory a key row is cut into 64-byte pieces
        and piece g of the 16 tokens of a page lies together, [pages, Hkv, row bytes / 64, 16, 64 bytes]."""
        kf, vf = self.raw_pools(layer)
        sh = self.shape
        per_piece = 32 if self.kv_scales is None else 64          # elements in 64 bytes
        kt = kf.view(self.num_pages, sh.n_kv_heads, sh.head_dim // per_piece, 16, per_piece)
        kt = kt.permute(0, 1, 3, 2, 4).reshape(self.num_pages, sh.n_kv_heads, 16, sh.head_dim)
        vt = vf.view(self.num_pages, sh.n_kv_heads, sh.head_dim, 16)
        return kt, vt

    POISON_CODE = 0x7F   # the NaN of the 8-bit format

    def poison(self):
        for l in range(self.shape.n_layers):
            for t in self.raw_pools(l):
                t.fill_(float("nan") if self.kv_scales is None else self.POISON_CODE)
        torch.cuda.synchronize()

    def close(self):
        if self.h:
            self.tdp.tdp_stage_destroy(self.h)
            self.h = None

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()


def i32(a, device="cuda") -> torch.Tensor:
    return torch.as_tensor(np.ascontiguousarray(a, dtype=np.int32), device=device)

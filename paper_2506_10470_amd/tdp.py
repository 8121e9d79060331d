"""ctypes binding of libtdp.so: the same entry points as include/tdp.h, argument marshalling
only.  Every step of the stage runs in the library's HIP kernels; torch is used by callers for
device memory and streams.  Importing this module fails loudly when the library is not built.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("TDP_LIB", os.path.join(_HERE, "libtdp.so"))   # TDP_LIB: alternative build

OK, EINVAL, ENOMEM, EHIP = 0, -1, -2, -3
WQ, WK, WV, WO, WG, WU, WD, G_ATTN, G_MLP, BQ, BK, BV = range(12)
WEIGHT_IDS = {"wq": WQ, "wk": WK, "wv": WV, "wo": WO, "wg": WG, "wu": WU, "wd": WD,
              "g_attn": G_ATTN, "g_mlp": G_MLP, "bq": BQ, "bk": BK, "bv": BV}
F32, BF16 = 0, 1
HOST, DEVICE = 0, 1
KV_BF16, KV_FP8_E4M3 = 0, 1
TIMING_CLASSES = ("rmsnorm", "gemm_qkv", "rope_kv", "attention", "gemm_o", "gemm_gate_up", "gemm_down",
                  "attention_merge")


class StageConfig(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ff", C.c_int32),
                ("rms_eps", C.c_float), ("rope_base", C.c_float), ("page_size", C.c_int32),
                ("num_pages", C.c_int32), ("max_batch", C.c_int32), ("max_tokens", C.c_int32),
                ("max_seqs", C.c_int32), ("max_pages_per_seq", C.c_int32),
                ("kv_dtype", C.c_int32), ("k_scale", C.c_float), ("v_scale", C.c_float),
                ("decode_micro_batches", C.c_int32)]


class EndsConfig(C.Structure):
    _fields_ = [("vocab_size", C.c_int32), ("d_model", C.c_int32), ("rms_eps", C.c_float),
                ("max_tokens", C.c_int32)]


E_EMBEDDING, E_FINAL_NORM, E_LM_HEAD = 0, 1, 2


class TdpError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("tdp error %d: %s" % (code, msg))
        self.code = code


# torch ships its own HIP runtime; it must be the one libtdp.so binds to (two runtimes in one
# process cannot both own the GPU), so torch is loaded first.
import torch  # noqa: E402,F401

if not os.path.exists(LIB_PATH):
    raise ImportError("libtdp.so is not built: run `python -m paper_2506_10470_amd.build` "
                      "(there is no CPU fallback)")
lib = C.CDLL(LIB_PATH)

_vp, _i32, _i64 = C.c_void_p, C.c_int32, C.c_int64
_SIGS = {
    "tdp_abi_version": (C.c_int, []),
    "tdp_last_error": (C.c_char_p, []),
    "tdp_stage_create": (C.c_int, [C.POINTER(StageConfig), C.POINTER(_vp)]),
    "tdp_stage_destroy": (None, [_vp]),
    "tdp_stage_set_weight": (C.c_int, [_vp, _i32, _i32, _vp, _i32, _i32, _i64, _i64]),
    "tdp_stage_kv_pool": (C.c_int, [_vp, _i32, C.POINTER(_vp), C.POINTER(_vp), C.POINTER(_i64)]),
    "tdp_stage_kv_import": (C.c_int, [_vp, _i32, _vp, _vp, _vp, _vp, _i32, _i32, _vp]),
    "tdp_stage_kv_export": (C.c_int, [_vp, _i32, _vp, _vp, _vp, _vp, _i32, _i32, _vp]),
    "tdp_stage_prefill": (C.c_int, [_vp, _vp, _vp, _vp, _i32, _i32, _vp, _vp]),
    "tdp_stage_decode": (C.c_int, [_vp, _vp, _vp, _vp, _i32, _vp, _vp]),
    "tdp_stage_check_decode": (C.c_int, [_vp, _vp, _vp, _i32, _vp]),
    "tdp_stage_check_prefill": (C.c_int, [_vp, _vp, _vp, _i32, _i32, _vp]),
    "tdp_stage_set_layer_range": (C.c_int, [_vp, _i32, _i32]),
    "tdp_stage_set_decode_span": (C.c_int, [_vp, _i32]),
    "tdp_gemm_bf16": (C.c_int, [_vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _i32, _vp]),
    "tdp_gemm_bf16_static": (C.c_int, [_vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _i32, _vp]),
    "tdp_e4m3_from_f32": (C.c_int, [_vp, _vp, _i64, C.c_float, _vp]),
    "tdp_e4m3_to_f32": (C.c_int, [_vp, _vp, _i64, _vp]),
    "tdp_probe_hbm_read": (C.c_int, [_vp, _i64, _i32, _i32, C.POINTER(_i64), C.POINTER(C.c_float), _vp]),
    "tdp_probe_mfma_bf16": (C.c_int, [_i32, _i32, _i32, C.POINTER(C.c_double), C.POINTER(C.c_float), _vp]),
    "tdp_stage_timing_enable": (C.c_int, [_vp, _i32]),
    "tdp_stage_timing_read": (C.c_int, [_vp, C.POINTER(C.c_float)]),
    "tdp_ends_create": (C.c_int, [C.POINTER(EndsConfig), C.POINTER(_vp)]),
    "tdp_ends_destroy": (None, [_vp]),
    "tdp_ends_set_weight": (C.c_int, [_vp, _i32, _vp, _i32, _i32, _i64, _i64]),
    "tdp_embed_tokens": (C.c_int, [_vp, _vp, _i32, _vp, _vp]),
    "tdp_lm_head": (C.c_int, [_vp, _vp, _i32, _vp, _i32, _vp, _vp, _vp]),
    "tdp_argmax_rows": (C.c_int, [_vp, _i32, _i32, _i64, _vp, _vp]),
}
for _name, (_res, _args) in _SIGS.items():
    _f = getattr(lib, _name)
    _f.restype = _res
    _f.argtypes = _args


def last_error() -> str:
    return lib.tdp_last_error().decode()


def _check(rc: int) -> None:
    if rc != OK:
        raise TdpError(rc, last_error())


def _ptr(t) -> Optional[int]:
    """Address of a torch tensor / numpy array / int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if hasattr(t, "data_ptr"):
        return t.data_ptr()
    return t.ctypes.data


def _stream(stream) -> Optional[int]:
    if stream is None:
        return None
    return getattr(stream, "cuda_stream", stream)


def tdp_abi_version() -> int:
    return lib.tdp_abi_version()


def tdp_stage_create(cfg: StageConfig) -> int:
    h = _vp()
    _check(lib.tdp_stage_create(C.byref(cfg), C.byref(h)))
    return h.value


def tdp_stage_destroy(st: int) -> None:
    lib.tdp_stage_destroy(st)


def tdp_stage_set_weight(st, layer, which, src, dtype, mem, rows, cols) -> None:
    _check(lib.tdp_stage_set_weight(st, layer, which, _ptr(src), dtype, mem, rows, cols))


def tdp_stage_kv_pool(st, layer):
    k, v, n = _vp(), _vp(), _i64()
    _check(lib.tdp_stage_kv_pool(st, layer, C.byref(k), C.byref(v), C.byref(n)))
    return k.value, v.value, n.value


def tdp_stage_kv_import(st, layer, k_packed, v_packed, cu_seqlens, block_tables, n_seqs, total_tokens,
                        stream=None) -> None:
    _check(lib.tdp_stage_kv_import(st, layer, _ptr(k_packed), _ptr(v_packed), _ptr(cu_seqlens),
                                   _ptr(block_tables), n_seqs, total_tokens, _stream(stream)))


def tdp_stage_kv_export(st, layer, k_packed, v_packed, cu_seqlens, block_tables, n_seqs, total_tokens,
                        stream=None) -> None:
    _check(lib.tdp_stage_kv_export(st, layer, _ptr(k_packed), _ptr(v_packed), _ptr(cu_seqlens),
                                   _ptr(block_tables), n_seqs, total_tokens, _stream(stream)))


def tdp_stage_prefill(st, hidden_in, cu_seqlens, block_tables, n_seqs, total_tokens, hidden_out,
                      stream=None) -> None:
    _check(lib.tdp_stage_prefill(st, _ptr(hidden_in), _ptr(cu_seqlens), _ptr(block_tables), n_seqs,
                                 total_tokens, _ptr(hidden_out), _stream(stream)))


def tdp_stage_decode(st, hidden_in, ctx_lens, block_tables, batch, hidden_out, stream=None) -> None:
    _check(lib.tdp_stage_decode(st, _ptr(hidden_in), _ptr(ctx_lens), _ptr(block_tables), batch,
                                _ptr(hidden_out), _stream(stream)))


def tdp_stage_check_decode(st, ctx_lens, block_tables, batch, stream=None) -> None:
    _check(lib.tdp_stage_check_decode(st, _ptr(ctx_lens), _ptr(block_tables), batch, _stream(stream)))


def tdp_stage_check_prefill(st, cu_seqlens, block_tables, n_seqs, total_tokens, stream=None) -> None:
    _check(lib.tdp_stage_check_prefill(st, _ptr(cu_seqlens), _ptr(block_tables), n_seqs, total_tokens,
                                       _stream(stream)))


def tdp_stage_set_layer_range(st, first: int, count: int) -> None:
    _check(lib.tdp_stage_set_layer_range(st, first, count))


def tdp_stage_set_decode_span(st, span_tokens: int) -> None:
    _check(lib.tdp_stage_set_decode_span(st, span_tokens))


def tdp_gemm_bf16(A, W, residual, out, M, N, K, epilogue=0, tile=0, splits=0, stream=None) -> None:
    _check(lib.tdp_gemm_bf16(_ptr(A), _ptr(W), _ptr(residual), _ptr(out), M, N, K, epilogue, tile, splits,
                             _stream(stream)))


def tdp_gemm_bf16_static(A, W, residual, out, M, N, K, epilogue=0, tile=0, splits=0, stream=None) -> None:
    _check(lib.tdp_gemm_bf16_static(_ptr(A), _ptr(W), _ptr(residual), _ptr(out), M, N, K, epilogue, tile, splits,
                                    _stream(stream)))


def tdp_e4m3_from_f32(src, codes, n, scale=1.0, stream=None) -> None:
    _check(lib.tdp_e4m3_from_f32(_ptr(src), _ptr(codes), n, scale, _stream(stream)))


def tdp_e4m3_to_f32(codes, dst, n, stream=None) -> None:
    _check(lib.tdp_e4m3_to_f32(_ptr(codes), _ptr(dst), n, _stream(stream)))


def tdp_probe_hbm_read(buf, nbytes: int, scattered: bool, launches: int = 5, stream=None, non_temporal: bool = False):
    """-> (bytes read per launch, ms per launch)"""
    n, ms = _i64(), C.c_float()
    _check(lib.tdp_probe_hbm_read(_ptr(buf), nbytes, int(bool(scattered)) | (2 if non_temporal else 0), launches,
                                  C.byref(n), C.byref(ms), _stream(stream)))
    return n.value, ms.value


def tdp_probe_mfma_bf16(iters: int, launches: int = 5, random_operands: bool = True, stream=None):
    """-> (flop per launch, ms per launch)"""
    f, ms = C.c_double(), C.c_float()
    _check(lib.tdp_probe_mfma_bf16(iters, launches, int(bool(random_operands)), C.byref(f), C.byref(ms),
                                   _stream(stream)))
    return f.value, ms.value


def tdp_stage_timing_enable(st, on: bool) -> None:
    _check(lib.tdp_stage_timing_enable(st, 1 if on else 0))


def tdp_stage_timing_read(st) -> dict:
    ms = (C.c_float * len(TIMING_CLASSES))()
    _check(lib.tdp_stage_timing_read(st, ms))
    return dict(zip(TIMING_CLASSES, [float(x) for x in ms]))


def tdp_ends_create(cfg: EndsConfig) -> int:
    h = _vp()
    _check(lib.tdp_ends_create(C.byref(cfg), C.byref(h)))
    return h.value


def tdp_ends_destroy(e: int) -> None:
    lib.tdp_ends_destroy(e)


def tdp_ends_set_weight(e, which, src, dtype, mem, rows, cols) -> None:
    _check(lib.tdp_ends_set_weight(e, which, _ptr(src), dtype, mem, rows, cols))


def tdp_embed_tokens(e, token_ids, M, hidden_out, stream=None) -> None:
    _check(lib.tdp_embed_tokens(e, _ptr(token_ids), M, _ptr(hidden_out), _stream(stream)))


def tdp_lm_head(e, hidden_in, n_rows_in, row_index, M, logits_out, next_token, stream=None) -> None:
    _check(lib.tdp_lm_head(e, _ptr(hidden_in), n_rows_in, _ptr(row_index), M, _ptr(logits_out), _ptr(next_token),
                           _stream(stream)))


def tdp_argmax_rows(logits, M, n, ld, out, stream=None) -> None:
    _check(lib.tdp_argmax_rows(_ptr(logits), M, n, ld, _ptr(out), _stream(stream)))

"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching the device."""
import os
import re

import pytest

from paper_2506_10470_amd import tdp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def good_config(**kw):
    base = dict(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64, d_ff=688, rms_eps=1e-5,
                rope_base=10000.0, page_size=16, num_pages=8, max_batch=4, max_tokens=64, max_seqs=4,
                max_pages_per_seq=4)
    base.update(kw)
    return tdp.StageConfig(**base)


def test_every_declared_symbol_is_exported():
    text = open(os.path.join(ROOT, "include", "tdp.h")).read()
    declared = set(re.findall(r"TDP_API\s+[\w\s\*]+?\b(tdp_\w+)\s*\(", text))
    assert len(declared) >= 12
    for name in declared:
        assert hasattr(tdp.lib, name), name
        assert name in tdp._SIGS, "binding lacks " + name
    assert tdp.tdp_abi_version() == 5


@pytest.mark.parametrize("bad", [
    dict(n_layers=0), dict(d_model=100), dict(head_dim=96), dict(n_q_heads=6, n_kv_heads=4),
    dict(n_q_heads=34, n_kv_heads=2), dict(d_ff=0), dict(d_ff=690), dict(page_size=32), dict(num_pages=0),
    dict(max_batch=0, max_tokens=0), dict(max_batch=-1), dict(max_pages_per_seq=0), dict(rope_base=0.0),
    dict(max_tokens=8, max_seqs=0), dict(kv_dtype=2), dict(kv_dtype=-1),
    dict(kv_dtype=1, k_scale=-1.0), dict(kv_dtype=1, v_scale=float("inf")), dict(kv_dtype=1, k_scale=float("nan")),
    dict(decode_micro_batches=3), dict(decode_micro_batches=-1),
])
def test_create_rejects_bad_config_before_any_gpu_work(bad):
    with pytest.raises(tdp.TdpError) as e:
        tdp.tdp_stage_create(good_config(**bad))
    assert e.value.code == tdp.EINVAL
    assert tdp.last_error() != ""


def test_null_arguments_are_einval():
    import ctypes as C
    assert tdp.lib.tdp_stage_create(None, None) == tdp.EINVAL
    h = C.c_void_p()
    assert tdp.lib.tdp_stage_create(None, C.byref(h)) == tdp.EINVAL
    assert tdp.lib.tdp_stage_decode(None, None, None, None, 1, None, None) == tdp.EINVAL
    assert tdp.lib.tdp_stage_prefill(None, None, None, None, 1, 1, None, None) == tdp.EINVAL
    assert tdp.lib.tdp_stage_kv_pool(None, 0, None, None, None) == tdp.EINVAL
    assert tdp.lib.tdp_stage_set_weight(None, 0, 0, None, 0, 0, 1, 1) == tdp.EINVAL
    assert tdp.lib.tdp_stage_timing_read(None, None) == tdp.EINVAL
    tdp.lib.tdp_stage_destroy(None)          # allowed


def test_e4m3_diagnostics_reject_bad_arguments():
    assert tdp.lib.tdp_e4m3_from_f32(None, None, 4, 1.0, None) == tdp.EINVAL
    assert tdp.lib.tdp_e4m3_from_f32(16, 16, -1, 1.0, None) == tdp.EINVAL
    assert tdp.lib.tdp_e4m3_from_f32(16, 16, 4, 0.0, None) == tdp.EINVAL
    assert tdp.lib.tdp_e4m3_to_f32(None, None, 4, None) == tdp.EINVAL
    assert tdp.lib.tdp_e4m3_to_f32(16, 16, 6, None) == tdp.EINVAL          # not a multiple of 4
    assert tdp.lib.tdp_e4m3_to_f32(18, 16, 4, None) == tdp.EINVAL          # misaligned codes
    assert tdp.lib.tdp_e4m3_from_f32(None, None, 0, 1.0, None) == tdp.OK   # empty: nothing to do


def test_gemm_entry_rejects_bad_shapes():
    for M, N, K, epi, tile, splits in [(-1, 64, 64, 0, 0, 0), (1, 0, 64, 0, 0, 0), (1, 64, 100, 0, 0, 0),
                                       (1, 66, 64, 0, 0, 0), (1, 64, 64, 3, 0, 0), (1, 68, 64, 2, 0, 0), (1, 64, 64, 0, 17, 0),
                                       (1, 64, 64, 0, 0, -1)]:
        assert tdp.lib.tdp_gemm_bf16(None, None, None, None, M, N, K, epi, tile, splits, None) == tdp.EINVAL
    # M = 0 is a no-op, and null pointers with M > 0 are rejected
    assert tdp.lib.tdp_gemm_bf16(None, None, None, None, 0, 64, 64, 0, 0, 0, None) == tdp.OK
    assert tdp.lib.tdp_gemm_bf16(None, None, None, None, 1, 64, 64, 0, 0, 0, None) == tdp.EINVAL


def test_allocation_free_gemm_entry_checks_its_limits_before_any_gpu_work():
    G = tdp.lib.tdp_gemm_bf16_static
    for M, N, K, epi, tile, splits in [(-1, 64, 64, 0, 0, 0), (1, 0, 64, 0, 0, 0), (1, 64, 100, 0, 0, 0),
                                       (1, 66, 64, 0, 0, 0), (1, 64, 64, 2, 0, 0), (1, 64, 64, 0, 17, 0),
                                       (1, 64, 64, 0, 0, -1)]:
        assert G(None, None, None, None, M, N, K, epi, tile, splits, None) == tdp.EINVAL
    assert G(16, 16, None, 16, 1, 4096, 4096, 0, 0, 0, None) == tdp.EINVAL      # 16 Mi weight elements > 8 Mi
    assert "static scratch" in tdp.last_error()
    assert G(16, 16, None, 16, 4096, 256, 64, 0, 0, 0, None) == tdp.EINVAL      # 16 Mi floats of partials > 12 Mi
    assert "workspace" in tdp.last_error()
    assert G(None, None, None, None, 0, 64, 64, 0, 0, 0, None) == tdp.OK
    assert G(None, None, None, None, 1, 64, 64, 0, 0, 0, None) == tdp.EINVAL    # null pointers


def test_layer_range_and_timing_calls_reject_null_stage():
    assert tdp.lib.tdp_stage_set_layer_range(None, 0, 1) == tdp.EINVAL
    assert tdp.lib.tdp_stage_timing_enable(None, 1) == tdp.EINVAL
    assert tdp.lib.tdp_stage_set_decode_span(None, 256) == tdp.EINVAL
    assert tdp.lib.tdp_stage_kv_import(None, 0, None, None, None, None, 1, 1, None) == tdp.EINVAL
    assert tdp.lib.tdp_stage_kv_export(None, 0, None, None, None, None, 1, 1, None) == tdp.EINVAL
    assert tdp.lib.tdp_stage_check_decode(None, None, None, 1, None) == tdp.EINVAL
    assert tdp.lib.tdp_stage_check_prefill(None, None, None, 1, 1, None) == tdp.EINVAL


def test_ends_entry_points_reject_bad_arguments():
    import ctypes as C
    for bad in [dict(vocab_size=0), dict(vocab_size=1001), dict(d_model=100), dict(rms_eps=-1.0), dict(max_tokens=0)]:
        base = dict(vocab_size=1000, d_model=256, rms_eps=1e-5, max_tokens=8)
        base.update(bad)
        with pytest.raises(tdp.TdpError) as e:
            tdp.tdp_ends_create(tdp.EndsConfig(**base))
        assert e.value.code == tdp.EINVAL
    assert tdp.lib.tdp_ends_create(None, None) == tdp.EINVAL
    assert tdp.lib.tdp_embed_tokens(None, None, 1, None, None) == tdp.EINVAL
    assert tdp.lib.tdp_lm_head(None, None, 1, None, 1, None, None, None) == tdp.EINVAL
    assert tdp.lib.tdp_ends_set_weight(None, 0, None, 0, 0, 1, 1) == tdp.EINVAL
    assert tdp.lib.tdp_argmax_rows(None, 1, 0, 0, None, None) == tdp.EINVAL
    assert tdp.lib.tdp_argmax_rows(None, 1, 8, 4, None, None) == tdp.EINVAL      # ld < n
    assert tdp.lib.tdp_argmax_rows(None, 1, 8, 8, None, None) == tdp.EINVAL      # null pointers
    assert tdp.lib.tdp_argmax_rows(None, 0, 8, 8, None, None) == tdp.OK          # empty is a no-op
    tdp.lib.tdp_ends_destroy(None)


def test_probe_entry_points_reject_bad_arguments():
    import ctypes as C
    n, ms, fl = C.c_int64(), C.c_float(), C.c_double()
    P = tdp.lib.tdp_probe_hbm_read
    assert P(None, 1 << 20, 0, 1, C.byref(n), C.byref(ms), None) == tdp.EINVAL          # null buffer
    assert P(4096, 1 << 20, 0, 1, None, C.byref(ms), None) == tdp.EINVAL                # null result
    assert P(4100, 1 << 20, 0, 1, C.byref(n), C.byref(ms), None) == tdp.EINVAL          # misaligned
    assert P(4096, 1 << 18, 0, 1, C.byref(n), C.byref(ms), None) == tdp.EINVAL          # below 512 KiB
    assert P(4096, 1 << 20, 4, 1, C.byref(n), C.byref(ms), None) == tdp.EINVAL          # pattern
    assert P(4096, 1 << 20, -1, 1, C.byref(n), C.byref(ms), None) == tdp.EINVAL
    assert P(4096, 1 << 20, 0, 0, C.byref(n), C.byref(ms), None) == tdp.EINVAL          # launches
    assert P(4096, 1 << 20, 0, 1001, C.byref(n), C.byref(ms), None) == tdp.EINVAL
    M = tdp.lib.tdp_probe_mfma_bf16
    assert M(0, 1, 1, C.byref(fl), C.byref(ms), None) == tdp.EINVAL
    assert M((1 << 22) + 1, 1, 1, C.byref(fl), C.byref(ms), None) == tdp.EINVAL
    assert M(16, 0, 1, C.byref(fl), C.byref(ms), None) == tdp.EINVAL
    assert M(16, 1, 2, C.byref(fl), C.byref(ms), None) == tdp.EINVAL
    assert M(16, 1, 1, None, C.byref(ms), None) == tdp.EINVAL
    assert "iters" in tdp.last_error() or "null" in tdp.last_error()

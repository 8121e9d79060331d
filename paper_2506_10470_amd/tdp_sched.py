"""ctypes binding of libtdp_sched.so: the entry points of include/tdp_sched.h under the same names,
argument marshalling only.  Host code: needs neither torch nor a GPU.  Importing this module fails
loudly when the library is not built."""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("TDP_SCHED_LIB", os.path.join(_HERE, "libtdp_sched.so"))
if not os.path.exists(LIB_PATH):
    raise ImportError("libtdp_sched.so is not built: run `python -m paper_2506_10470_amd.build`")
lib = C.CDLL(LIB_PATH)

EINVAL, EABORT = -1, -2
EVENT_KINDS = ("prefill", "decode", "switch_to_prefill")


class SimConfig(C.Structure):
    _fields_ = [("n_stages", C.c_int32), ("kv_capacity", C.c_int64), ("prefill_token_budget", C.c_int32),
                ("greedy_prefill", C.c_int32), ("work_stealing", C.c_int32), ("intensity_switch", C.c_int32),
                ("count_decode_steps", C.c_int32)]


class SimResult(C.Structure):
    _fields_ = [("total_ms", C.c_double), ("busy_ms", C.c_double), ("generated_tokens", C.c_int64),
                ("prefill_tokens", C.c_int64), ("peak_kv_tokens", C.c_int64), ("n_events", C.c_int64),
                ("phase_switches", C.c_int32), ("recomputes", C.c_int32)]


class SimEvent(C.Structure):
    _fields_ = [("kind", C.c_int32), ("time_ms", C.c_double), ("a", C.c_int64), ("b", C.c_int64)]


_vp, _i32, _i64, _dbl = C.c_void_p, C.c_int32, C.c_int64, C.c_double
_pi32, _pi64, _pd = C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.POINTER(C.c_double)

PREFILL_FN = C.CFUNCTYPE(C.c_int, _vp, _pi64, _pi32, _i32)
DECODE_FN = C.CFUNCTYPE(C.c_int, _vp, _i32, _pi64, _pi32, _i32)
RELEASE_FN = C.CFUNCTYPE(C.c_int, _vp, _pi64, _i32, _i32)


class SimExecutor(C.Structure):
    _fields_ = [("user", _vp), ("prefill", PREFILL_FN), ("decode", DECODE_FN), ("release", RELEASE_FN)]

_SIGS = {
    "tdp_sched_abi_version": (C.c_int, []),
    "tdp_prefill_switch_create": (C.c_int, [_i64, _pi32, _i32, C.POINTER(_vp)]),
    "tdp_prefill_switch_destroy": (None, [_vp]),
    "tdp_prefill_switch_reset": (C.c_int, [_vp]),
    "tdp_prefill_switch_update": (C.c_int, [_vp, _i32, _i32]),
    "tdp_prefill_switch_usage": (C.c_int, [_vp, _pi64, _i32]),
    "tdp_prefill_switch_check": (C.c_int, [_vp]),
    "tdp_work_stealing_create": (C.c_int, [_i32, _pi64, _i32, C.POINTER(_vp)]),
    "tdp_work_stealing_destroy": (None, [_vp]),
    "tdp_work_stealing_batch": (C.c_int, [_vp, _i32, _pi64, _i32, _pi32]),
    "tdp_work_stealing_withheld": (C.c_int, [_vp, _pi64, _i32, _pi32]),
    "tdp_work_stealing_on_return": (C.c_int, [_vp, _i32, _pi64, _i32, _pi64, _i32, _pi32]),
    "tdp_profile_time": (_dbl, [_pd, _pd, _i32, _dbl]),
    "tdp_spatial_intensity": (_dbl, [_pd, _pd, _i32, _dbl]),
    "tdp_temporal_intensity": (_dbl, [_pd, _i32, _dbl, _i32, _i32]),
    "tdp_switch_to_prefill": (C.c_int, [_pd, _pd, _i32, _dbl, _pd, _i32, _dbl, _i32, _i32]),
    "tdp_simulate": (C.c_int, [C.POINTER(SimConfig), _pi32, _pi32, _pi32, _i64, _pd, _pd, _i32, _pd, _pd, _i32,
                               C.POINTER(SimResult), C.POINTER(SimEvent), _i64]),
    "tdp_simulate_exec": (C.c_int, [C.POINTER(SimConfig), _pi32, _pi32, _pi32, _i64, _pd, _pd, _i32, _pd, _pd, _i32,
                                    C.POINTER(SimResult), C.POINTER(SimEvent), _i64, C.POINTER(SimExecutor)]),
}
for _name, (_res, _args) in _SIGS.items():
    _f = getattr(lib, _name)
    _f.restype = _res
    _f.argtypes = _args


class SchedError(RuntimeError):
    pass


def _check(rc: int) -> int:
    if rc == EABORT:
        raise SchedError("tdp_sched: the run was stopped by an executor callback")
    if rc < 0:
        raise SchedError("tdp_sched: invalid argument")
    return rc


def _arr(ctype, values):
    values = list(values)
    return (ctype * max(len(values), 1))(*values), len(values)


def tdp_sched_abi_version() -> int:
    return lib.tdp_sched_abi_version()


# ---- Algorithm 1
def tdp_prefill_switch_create(kv_capacity: int, future_points: Optional[Sequence[int]] = None) -> int:
    h = _vp()
    if future_points is None:
        _check(lib.tdp_prefill_switch_create(kv_capacity, None, 0, C.byref(h)))
    else:
        a, n = _arr(C.c_int32, future_points)
        _check(lib.tdp_prefill_switch_create(kv_capacity, a, n, C.byref(h)))
    return h.value


def tdp_prefill_switch_destroy(h: int) -> None:
    lib.tdp_prefill_switch_destroy(h)


def tdp_prefill_switch_reset(h: int) -> None:
    _check(lib.tdp_prefill_switch_reset(h))


def tdp_prefill_switch_update(h: int, input_len: int, predict_len: int) -> None:
    _check(lib.tdp_prefill_switch_update(h, input_len, predict_len))


def tdp_prefill_switch_usage(h: int, max_points: int = 4096) -> List[int]:
    buf = (C.c_int64 * max_points)()
    n = _check(lib.tdp_prefill_switch_usage(h, buf, max_points))
    return list(buf[:n])


def tdp_prefill_switch_check(h: int) -> bool:
    return bool(_check(lib.tdp_prefill_switch_check(h)))


# ---- work stealing
def tdp_work_stealing_create(n_batches: int, request_ids: Sequence[int]) -> int:
    h = _vp()
    a, n = _arr(C.c_int64, request_ids)
    _check(lib.tdp_work_stealing_create(n_batches, a, n, C.byref(h)))
    return h.value


def tdp_work_stealing_destroy(h: int) -> None:
    lib.tdp_work_stealing_destroy(h)


def tdp_work_stealing_batch(h: int, batch: int, cap: int = 1 << 16) -> List[int]:
    buf, n = (C.c_int64 * cap)(), C.c_int32()
    _check(lib.tdp_work_stealing_batch(h, batch, buf, cap, C.byref(n)))
    return list(buf[:n.value])


def tdp_work_stealing_withheld(h: int, cap: int = 1 << 16) -> List[int]:
    buf, n = (C.c_int64 * cap)(), C.c_int32()
    _check(lib.tdp_work_stealing_withheld(h, buf, cap, C.byref(n)))
    return list(buf[:n.value])


def tdp_work_stealing_on_return(h: int, batch: int, finished_ids: Sequence[int], cap: int = 1 << 16) -> List[int]:
    fin, nf = _arr(C.c_int64, finished_ids)
    buf, n = (C.c_int64 * cap)(), C.c_int32()
    _check(lib.tdp_work_stealing_on_return(h, batch, fin, nf, buf, cap, C.byref(n)))
    return list(buf[:n.value])


# ---- intensities
def _profile(profile: Sequence[Tuple[float, float]]):
    xs, n = _arr(C.c_double, [p[0] for p in profile])
    ms, _ = _arr(C.c_double, [p[1] for p in profile])
    return xs, ms, n


def tdp_profile_time(profile, at: float) -> float:
    xs, ms, n = _profile(profile)
    return lib.tdp_profile_time(xs, ms, n, at)


def tdp_spatial_intensity(profile, batch: float) -> float:
    xs, ms, n = _profile(profile)
    return lib.tdp_spatial_intensity(xs, ms, n, batch)


def tdp_temporal_intensity(pending_prefill_ms: Sequence[float], decode_ms: float, n_batches: int,
                           count_decode_steps: bool = True) -> float:
    a, n = _arr(C.c_double, pending_prefill_ms)
    return lib.tdp_temporal_intensity(a, n, decode_ms, n_batches, int(count_decode_steps))


def tdp_switch_to_prefill(profile, batch: float, pending_prefill_ms: Sequence[float], decode_ms: float,
                          n_batches: int, count_decode_steps: bool = True) -> bool:
    xs, ms, n = _profile(profile)
    a, na = _arr(C.c_double, pending_prefill_ms)
    return bool(_check(lib.tdp_switch_to_prefill(xs, ms, n, batch, a, na, decode_ms, n_batches,
                                                 int(count_decode_steps))))


# ---- simulated pipeline
def tdp_simulate(cfg: SimConfig, requests: Sequence[Tuple[int, int, int]], decode_profile, prefill_profile,
                 events_cap: int = 0):
    """Returns (SimResult, [(kind, time_ms, a, b), ...]) with at most events_cap events."""
    ins, n = _arr(C.c_int32, [r[0] for r in requests])
    outs, _ = _arr(C.c_int32, [r[1] for r in requests])
    preds, _ = _arr(C.c_int32, [r[2] for r in requests])
    dx, dms, nd = _profile(decode_profile)
    px, pms, npre = _profile(prefill_profile)
    res = SimResult()
    ev = (SimEvent * max(events_cap, 1))()
    _check(lib.tdp_simulate(C.byref(cfg), ins, outs, preds, n, dx, dms, nd, px, pms, npre, C.byref(res),
                            ev if events_cap else None, events_cap))
    k = min(res.n_events, events_cap)
    return res, [(EVENT_KINDS[ev[i].kind], ev[i].time_ms, ev[i].a, ev[i].b) for i in range(k)]


def tdp_simulate_exec(cfg: SimConfig, requests: Sequence[Tuple[int, int, int]], decode_profile, prefill_profile,
                      prefill=None, decode=None, release=None, events_cap: int = 0):
    """tdp_simulate with the work done by the caller: `prefill(ids, input_lens)`, `decode(batch, ids, contexts)`
    and `release(ids, reason)` are called with Python lists at the events they stand for (any may be None).
    An exception raised in a callback stops the run and is raised again here."""
    ins, n = _arr(C.c_int32, [r[0] for r in requests])
    outs, _ = _arr(C.c_int32, [r[1] for r in requests])
    preds, _ = _arr(C.c_int32, [r[2] for r in requests])
    dx, dms, nd = _profile(decode_profile)
    px, pms, npre = _profile(prefill_profile)
    res = SimResult()
    ev = (SimEvent * max(events_cap, 1))()
    failure: List[BaseException] = []

    def guard(fn, *args) -> int:
        try:
            fn(*args)
            return 0
        except BaseException as e:  # never let an exception cross the C frames
            failure.append(e)
            return 1

    c_prefill = PREFILL_FN(lambda _u, ids, lens, k: guard(prefill, [ids[i] for i in range(k)], [lens[i] for i in range(k)])) \
        if prefill else PREFILL_FN()
    c_decode = DECODE_FN(lambda _u, b, ids, ctx, k: guard(decode, b, [ids[i] for i in range(k)], [ctx[i] for i in range(k)])) \
        if decode else DECODE_FN()
    c_release = RELEASE_FN(lambda _u, ids, k, why: guard(release, [ids[i] for i in range(k)], why)) \
        if release else RELEASE_FN()
    ex = SimExecutor(None, c_prefill, c_decode, c_release)
    rc = lib.tdp_simulate_exec(C.byref(cfg), ins, outs, preds, n, dx, dms, nd, px, pms, npre, C.byref(res),
                               ev if events_cap else None, events_cap, C.byref(ex))
    if failure:
        raise failure[0]
    _check(rc)
    k = min(res.n_events, events_cap)
    return res, [(EVENT_KINDS[ev[i].kind], ev[i].time_ms, ev[i].a, ev[i].b) for i in range(k)]

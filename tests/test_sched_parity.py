"""The scheduler library (libtdp_sched.so, through its C ABI) against the plain-Python oracle.
Host code on both sides: no GPU needed.  Integer results must be identical; times are the same
formulas in the same order, compared to 1e-9 relative."""
import os
import random
import re

import pytest

from oracle import sched_oracle as S
from paper_2506_10470_amd import tdp_sched as L

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
DEC = [(16, 7.96), (32, 8.5), (64, 9.09), (128, 10.75), (256, 15.17), (512, 25.75)]
PRE = [(256, 8.0), (1024, 30.0), (4096, 120.0), (16384, 480.0)]


def test_every_declared_symbol_is_exported_and_bound():
    text = open(os.path.join(ROOT, "include", "tdp_sched.h")).read()
    declared = set(re.findall(r"TDP_SCHED_API\s+[\w\s\*]+?\b(tdp_\w+)\s*\(", text))
    assert len(declared) == 18
    for name in declared:
        assert hasattr(L.lib, name), name
        assert name in L._SIGS, "binding lacks " + name
    assert L.tdp_sched_abi_version() == 1


def test_bad_arguments_are_rejected():
    import ctypes as C
    assert L.lib.tdp_prefill_switch_create(100, None, 0, None) == L.EINVAL
    assert L.lib.tdp_prefill_switch_update(None, 1, 1) == L.EINVAL
    assert L.lib.tdp_prefill_switch_check(None) == L.EINVAL
    with pytest.raises(L.SchedError):
        L.tdp_prefill_switch_create(100, [64, 32])                    # not ascending
    with pytest.raises(L.SchedError):
        L.tdp_work_stealing_create(0, [1, 2, 3])
    h = L.tdp_work_stealing_create(2, [1, 2, 3])
    with pytest.raises(L.SchedError):
        L.tdp_work_stealing_on_return(h, 2, [])                       # no such batch
    with pytest.raises(L.SchedError):
        L.tdp_work_stealing_on_return(h, 0, [], cap=1)                # output array too small
    L.tdp_work_stealing_destroy(h)
    assert L.tdp_profile_time([(2, 1.0), (1, 2.0)], 1.5) != L.tdp_profile_time([(2, 1.0), (1, 2.0)], 1.5)  # NaN
    assert L.lib.tdp_simulate(None, None, None, None, 0, None, None, 0, None, None, 0, None, None, 0) == L.EINVAL
    L.tdp_prefill_switch_destroy(None)
    L.tdp_work_stealing_destroy(None)


# ------------------------------------------------------------------ Algorithm 1

@pytest.mark.parametrize("points", [None, (1, 2, 3, 5, 8), (32, 64)])
def test_prefill_switch_matches_oracle(points):
    rng = random.Random(21)
    cap = 40000
    o = S.PrefillSwitch(cap, points) if points else S.PrefillSwitch(cap)
    h = L.tdp_prefill_switch_create(cap, points)
    flips = 0
    for k in range(400):
        a, p = rng.randint(0, 1023), rng.randint(0, 1300)
        o.update_usage(a, p)
        L.tdp_prefill_switch_update(h, a, p)
        assert L.tdp_prefill_switch_usage(h) == [o.kv_usage[q] for q in o.future_points]
        assert L.tdp_prefill_switch_check(h) == o.check_switch()
        flips += o.check_switch()
        if k == 250:
            o = S.PrefillSwitch(cap, points) if points else S.PrefillSwitch(cap)
            L.tdp_prefill_switch_reset(h)
    assert flips > 0
    L.tdp_prefill_switch_destroy(h)


# ------------------------------------------------------------------ work stealing

def test_work_stealing_example_through_the_library():
    h = L.tdp_work_stealing_create(4, list(range(512)))
    assert [len(L.tdp_work_stealing_batch(h, i)) for i in range(4)] == [128] * 4
    b0 = L.tdp_work_stealing_batch(h, 0)
    assert len(L.tdp_work_stealing_on_return(h, 0, b0[:48])) == 80
    b1 = L.tdp_work_stealing_batch(h, 1)
    assert len(L.tdp_work_stealing_on_return(h, 1, b1[:8])) == 114
    assert len(L.tdp_work_stealing_withheld(h)) == 6
    assert len(L.tdp_work_stealing_on_return(h, 2, [])) == 114
    assert len(L.tdp_work_stealing_on_return(h, 3, [])) == 114
    assert len(L.tdp_work_stealing_withheld(h)) == 34
    assert len(L.tdp_work_stealing_on_return(h, 0, [])) == 114
    assert L.tdp_work_stealing_withheld(h) == []
    L.tdp_work_stealing_destroy(h)


@pytest.mark.parametrize("n,total,seed", [(4, 512, 1), (3, 100, 2), (8, 1000, 3), (2, 5, 4), (4, 0, 5)])
def test_work_stealing_matches_oracle_id_for_id(n, total, seed):
    rng = random.Random(seed)
    ids = [rng.randrange(10 ** 12) for _ in range(total)]
    ids = list(dict.fromkeys(ids))
    o = S.WorkStealing(n, ids)
    h = L.tdp_work_stealing_create(n, ids)
    for i in range(n):
        assert L.tdp_work_stealing_batch(h, i) == o.batches[i]
    for it in range(300):
        i = rng.randrange(n)
        done = [r for r in o.batches[i] if rng.random() < 0.05]
        rng.shuffle(done)
        assert L.tdp_work_stealing_on_return(h, i, done) == o.on_return(i, done)
        assert L.tdp_work_stealing_withheld(h) == list(o.withheld)
    L.tdp_work_stealing_destroy(h)


# ------------------------------------------------------------------ intensities

def test_intensities_match_oracle():
    rng = random.Random(9)
    for b in [0, 1, 15.5, 16, 17, 48, 64, 100, 511, 512, 513, 2000]:
        assert L.tdp_profile_time(DEC, b) == pytest.approx(S.interp_time(DEC, b), rel=1e-12)
        assert L.tdp_spatial_intensity(DEC, b) == pytest.approx(S.spatial_intensity(DEC, b), rel=1e-12)
    for _ in range(200):
        pend = [rng.uniform(1, 500) for _ in range(rng.randint(0, 6))]
        d = rng.uniform(5, 60)
        nb = rng.randint(1, 8)
        cnt = rng.random() < 0.5
        b = rng.uniform(1, 600)
        assert L.tdp_temporal_intensity(pend, d, nb, cnt) == pytest.approx(S.temporal_intensity(pend, d, nb, cnt),
                                                                           rel=1e-12, abs=1e-15)
        assert L.tdp_switch_to_prefill(DEC, b, pend, d, nb, cnt) == S.switch_to_prefill(DEC, b, pend, d, nb, cnt)


# ------------------------------------------------------------------ simulated pipeline

def _requests(n, seed, long_tail=False):
    rng = random.Random(seed)
    out = []
    for _ in range(n):
        a = rng.randint(4, 1000)
        o = rng.randint(1, 900 if long_tail else 300)
        p = max(0, int(o * rng.uniform(0.5, 1.5)))
        out.append((a, o, p))
    return out


CASES = [
    # n_requests, seed, stages, capacity, budget, greedy, stealing, intensity, count_steps
    (200, 1, 4, 60000, 4096, 1, 1, 1, 1),
    (200, 2, 4, 60000, 4096, 0, 0, 0, 1),
    (150, 3, 2, 30000, 2048, 1, 1, 1, 0),
    (150, 4, 8, 90000, 8192, 1, 0, 1, 1),
    (120, 5, 4, 9000, 4096, 1, 1, 1, 1),      # tight memory: recomputation happens
    (120, 6, 4, 9000, 4096, 0, 1, 0, 1),
    (60, 7, 1, 20000, 1024, 1, 1, 1, 1),
    (5, 8, 4, 20000, 4096, 1, 1, 1, 1),       # fewer requests than stages
    (0, 9, 4, 20000, 4096, 1, 1, 1, 1),
]


@pytest.mark.parametrize("case", CASES)
def test_simulation_matches_oracle_event_for_event(case):
    n_req, seed, stages, cap, budget, greedy, steal, inten, cnt = case
    reqs = _requests(n_req, seed, long_tail=cap < 10000)
    ocfg = S.SimConfig(n_stages=stages, kv_capacity=cap, prefill_token_budget=budget, greedy_prefill=bool(greedy),
                       work_stealing=bool(steal), intensity_switch=bool(inten), count_decode_steps=bool(cnt))
    ref = S.simulate(reqs, ocfg, DEC, PRE)
    cfg = L.SimConfig(stages, cap, budget, greedy, steal, inten, cnt)
    res, events = L.tdp_simulate(cfg, reqs, DEC, PRE, events_cap=len(ref.events) + 10)
    assert res.n_events == len(ref.events)
    assert (res.generated_tokens, res.prefill_tokens, res.peak_kv_tokens, res.phase_switches, res.recomputes) == \
        (ref.generated_tokens, ref.prefill_tokens, ref.peak_kv_tokens, ref.phase_switches, ref.recomputes)
    for got, want in zip(events, ref.events):
        assert got[0] == want[0] and got[2:] == tuple(want[2:]), (got, want)
        assert got[1] == pytest.approx(want[1], rel=1e-9)
    assert res.total_ms == pytest.approx(ref.total_ms, rel=1e-9)
    assert res.busy_ms == pytest.approx(ref.busy_ms, rel=1e-9)
    if case[5] == 1 and cap < 10000:
        assert ref.recomputes > 0          # the tight case really exercises the eviction path


def test_simulation_rejects_a_prompt_that_can_never_fit():
    cfg = L.SimConfig(4, 100, 4096, 1, 1, 1, 1)
    with pytest.raises(L.SchedError):
        L.tdp_simulate(cfg, [(500, 10, 10)], DEC, PRE)
    with pytest.raises(RuntimeError):
        S.simulate([(500, 10, 10)], S.SimConfig(n_stages=4, kv_capacity=100), DEC, PRE)


def test_events_cap_truncates_but_counts():
    reqs = _requests(50, 12)
    cfg = L.SimConfig(4, 60000, 4096, 1, 1, 1, 1)
    full, ev_full = L.tdp_simulate(cfg, reqs, DEC, PRE, events_cap=100000)
    cut, ev_cut = L.tdp_simulate(cfg, reqs, DEC, PRE, events_cap=7)
    none, ev_none = L.tdp_simulate(cfg, reqs, DEC, PRE, events_cap=0)
    assert full.n_events == cut.n_events == none.n_events > 7
    assert ev_cut == ev_full[:7] and ev_none == []
    assert cut.total_ms == full.total_ms

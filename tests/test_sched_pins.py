"""Pins for the scheduling oracle (oracle/sched_oracle.py): values the paper prints, brute force,
closed forms and invariants.  No GPU, no library."""
import os
import random

import pytest

from oracle import sched_oracle as S

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ Sec. 3.4: the worked example

def _example_rows():
    rows = []
    for line in open(os.path.join(GOLDEN, "work_stealing_example.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        rows.append(line.split())
    return rows


def test_work_stealing_reproduces_the_papers_example():
    rows = _example_rows()
    assert rows[0][0] == "initial"
    ws = S.WorkStealing(4, list(range(512)))
    assert [len(b) for b in ws.batches] == [int(x) for x in rows[0][1:]]
    for batch, finished, average, submitted, withheld in rows[1:]:
        batch, finished, average, submitted, withheld = map(int, (batch, finished, average, submitted, withheld))
        done = ws.batches[batch][:finished]
        out = ws.on_return(batch, done)
        assert -(-ws.live_total() // 4) == average
        assert len(out) == submitted
        assert len(ws.withheld) == withheld
        assert not set(out) & set(done)


def test_work_stealing_conserves_requests_and_balances():
    rng = random.Random(7)
    n = 4
    ws = S.WorkStealing(n, list(range(403)))
    alive = set(range(403))
    for it in range(400):
        i = it % n
        batch = ws.batches[i]
        done = [r for r in batch if rng.random() < 0.03]
        alive -= set(done)
        out = ws.on_return(i, done)
        held = set(ws.withheld)
        members = [r for b in ws.batches for r in b]
        assert len(members) == len(set(members)) and not held & set(members)       # nobody twice
        assert set(members) | held == alive                                        # nobody lost
        assert len(out) <= -(-len(alive) // n)                                     # never above the average
    sizes = [len(b) for b in ws.batches]
    assert max(sizes) - min(sizes) <= max(3, len(alive) // 20)


def test_work_stealing_initial_split_is_even():
    ws = S.WorkStealing(4, list(range(10)))
    assert [len(b) for b in ws.batches] == [3, 3, 2, 2]
    assert sum(ws.batches, []) == list(range(10))


# ------------------------------------------------------------------ Sec. 3.3: Algorithm 1

def test_future_points_are_every_32_steps_to_1024():
    assert S.FUTURE_POINTS[0] == 32 and S.FUTURE_POINTS[-1] == 1024 and len(S.FUTURE_POINTS) == 32
    assert all(b - a == 32 for a, b in zip(S.FUTURE_POINTS, S.FUTURE_POINTS[1:]))


def test_incremental_usage_equals_direct_simulation():
    rng = random.Random(3)
    reqs = [(rng.randint(1, 1023), rng.randint(1, 1500)) for _ in range(200)]
    sw = S.PrefillSwitch(10 ** 9)
    for k, (a, p) in enumerate(reqs):
        sw.update_usage(a, p)
        if k % 37 == 0 or k == len(reqs) - 1:
            for fp in S.FUTURE_POINTS:
                assert sw.kv_usage[fp] == S.usage_at_step_direct(reqs[:k + 1], fp)


def test_direct_usage_matches_a_step_by_step_decode():
    """usage_at_step_direct against an explicit token-by-token run of the decode phase."""
    reqs = [(5, 3), (7, 1), (2, 6), (9, 4)]
    length = [a for a, _ in reqs]
    alive = [True] * len(reqs)
    for step in range(1, 8):
        for i, (a, p) in enumerate(reqs):
            if alive[i]:
                length[i] += 1
        held = sum(length[i] for i in range(len(reqs)) if alive[i])
        assert held == S.usage_at_step_direct(reqs, step)
        for i, (a, p) in enumerate(reqs):
            if p <= step:
                alive[i] = False  # produced its last token at this step; its cache is freed afterwards


def test_switch_fires_exactly_when_some_future_point_exceeds_capacity():
    sw = S.PrefillSwitch(kv_capacity=1000, future_points=(32, 64))
    sw.update_usage(400, 40)          # 432 at step 32, gone by 64
    assert not sw.check_switch()
    sw.update_usage(500, 100)         # +532 at 32 (964), +564 at 64
    assert sw.kv_usage == {32: 964, 64: 564} and not sw.check_switch()
    sw.update_usage(5, 33)            # +37 at 32 -> 1001 > 1000
    assert sw.check_switch()


def test_short_requests_never_count():
    sw = S.PrefillSwitch(kv_capacity=10)
    for _ in range(100):
        sw.update_usage(1000, 31)     # finished before the first future point
    assert sw.max_usage() == 0 and not sw.check_switch()


# ------------------------------------------------------------------ Sec. 3.5: Eq. 1 and Eq. 2

PROFILE = [(16, 8.0), (32, 8.5), (64, 9.1), (128, 10.8), (256, 15.2), (512, 25.8)]


def test_spatial_intensity_is_one_at_the_peak_and_below_elsewhere():
    peak_batch = max(PROFILE, key=lambda p: p[0] / p[1])[0]
    assert S.spatial_intensity(PROFILE, peak_batch) == pytest.approx(1.0)
    vals = [S.spatial_intensity(PROFILE, b) for b, _ in PROFILE]
    assert all(0 < v <= 1.0 for v in vals)
    assert vals == sorted(vals)                     # this profile gets more efficient with batch size
    assert S.spatial_intensity(PROFILE, 16) == pytest.approx((16 / 8.0) / (512 / 25.8))
    assert S.spatial_intensity(PROFILE, 0) == 0.0


def test_interpolated_times():
    assert S.interp_time(PROFILE, 48) == pytest.approx(8.8)
    assert S.interp_time(PROFILE, 4) == 8.0           # not cheaper than the smallest profiled batch
    assert S.interp_time(PROFILE, 1024) == pytest.approx(51.6)


def test_temporal_intensity_closed_forms():
    assert S.temporal_intensity([30.0, 50.0], 60.0, 4) == 1.0                      # no bubble
    # one pending prefill p, decode step d < p, decode steps ignored: 1 - (p-d)/(2p-d)
    p, d = 100.0, 20.0
    assert S.temporal_intensity([p], d, 4, count_decode_steps=False) == pytest.approx(1 - (p - d) / (2 * p - d))
    # with the decode steps counted the total grows by n*d
    assert S.temporal_intensity([p], d, 4) == pytest.approx(1 - (p - d) / (2 * p - d + 4 * d))
    # more pending work amortises the same bubble
    assert S.temporal_intensity([p] * 8, d, 4) > S.temporal_intensity([p], d, 4)
    assert S.temporal_intensity([], d, 4) == 0.0


def test_decision_rule():
    # large batch: decode is efficient, stay; small batch with lots of pending prefill: switch
    assert not S.switch_to_prefill(PROFILE, 512, [100.0], 25.8, 4)
    assert S.switch_to_prefill(PROFILE, 16, [100.0] * 10, 8.0, 4)
    assert not S.switch_to_prefill(PROFILE, 16, [], 8.0, 4)


# ------------------------------------------------------------------ simulated pipeline: invariants

PREFILL_PROFILE = [(256, 8.0), (1024, 30.0), (4096, 120.0), (16384, 480.0)]


def _requests(n, seed):
    rng = random.Random(seed)
    out = []
    for _ in range(n):
        a = rng.randint(8, 900)
        o = rng.randint(1, 600)
        p = max(1, int(o * rng.uniform(0.6, 1.4)))
        out.append((a, o, p))
    return out


@pytest.mark.parametrize("flags", [(True, True, True), (False, False, False), (True, False, True), (True, True, False)])
def test_simulation_finishes_every_request_and_conserves_tokens(flags):
    reqs = _requests(300, 11)
    cfg = S.SimConfig(n_stages=4, kv_capacity=60000, greedy_prefill=flags[0], work_stealing=flags[1],
                      intensity_switch=flags[2])
    res = S.simulate(reqs, cfg, PROFILE, PREFILL_PROFILE)
    assert res.generated_tokens >= sum(o for _, o, _ in reqs)          # recomputed tokens are generated twice
    if res.recomputes == 0:
        assert res.generated_tokens == sum(o for _, o, _ in reqs)
        assert res.prefill_tokens == sum(a for a, _, _ in reqs)
    assert res.peak_kv_tokens <= cfg.kv_capacity + 4 * 512             # overshoot is bounded by one step
    times = [e[1] for e in res.events]
    assert all(t >= 0 for t in times) and res.total_ms >= max(times)
    assert 0.0 <= S.bubble_ratio(res, 4) < 1.0


def test_single_stage_single_request_timeline():
    """One stage, one request of 3 output tokens: prefill, then two decode steps, back to back."""
    cfg = S.SimConfig(n_stages=1, kv_capacity=10000)
    res = S.simulate([(100, 3, 3)], cfg, PROFILE, PREFILL_PROFILE)
    assert res.generated_tokens == 3 and res.prefill_tokens == 100
    assert res.total_ms == pytest.approx(8.0 + 2 * 8.0)
    assert S.bubble_ratio(res, 1) == pytest.approx(0.0)


def test_two_stage_timeline_by_hand_phase_switches_are_compact():
    """Two stages, two prompts that need a prefill batch each (p = 10 ms per stage), decode steps of
    d = 2 ms per stage, three output tokens per request.  By hand: the prefills leave the pipeline at
    2p = 20 and 3p = 30.  Decode batch 0 (the first request, whose token exists at 20) does not wait
    for the second prefill to leave: it enters stage 0 at 20, finds stage 1 busy until 30 and returns
    at 30 + d = 32; batch 1 (ready at 30) follows it: 34; their second steps return at 36 and 38.
    (Waiting for the pipeline to drain first would give 34, 36, 38, 40.)"""
    flat_decode = [(1, 2.0), (64, 2.0)]
    flat_prefill = [(1, 10.0), (64, 10.0)]
    cfg = S.SimConfig(n_stages=2, kv_capacity=10000, prefill_token_budget=8, intensity_switch=False)
    res = S.simulate([(8, 3, 3), (8, 3, 3)], cfg, flat_decode, flat_prefill)
    assert [(k, a, b) for k, _, a, b in res.events] == [("prefill", 1, 8), ("prefill", 1, 8), ("decode", 0, 1),
                                                        ("decode", 1, 1), ("decode", 0, 0), ("decode", 1, 0)]
    assert [t for _, t, _, _ in res.events] == pytest.approx([20.0, 30.0, 32.0, 34.0, 36.0, 38.0])
    assert res.total_ms == pytest.approx(38.0)
    # stage time used: 2 prefills + 4 decode steps on each of 2 stages
    assert res.busy_ms == pytest.approx(2 * (2 * 10.0 + 4 * 2.0))


def test_switch_to_prefill_does_not_wait_for_the_steps_in_flight():
    """A decode phase that hands over to prefills: the first prefill enters stage 0 behind the decode
    steps that are still in the pipeline, so it leaves the pipeline earlier than the last of them
    plus a full pass would allow."""
    rng = random.Random(11)
    reqs = [(rng.randint(20, 60), rng.randint(2, 40), rng.randint(2, 40)) for _ in range(120)]
    cfg = S.SimConfig(n_stages=4, kv_capacity=1500, prefill_token_budget=256)
    res = S.simulate(reqs, cfg, PROFILE, PREFILL_PROFILE)
    ev = res.events
    switches = [i for i, e in enumerate(ev) if e[0] == "switch_to_prefill"]
    assert switches, "the run must contain a switch for this pin to say anything"
    compact = 0
    for i in switches:
        later_decodes = [e[1] for e in ev[i + 1:] if e[0] == "decode"]
        first_prefill = next((e for e in ev[i + 1:] if e[0] == "prefill"), None)
        if first_prefill is None or not later_decodes:
            continue
        tokens = first_prefill[3]
        full_pass = 4 * S.interp_time(PREFILL_PROFILE, tokens)
        # drained-first scheduling could not finish the prefill before (last in-flight return + 4 stage times)
        last_inflight = max([t for k, t, _, _ in ev[i + 1: ev.index(first_prefill)] if k == "decode"] + [ev[i][1]])
        if first_prefill[1] < last_inflight + full_pass - 1e-9:
            compact += 1
    assert compact > 0


def test_work_stealing_does_not_hurt_a_skewed_decode_phase():
    """Batches that lose requests at different rates: stealing must not lengthen the run."""
    rng = random.Random(5)
    reqs = []
    for i in range(512):
        o = rng.randint(5, 40) if i < 128 else rng.randint(300, 400)   # the first batch empties early
        reqs.append((64, o, o))
    base = dict(n_stages=4, kv_capacity=10 ** 7, intensity_switch=False)
    on = S.simulate(reqs, S.SimConfig(work_stealing=True, **base), PROFILE, PREFILL_PROFILE)
    off = S.simulate(reqs, S.SimConfig(work_stealing=False, **base), PROFILE, PREFILL_PROFILE)
    assert on.generated_tokens == off.generated_tokens
    assert on.total_ms <= off.total_ms * 1.001

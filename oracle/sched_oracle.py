"""Plain-Python oracle for TD-Pipe's control decisions and a simulated pipeline driven by them.

TEST INFRASTRUCTURE ONLY.  This file is the slow, obvious statement of what the scheduler library
must decide.  It is imported by tests only, never by the product path, and shares no code with the
C++ implementation.

What it covers (paper Sec. 3.3 - 3.5):
  * PrefillSwitch      - the prefill-to-decode switch of Algorithm 1: predicted KV-cache usage at
                         the future decode steps 32, 64, ..., 1024, updated per launched prefill
                         request, compared with the capacity (Sec. 3.3).
  * WorkStealing       - inter-batch work stealing with a sliding window as long as the number of
                         pipeline stages (Sec. 3.4).
  * spatial_intensity, temporal_intensity, switch_to_prefill
                       - Eq. 1, Eq. 2 and the decode-to-prefill rule (Sec. 3.5).
  * simulate           - an n-stage pipeline whose stage times come from a measured profile of the
                         stage library, driven by the three decisions above (Sec. 3.1 - 3.2).

Readings where the paper is silent (each is listed in the design notes as well):
  * kvUsage and kvCapacity count tokens.
  * The average batch size of Sec. 3.4 is ceil(live requests / stages): with the floor, up to
    stages-1 requests could stay withheld for ever; the worked example divides exactly either way.
  * The live-request total counts the withheld requests too (the example's third and fourth
    batches are trimmed to 114, which only follows if the 6 already withheld are counted).
  * Stolen requests are taken from the tail of the batch; withheld requests are handed out first
    in, first out.
  * Stage time for a batch size between two profiled sizes is linearly interpolated; below the
    smallest profiled size it is that size's time (a decode step cannot be cheaper than streaming
    the weights once); above the largest it grows in proportion.
  * Peak of Eq. 1 is the largest Achieved value in the profile.
  * With no pending prefill the temporal intensity is 0: there is nothing to switch to.
  * Requests carried over from an earlier decode phase enter Algorithm 1 with their current length
    as input length and their remaining predicted length (at least 1).

Pinned by tests/test_sched_pins.py: the worked example of Sec. 3.4, brute-force simulation of the
usage curve against Algorithm 1's incremental update, closed forms of both intensities, and
conservation invariants of the simulated pipeline.
"""
from __future__ import annotations

from collections import deque
from dataclasses import dataclass, field
from typing import Dict, List, Sequence, Tuple

FUTURE_POINTS: Tuple[int, ...] = tuple(range(32, 1024 + 1, 32))


# ------------------------------------------------------------------------------ Sec. 3.3, Algorithm 1

class PrefillSwitch:
    """Predicted KV usage (tokens) at each future decode step in `future_points`."""

    def __init__(self, kv_capacity: int, future_points: Sequence[int] = FUTURE_POINTS):
        self.kv_capacity = int(kv_capacity)
        self.future_points = tuple(int(p) for p in future_points)
        self.kv_usage: Dict[int, int] = {p: 0 for p in self.future_points}

    def update_usage(self, input_len: int, predict_len: int) -> None:
        """UpdateUsage: a request predicted to still be decoding at step p holds input_len + p tokens then."""
        for p in self.future_points:
            if p <= predict_len:
                self.kv_usage[p] += input_len + p

    def max_usage(self) -> int:
        return max(self.kv_usage.values()) if self.kv_usage else 0

    def check_switch(self) -> bool:
        """CheckSwitch: True = switch to decode, False = remain in prefill."""
        return self.max_usage() > self.kv_capacity


def usage_at_step_direct(requests: Sequence[Tuple[int, int]], step: int) -> int:
    """The quantity Algorithm 1 tracks, from its definition: after `step` decode steps, every
    request (input_len, predict_len) that has not finished by then holds its prompt plus `step` tokens."""
    total = 0
    for input_len, predict_len in requests:
        if predict_len >= step:
            total += input_len + step
    return total


# ------------------------------------------------------------------------------ Sec. 3.4

class WorkStealing:
    def __init__(self, n_batches: int, request_ids: Sequence[int]):
        """Divide the requests into n_batches batches of equal size (the first len % n get one more)."""
        self.n = int(n_batches)
        ids = list(request_ids)
        q, r = divmod(len(ids), self.n)
        self.batches: List[List[int]] = []
        pos = 0
        for i in range(self.n):
            size = q + (1 if i < r else 0)
            self.batches.append(ids[pos:pos + size])
            pos += size
        self.withheld: deque = deque()

    def live_total(self) -> int:
        return sum(len(b) for b in self.batches) + len(self.withheld)

    def on_return(self, i: int, finished_ids: Sequence[int]) -> List[int]:
        """Batch i has come back from the last stage: drop its finished requests, compare what is
        left with the average over the window, withhold the excess or top up from the withheld."""
        done = set(finished_ids)
        batch = [r for r in self.batches[i] if r not in done]
        self.batches[i] = batch
        total = self.live_total()
        average = -(-total // self.n)  # ceil
        if len(batch) > average:
            excess = batch[average:]
            del batch[average:]
            self.withheld.extend(excess)
        else:
            while len(batch) < average and self.withheld:
                batch.append(self.withheld.popleft())
        return list(batch)


# ------------------------------------------------------------------------------ Sec. 3.5

Profile = Sequence[Tuple[float, float]]  # (batch size or token count, milliseconds), ascending


def interp_time(profile: Profile, x: float) -> float:
    pts = list(profile)
    if x <= pts[0][0]:
        return pts[0][1]
    if x >= pts[-1][0]:
        return pts[-1][1] * (x / pts[-1][0])
    for (x0, t0), (x1, t1) in zip(pts[:-1], pts[1:]):
        if x0 <= x <= x1:
            return t0 + (t1 - t0) * ((x - x0) / (x1 - x0))
    raise AssertionError("profile is not ascending")


def achieved(profile: Profile, batch: float) -> float:
    """Reciprocal of the average execution time per request at this batch size."""
    return batch / interp_time(profile, batch)


def peak(profile: Profile) -> float:
    return max(b / t for b, t in profile)


def spatial_intensity(profile: Profile, batch: float) -> float:
    """Eq. 1: Achieved / Peak."""
    if batch <= 0:
        return 0.0
    return achieved(profile, batch) / peak(profile)


def temporal_intensity(pending_prefill_ms: Sequence[float], decode_ms: float, n_batches: int,
                       count_decode_steps: bool = True) -> float:
    """Eq. 2: 1 - bubble / total.  bubble = longest pending prefill - current decode step (not
    below 0); total = the pending prefills + one decode step of each batch (optional) + the bubble."""
    if not pending_prefill_ms:
        return 0.0
    bubble = max(0.0, max(pending_prefill_ms) - decode_ms)
    total = sum(pending_prefill_ms) + bubble
    if count_decode_steps:
        total += n_batches * decode_ms
    return 1.0 - bubble / total


def switch_to_prefill(profile: Profile, batch: float, pending_prefill_ms: Sequence[float], decode_ms: float,
                      n_batches: int, count_decode_steps: bool = True) -> bool:
    return spatial_intensity(profile, batch) < temporal_intensity(pending_prefill_ms, decode_ms, n_batches,
                                                                  count_decode_steps)


# ------------------------------------------------------------------------------ simulated pipeline

@dataclass
class SimConfig:
    n_stages: int = 4
    kv_capacity: int = 1 << 20          # tokens
    prefill_token_budget: int = 4096    # tokens per prefill batch (at least one prompt goes in)
    greedy_prefill: bool = True         # Algorithm 1; else: prefill while the prompts themselves fit
    work_stealing: bool = True
    intensity_switch: bool = True       # Sec. 3.5; else: decode until every running request is done
    count_decode_steps: bool = True
    future_points: Tuple[int, ...] = FUTURE_POINTS


@dataclass
class _Req:
    rid: int
    input_len: int      # tokens to prefill (grows when a request is recomputed)
    output_len: int     # tokens still to generate, counted from this prefill
    predict_len: int
    generated: int = 0


@dataclass
class SimResult:
    total_ms: float = 0.0
    generated_tokens: int = 0
    prefill_tokens: int = 0
    phase_switches: int = 0
    recomputes: int = 0
    peak_kv_tokens: int = 0
    busy_ms: float = 0.0                # sum over stages of time spent computing
    events: List[Tuple] = field(default_factory=list)   # (kind, time_ms, a, b)


def plan_prefill(waiting: Sequence[_Req], running: Sequence[_Req], cfg: SimConfig) -> List[List[int]]:
    """The prefill batches the next prefill phase will launch, as lists of positions in `waiting`:
    prompts are packed first come first served up to the token budget; after each launch
    Algorithm 1 (or, without it, plain prompt occupancy) decides whether to go on."""
    sw = PrefillSwitch(cfg.kv_capacity, cfg.future_points)
    held = 0
    for r in running:
        sw.update_usage(r.input_len + r.generated, max(r.predict_len - r.generated, 1))
        held += r.input_len + r.generated
    batches: List[List[int]] = []
    pos = 0
    while pos < len(waiting):
        batch: List[int] = []
        tokens = 0
        while pos < len(waiting) and (not batch or tokens + waiting[pos].input_len <= cfg.prefill_token_budget):
            if held + tokens + waiting[pos].input_len + 1 > cfg.kv_capacity:
                break  # the prompt itself does not fit now
            batch.append(pos)
            tokens += waiting[pos].input_len
            pos += 1
        if not batch:
            break
        batches.append(batch)
        held += tokens + len(batch)  # prompt plus the first generated token of each
        for p in batch:
            sw.update_usage(waiting[p].input_len, waiting[p].predict_len)
        if cfg.greedy_prefill and sw.check_switch():
            break
    return batches


def simulate(requests: Sequence[Tuple[int, int, int]], cfg: SimConfig, decode_profile: Profile,
             prefill_profile: Profile) -> SimResult:
    """Offline run (every request present at time 0, as in the throughput runs of Sec. 4.2).

    Pipeline model: a batch visits the n stages in order; a stage runs one batch at a time; a
    stage's time for a decode batch of b requests is interp_time(decode_profile, b), for a
    prefill batch of T tokens interp_time(prefill_profile, T).  A decode batch re-enters stage 0
    when its previous step has left the last stage (Sec. 2.2.3)."""
    n = cfg.n_stages
    res = SimResult()
    waiting: List[_Req] = [_Req(i, a, b, c) for i, (a, b, c) in enumerate(requests)]
    running: List[_Req] = []
    stage_free = [0.0] * n
    by_id: Dict[int, _Req] = {r.rid: r for r in waiting}

    def run_batch(ready: float, dur: float) -> float:
        t = ready
        for s in range(n):
            start = max(t, stage_free[s])
            t = start + dur
            stage_free[s] = t
            res.busy_ms += dur
        return t

    def kv_tokens() -> int:
        return sum(r.input_len + r.generated for r in running)

    now = 0.0
    ready_at: Dict[int, float] = {}  # when a request's newest token became available (its prefill left the pipeline)
    while waiting or running:
        # ---------------- prefill phase
        plan = plan_prefill(waiting, running, cfg)
        taken = 0
        last_finish = now
        for batch in plan:
            reqs = [waiting[p] for p in batch]
            tokens = sum(r.input_len for r in reqs)
            finish = run_batch(max(now, stage_free[0]), interp_time(prefill_profile, tokens))
            res.events.append(("prefill", finish, len(reqs), tokens))
            res.prefill_tokens += tokens
            for r in reqs:
                r.generated = 1  # the prefill produces the first output token
                res.generated_tokens += 1
                running.append(r)
                ready_at[r.rid] = finish
            taken += len(batch)
            last_finish = max(last_finish, finish)
        del waiting[:taken]
        res.peak_kv_tokens = max(res.peak_kv_tokens, kv_tokens())
        # requests whose only output token came from the prefill are finished already
        running = [r for r in running if r.generated < r.output_len]
        if not running:
            if not plan:
                raise RuntimeError("a prompt does not fit the KV capacity on its own")
            now = last_finish
            continue
        res.phase_switches += 1
        # ---------------- decode phase, entered compactly (Sec. 3.1: phase switches leave minimal
        # bubbles): a batch starts as soon as stage 0 is free and every request in it has the token its
        # prefill produced, so the batches of older requests follow the last prefills through the pipeline
        ws = WorkStealing(n, [r.rid for r in running])
        compositions = [list(b) for b in ws.batches]
        returns: List[Tuple[float, int]] = []  # (return time, batch) of the steps in flight
        for i in range(n):
            if compositions[i]:
                ready = max([now] + [ready_at.get(rid, 0.0) for rid in compositions[i]])
                returns.append((run_batch(max(ready, stage_free[0]), interp_time(decode_profile, len(compositions[i]))), i))
        draining = False
        t_switch = 0.0
        while returns:
            returns.sort()
            t_ret, i = returns.pop(0)
            now = t_ret
            step_ms = interp_time(decode_profile, len(compositions[i]))
            finished = []
            for rid in compositions[i]:
                r = by_id[rid]
                r.generated += 1
                res.generated_tokens += 1
                if r.generated >= r.output_len:
                    finished.append(rid)
            res.peak_kv_tokens = max(res.peak_kv_tokens, kv_tokens())
            running = [r for r in running if r.rid not in set(finished)]
            # memory overflow: the most recently admitted request of this batch is recomputed later
            evicted = []
            while kv_tokens() > cfg.kv_capacity:
                cand = [rid for rid in compositions[i] if rid not in finished and rid not in evicted]
                if not cand:
                    break
                victim = by_id[cand[-1]]
                evicted.append(victim.rid)
                running = [r for r in running if r.rid != victim.rid]
                victim.input_len += victim.generated
                victim.output_len -= victim.generated
                victim.predict_len = max(victim.predict_len - victim.generated, 1)
                victim.generated = 0
                waiting.insert(0, victim)
                res.recomputes += 1
            gone = finished + evicted
            if cfg.work_stealing:
                compositions[i] = ws.on_return(i, gone)
            else:
                ws.batches[i] = [rid for rid in ws.batches[i] if rid not in set(gone)]
                compositions[i] = list(ws.batches[i])
            res.events.append(("decode", t_ret, i, len(compositions[i])))
            if draining:
                continue
            if cfg.intensity_switch and waiting and running:
                pending = plan_prefill(waiting, running, cfg)
                pend_ms = [interp_time(prefill_profile, sum(waiting[p].input_len for p in b)) for b in pending]
                size = len(compositions[i])
                if pend_ms and size > 0 and switch_to_prefill(decode_profile, size, pend_ms, step_ms, n,
                                                               cfg.count_decode_steps):
                    draining = True  # the steps in flight come back, nothing is resubmitted
                    t_switch = t_ret
                    res.events.append(("switch_to_prefill", t_ret, size, len(pend_ms)))
                    continue
            if compositions[i]:
                returns.append((run_batch(t_ret, interp_time(decode_profile, len(compositions[i]))), i))
            # a batch that ran empty earlier is revived as soon as withheld requests exist
            if cfg.work_stealing:
                in_flight = {b for _, b in returns}
                for k in range(n):
                    if k not in in_flight and ws.withheld:
                        compositions[k] = ws.on_return(k, [])
                        if compositions[k]:
                            returns.append((run_batch(t_ret, interp_time(decode_profile, len(compositions[k]))), k))
        if draining:
            res.phase_switches += 1
            # the prefills enter stage 0 behind the steps still in flight instead of waiting for them to
            # return: the bubble of the switch is the mismatch of step times (Sec. 3.5), not a drained pipeline
            now = t_switch
        # every request still alive (in a batch or withheld) is carried into the next phase
    res.total_ms = max(stage_free)
    return res


def bubble_ratio(res: SimResult, n_stages: int) -> float:
    """Share of stage time spent idle between time 0 and the end of the run."""
    return 1.0 - res.busy_ms / (n_stages * res.total_ms) if res.total_ms > 0 else 0.0

"""The executor interface of the scheduling library (tdp_simulate_exec): the run takes the oracle's
decisions and hands every batch to the caller.  No GPU: the callbacks here only keep books, and the
books are checked against what the method fixes (every request is prefilled, decoded one token at
a time from the position its prefill left it at, released exactly once when its last token is out,
re-prefilled with its generated tokens after an eviction) and against the oracle's event list."""
import math

import numpy as np
import pytest

from oracle import sched_oracle as S
from paper_2506_10470_amd import tdp_sched as L

DEC = [(1, 1.0), (8, 1.2), (32, 2.0), (128, 5.5)]
PRE = [(16, 1.0), (256, 8.0), (2048, 60.0)]


def requests(n, seed, max_in=40, max_out=30):
    rng = np.random.default_rng(seed)
    return [(int(rng.integers(4, max_in)), int(rng.integers(1, max_out)), int(rng.integers(1, max_out)))
            for _ in range(n)]


class Books:
    """What a worker would hold, without the compute: positions, pages, token counts."""

    def __init__(self, reqs, capacity_tokens):
        self.reqs = reqs
        self.cached = {}                       # request -> tokens in the cache
        self.have = [0] * len(reqs)            # tokens generated so far (over all its lives)
        self.prompt_now = [r[0] for r in reqs]  # prompt length of the current life
        self.released = [0] * len(reqs)
        self.prefills = [0] * len(reqs)
        self.evictions = [0] * len(reqs)
        self.free_pages = math.ceil(capacity_tokens / 16) + len(reqs)
        self.min_free = self.free_pages
        self.pages = {}
        self.log = []

    def _pages(self, rid, need):
        extra = need - self.pages.get(rid, 0)
        if extra > 0:
            self.free_pages -= extra
            assert self.free_pages >= 0, "ran out of pages"
            self.min_free = min(self.min_free, self.free_pages)
            self.pages[rid] = need

    def prefill(self, ids, lens):
        self.log.append(("prefill", len(ids), sum(lens)))
        for rid, n in zip(ids, lens):
            assert rid not in self.cached, "prefilled while resident"
            assert n == self.reqs[rid][0] + self.have[rid], "a re-prefill covers the prompt and everything generated"
            self.cached[rid] = n
            self._pages(rid, math.ceil(n / 16))
            self.have[rid] += 1
            self.prefills[rid] += 1

    def decode(self, batch, ids, ctx):
        self.log.append(("decode", batch, len(ids)))
        assert len(set(ids)) == len(ids)
        for rid, c in zip(ids, ctx):
            assert self.cached[rid] == c, "the step appends at the position the cache ends at"
            self.cached[rid] = c + 1
            self._pages(rid, c // 16 + 1)
            self.have[rid] += 1

    def release(self, ids, reason):
        for rid in ids:
            del self.cached[rid]
            self.free_pages += self.pages.pop(rid)
            if reason == 0:
                assert self.have[rid] == self.reqs[rid][1], "released when the last token is out, not before or after"
                self.released[rid] += 1
            else:
                assert self.have[rid] < self.reqs[rid][1]
                self.evictions[rid] += 1


@pytest.mark.parametrize("n_stages,capacity,flags", [(1, 4000, (1, 1, 1)), (2, 600, (1, 1, 1)), (4, 900, (1, 1, 1)),
                                                     (3, 700, (0, 1, 1)), (2, 650, (1, 0, 1)), (4, 2500, (1, 1, 0))])
def test_executor_sees_a_consistent_schedule_and_the_oracles_events(n_stages, capacity, flags):
    reqs = requests(80, 10 * n_stages + capacity)
    cfg = L.SimConfig(n_stages, capacity, 128, flags[0], flags[1], flags[2], 1)
    books = Books(reqs, capacity)
    res, ev = L.tdp_simulate_exec(cfg, reqs, DEC, PRE, books.prefill, books.decode, books.release, events_cap=1 << 20)
    ref = S.simulate(reqs, S.SimConfig(n_stages, capacity, 128, bool(flags[0]), bool(flags[1]), bool(flags[2]), True),
                     DEC, PRE)
    assert [(k, a, b) for k, _, a, b in ev] == [(k, a, b) for k, _, a, b in ref.events]
    assert np.allclose([t for _, t, _, _ in ev], [t for _, t, _, _ in ref.events], rtol=0, atol=1e-9)
    # the callbacks are the prefill and decode events, in order (prefill: number of prompts; decode: batch index)
    assert [e[:2] for e in books.log] == [(k, a) for k, _, a, _ in ev if k != "switch_to_prefill"]
    assert [e[2] for e in books.log if e[0] == "prefill"] == [b for k, _, _, b in ev if k == "prefill"]
    assert not books.cached and not books.pages                                  # everything was released
    assert books.released == [1] * len(reqs)
    assert [p - e for p, e in zip(books.prefills, books.evictions)] == [1] * len(reqs)
    assert books.have == [r[1] for r in reqs]
    assert sum(books.evictions) == res.recomputes == ref.recomputes
    assert res.generated_tokens == sum(r[1] for r in reqs)
    assert books.min_free >= 0


def test_memory_tight_run_evicts_and_recomputes():
    reqs = requests(60, 3)
    cfg = L.SimConfig(2, 600, 128, 1, 1, 1, 1)
    books = Books(reqs, 600)
    res, _ = L.tdp_simulate_exec(cfg, reqs, DEC, PRE, books.prefill, books.decode, books.release)
    assert res.recomputes > 0 and sum(books.evictions) == res.recomputes


def test_without_callbacks_it_is_the_plain_simulation():
    reqs = requests(50, 5)
    cfg = L.SimConfig(3, 800, 128, 1, 1, 1, 1)
    a, ev_a = L.tdp_simulate(cfg, reqs, DEC, PRE, events_cap=1 << 16)
    b, ev_b = L.tdp_simulate_exec(cfg, reqs, DEC, PRE, events_cap=1 << 16)
    assert ev_a == ev_b and a.total_ms == b.total_ms and a.generated_tokens == b.generated_tokens


def test_an_exception_in_a_callback_stops_the_run_and_comes_back():
    reqs = requests(30, 7)
    cfg = L.SimConfig(2, 2000, 128, 1, 1, 1, 1)
    calls = []

    def decode(batch, ids, ctx):
        calls.append(batch)
        if len(calls) == 3:
            raise KeyError("stop here")

    with pytest.raises(KeyError):
        L.tdp_simulate_exec(cfg, reqs, DEC, PRE, decode=decode)
    assert len(calls) == 3
    assert L.lib.tdp_simulate_exec(None, None, None, None, 0, None, None, 0, None, None, 0, None, None, 0, None) == L.EINVAL

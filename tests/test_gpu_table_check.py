"""The optional validation of device-side tables (tdp_stage_check_decode / tdp_stage_check_prefill):
tables that the parity tests run with pass, and each kind of page-allocation mistake is reported as
TDP_EINVAL with the offending row - by kernels that stay in bounds whatever the tables hold, so that
no invalid table ever reaches the stage itself.  Integer work: the verdicts are exact."""
import numpy as np
import pytest
import torch

from harness import workload as W
from harness.runner import Stage, i32

pytestmark = pytest.mark.gpu

MAX_PPS, NUM_PAGES = 8, 40


@pytest.fixture(scope="module")
def stage():
    from paper_2506_10470_amd import tdp
    sh = W.SHAPES["tiny"]
    with Stage(tdp, sh, num_pages=NUM_PAGES, max_batch=6, max_tokens=256, max_seqs=6, max_pages_per_seq=MAX_PPS,
               load_weights=False) as st:
        yield tdp, st


def tables_for(lengths):
    """Disjoint pages, dealt in order; unused entries hold a wild value on purpose: never read."""
    t = np.full((len(lengths), MAX_PPS), 10 ** 9, dtype=np.int32)
    nxt = 0
    for r, n in enumerate(lengths):
        k = (n + 15) // 16
        t[r, :k] = np.arange(nxt, nxt + k)
        nxt += k
    assert nxt <= NUM_PAGES
    return t


def decode_verdict(tdp, st, ctx, tables):
    try:
        tdp.tdp_stage_check_decode(st.h, i32(ctx), i32(tables), len(ctx))
        return None
    except tdp.TdpError as e:
        assert e.code == tdp.EINVAL
        return str(e)


def prefill_verdict(tdp, st, lens, tables, total=None):
    cu = np.zeros(len(lens) + 1, dtype=np.int64)
    cu[1:] = np.cumsum(lens)
    try:
        tdp.tdp_stage_check_prefill(st.h, i32(cu), i32(tables), len(lens), int(cu[-1]) if total is None else total)
        return None
    except tdp.TdpError as e:
        assert e.code == tdp.EINVAL
        return str(e)


CTX = [0, 15, 16, 47, 100, 127]          # a first token, page ends, a new page, the longest a row holds


def test_valid_decode_tables_pass_and_unused_entries_are_never_read(stage):
    tdp, st = stage
    assert decode_verdict(tdp, st, CTX, tables_for([c + 1 for c in CTX])) is None
    # read-only pages may be shared (a common prefix): rows 3 and 4 share their first two pages
    t = tables_for([c + 1 for c in CTX])
    t[4, :2] = t[3, :2]
    assert decode_verdict(tdp, st, CTX, t) is None


def test_decode_context_that_does_not_fit_a_row_is_reported(stage):
    tdp, st = stage
    for bad in (128, -1, 2 ** 31 - 1, -2 ** 31):
        ctx = list(CTX)
        ctx[2] = bad
        msg = decode_verdict(tdp, st, ctx, tables_for([c + 1 for c in CTX]))
        assert msg and "row 2" in msg and "length" in msg, (bad, msg)


def test_decode_page_outside_the_pool_is_reported(stage):
    tdp, st = stage
    for bad in (NUM_PAGES, -1, 10 ** 9):
        t = tables_for([c + 1 for c in CTX])
        t[4, 3] = bad
        msg = decode_verdict(tdp, st, CTX, t)
        assert msg and "row 4" in msg and "page id" in msg, (bad, msg)


def test_decode_two_requests_appending_into_one_page_is_reported(stage):
    tdp, st = stage
    t = tables_for([c + 1 for c in CTX])
    t[5, 127 // 16] = t[1, 0]            # row 5 would append where row 1 appends
    msg = decode_verdict(tdp, st, CTX, t)
    assert msg and "appears more than once" in msg and ("row 1" in msg or "row 5" in msg), msg


def test_decode_reading_a_page_another_request_appends_to_is_reported(stage):
    tdp, st = stage
    t = tables_for([c + 1 for c in CTX])
    t[4, 0] = t[0, 0]                    # row 4 reads the page row 0 writes its first token into
    msg = decode_verdict(tdp, st, CTX, t)
    assert msg and "row 4" in msg and "appears more than once" in msg, msg
    t = tables_for([c + 1 for c in CTX])
    t[4, 1] = t[4, 100 // 16]            # a request's own append page listed twice
    msg = decode_verdict(tdp, st, CTX, t)
    assert msg and "row 4" in msg, msg


def test_the_first_offending_row_is_named_and_all_are_counted(stage):
    tdp, st = stage
    t = tables_for([c + 1 for c in CTX])
    t[3, 0] = -5
    t[5, 2] = NUM_PAGES + 7
    msg = decode_verdict(tdp, st, CTX, t)
    assert msg and msg.count("row 3") == 1 and "2 table violation" in msg, msg


LENS = [1, 16, 17, 33, 128, 40]


def test_valid_prefill_tables_pass(stage):
    tdp, st = stage
    assert prefill_verdict(tdp, st, LENS, tables_for(LENS)) is None
    assert prefill_verdict(tdp, st, [5, 0, 7], tables_for([5, 0, 7])) is None     # an empty prompt writes nothing


def test_prefill_lengths_and_prefix_sums_are_checked(stage):
    tdp, st = stage
    t = tables_for(LENS)
    msg = prefill_verdict(tdp, st, [1, 16, 129, 33, 20, 40], t)                      # 129 tokens > 8 pages
    assert msg and "row 2" in msg and "length" in msg, msg
    # decreasing prefix sums: a negative length
    cu = np.array([0, 10, 5, 30], dtype=np.int32)
    with pytest.raises(tdp.TdpError) as e:
        tdp.tdp_stage_check_prefill(st.h, i32(cu), i32(tables_for([10, 1, 25])), 3, 30)
    assert "row 1" in str(e.value) and "length" in str(e.value)
    # ends of cu_seqlens
    msg = prefill_verdict(tdp, st, LENS, t, total=sum(LENS) + 1)
    assert msg and "cu_seqlens" in msg, msg
    cu = np.array([3, 10, 20], dtype=np.int32)
    with pytest.raises(tdp.TdpError) as e:
        tdp.tdp_stage_check_prefill(st.h, i32(cu), i32(tables_for([7, 10])), 2, 20)
    assert "cu_seqlens" in str(e.value)


def test_prefill_pages_must_be_distinct_and_inside_the_pool(stage):
    tdp, st = stage
    t = tables_for(LENS)
    t[4, 7] = t[2, 1]                    # two prompts writing one page
    msg = prefill_verdict(tdp, st, LENS, t)
    assert msg and "appears more than once" in msg, msg
    t = tables_for(LENS)
    t[3, 2] = t[3, 0]                    # one prompt listing a page twice
    msg = prefill_verdict(tdp, st, LENS, t)
    assert msg and "row 3" in msg and "appears more than once" in msg, msg
    t = tables_for(LENS)
    t[5, 1] = NUM_PAGES
    msg = prefill_verdict(tdp, st, LENS, t)
    assert msg and "row 5" in msg and "page id" in msg, msg


def test_limits_are_those_of_the_guarded_call(stage):
    tdp, st = stage
    z = i32(np.zeros(64))
    for call in (lambda: tdp.tdp_stage_check_decode(st.h, z, z, 7),
                 lambda: tdp.tdp_stage_check_prefill(st.h, z, z, 7, 10),
                 lambda: tdp.tdp_stage_check_prefill(st.h, z, z, 2, 257),
                 lambda: tdp.tdp_stage_check_decode(st.h, None, z, 2)):
        with pytest.raises(tdp.TdpError) as e:
            call()
        assert e.value.code == tdp.EINVAL
    tdp.tdp_stage_check_decode(st.h, None, None, 0)             # empty batches: nothing to check
    tdp.tdp_stage_check_prefill(st.h, None, None, 0, 0)


def test_random_tables_agree_with_a_host_reference(stage):
    """Random tables with random mistakes: the verdict (valid or not) equals a plain host check."""
    tdp, st = stage
    rng = np.random.default_rng(250610470)
    n_bad = 0
    for trial in range(40):
        B = int(rng.integers(1, 7))
        ctx = rng.integers(0, 128, size=B)
        t = tables_for([int(c) + 1 for c in ctx])
        if rng.random() < 0.7:                       # plant something in an entry the call uses
            r = int(rng.integers(0, B))
            j = int(rng.integers(0, int(ctx[r]) // 16 + 1))
            r2 = int(rng.integers(0, B))
            kind = int(rng.integers(0, 4))
            t[r, j] = [-1, NUM_PAGES, t[r2, int(ctx[r2]) // 16], t[r2, 0]][kind]
        ok = True
        writes = {}
        for r in range(B):
            k = int(ctx[r]) // 16
            if not (0 <= t[r, k] < NUM_PAGES) or t[r, k] in writes:
                ok = False
            writes[t[r, k]] = r
        for r in range(B):
            for j in range(int(ctx[r]) // 16):
                if not (0 <= t[r, j] < NUM_PAGES) or t[r, j] in writes:
                    ok = False
        got = decode_verdict(tdp, st, ctx, t)
        assert (got is None) == ok, (trial, ctx, t, got)
        n_bad += not ok
    assert 5 < n_bad < 40
    torch.cuda.synchronize()

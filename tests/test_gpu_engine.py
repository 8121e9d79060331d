"""The scheduling decisions driving the stage library on one GPU: a StageWorker executes the schedule
of tdp_simulate_exec (prefill batches, decode steps of the pipeline's batches, evictions) with the
HIP kernels, from token ids to token ids.

Checked here: the run takes exactly the oracle's decisions (event list); every request ends up
with exactly its output length in tokens, also when it was evicted and recomputed on the way; all
pages come back; and the first token of sampled requests is the oracle's greedy choice for that
prompt (a floating-point decision: it must be the oracle's token wherever the oracle's two best
logits are further apart than the logits tolerance, else one of the near-ties).  Later tokens
depend on earlier GPU choices and are not compared with the oracle; instead a request that ran
inside mixed batches must produce the same first tokens as the same request run on its own."""
import numpy as np
import pytest
import torch

from harness import workload as W
from oracle import ends_oracle as E
from oracle import sched_oracle as S
from oracle import stage_oracle as O
from paper_2506_10470_amd import tdp
from paper_2506_10470_amd import tdp_sched as L
from paper_2506_10470_amd.engine import StageWorker
from stage_helpers import Stage, f64, oracle_layers, oracle_shape
from test_gpu_ends import Ends, check_tokens

pytestmark = pytest.mark.gpu

DEC = [(1, 1.0), (8, 1.2), (32, 2.0), (128, 5.5)]
PRE = [(16, 1.0), (256, 8.0), (2048, 60.0)]
VOCAB = 512


def make_requests(n, seed):
    rng = np.random.default_rng(seed)
    reqs = [(int(rng.integers(4, 40)), int(rng.integers(1, 24)), int(rng.integers(1, 24))) for _ in range(n)]
    prompts = [W.token_ids(VOCAB, r[0], 100 + i) for i, r in enumerate(reqs)]
    return reqs, prompts


def run_engine(sh, reqs, prompts, n_stages, capacity, budget=128, check_tables=True):
    max_len = max(r[0] + r[1] for r in reqs) + 1
    max_pps = (max_len + 15) // 16 + 1
    num_pages = (capacity + 15) // 16 + len(reqs)
    with Stage(tdp, sh, num_pages, len(reqs), max(budget, max_len), len(reqs), max_pps) as st, \
            Ends(sh, VOCAB, max(budget, max_len, len(reqs))) as ends:
        st.poison()
        w = StageWorker(tdp, st.h, ends.h, sh.d_model, num_pages, max_pps, len(reqs), max(budget, max_len), len(reqs),
                        prompts, check_tables=check_tables)   # every call's tables are validated on the GPU first
        cfg = L.SimConfig(n_stages, capacity, budget, 1, 1, 1, 1)
        res, ev = w.run(L, cfg, reqs, DEC, PRE, events_cap=1 << 20)
        torch.cuda.synchronize()
        return w, res, ev


@pytest.mark.parametrize("shape,n_stages,capacity", [("tiny", 2, 600), ("tiny_gqa", 3, 2500)])
def test_worker_executes_the_oracles_schedule_with_real_kernels(shape, n_stages, capacity):
    sh = W.SHAPES[shape]
    reqs, prompts = make_requests(40, 11)
    w, res, ev = run_engine(sh, reqs, prompts, n_stages, capacity)
    ref = S.simulate(reqs, S.SimConfig(n_stages, capacity, 128, True, True, True, True), DEC, PRE)
    assert [(k, a, b) for k, _, a, b in ev] == [(k, a, b) for k, _, a, b in ref.events]
    assert [len(g) for g in w.generated] == [r[1] for r in reqs]
    assert all(0 <= t < VOCAB for g in w.generated for t in g)
    assert len(w.free_pages) == w.num_pages and sorted(w.free_pages) == list(range(w.num_pages)) and not w.pages
    assert w.stats["released"] == len(reqs) and w.stats["evicted"] == res.recomputes == ref.recomputes
    assert w.stats["prefill_tokens"] == res.prefill_tokens
    assert w.stats["decode_tokens"] == res.generated_tokens - (len(reqs) + res.recomputes)
    if capacity == 600:
        assert res.recomputes > 0 and res.phase_switches > 2      # the tight run really evicts and switches
    # first token of sampled requests against the oracle's logits for that prompt
    layers = list(oracle_layers(sh))
    table, head, gain = f64(w_ends_table(sh)), f64(w_ends_head(sh)), f64(w_ends_gain(sh))
    sample = [0, 7, 19, 39]
    ref_logits = []
    for i in sample:
        x = E.embed(prompts[i], table)
        out, _ = O.stage_forward(x, None, layers, oracle_shape(sh))
        ref_logits.append(E.final_logits(out[-1:], gain, head, sh.rms_eps)[0])
    check_tokens([w.generated[i][0] for i in sample], np.stack(ref_logits))


def test_a_pipeline_of_two_stages_on_one_gpu_generates_the_models_tokens():
    """The worker runs a chain of stages (one layer each here) on every batch, as the stages of a
    pipeline would on their GPUs: same decisions, same page accounting, and the first tokens are the
    oracle's for the whole two-layer model."""
    sh = W.SHAPES["tiny_gqa"]
    one = sh.with_layers(1)
    reqs, prompts = make_requests(24, 7)
    n_stages, capacity, budget = 2, 700, 128
    max_len = max(r[0] + r[1] for r in reqs) + 1
    max_pps = (max_len + 15) // 16 + 1
    num_pages = (capacity + 15) // 16 + len(reqs)
    rows = max(budget, max_len, len(reqs))
    with Stage(tdp, one, num_pages, len(reqs), rows, len(reqs), max_pps) as s0, \
            Stage(tdp, one, num_pages, len(reqs), rows, len(reqs), max_pps, layer_offset=1) as s1, \
            Ends(sh, VOCAB, rows) as ends:
        s0.poison()
        s1.poison()
        w = StageWorker(tdp, [s0.h, s1.h], ends.h, sh.d_model, num_pages, max_pps, len(reqs), rows, len(reqs), prompts,
                        check_tables=True)
        res, ev = w.run(L, L.SimConfig(n_stages, capacity, budget, 1, 1, 1, 1), reqs, DEC, PRE, events_cap=1 << 20)
        torch.cuda.synchronize()
    ref = S.simulate(reqs, S.SimConfig(n_stages, capacity, budget, True, True, True, True), DEC, PRE)
    assert [(k, a, b) for k, _, a, b in ev] == [(k, a, b) for k, _, a, b in ref.events]
    assert [len(g) for g in w.generated] == [r[1] for r in reqs]
    assert sorted(w.free_pages) == list(range(num_pages)) and not w.pages
    layers = list(oracle_layers(sh))          # both layers of the model
    table, head, gain = f64(w_ends_table(sh)), f64(w_ends_head(sh)), f64(w_ends_gain(sh))
    sample = [0, 5, 13, 23]
    ref_logits = []
    for i in sample:
        x = E.embed(prompts[i], table)
        out, _ = O.stage_forward(x, None, layers, oracle_shape(sh))
        ref_logits.append(E.final_logits(out[-1:], gain, head, sh.rms_eps)[0])
    check_tokens([w.generated[i][0] for i in sample], np.stack(ref_logits))


def w_ends_table(sh):
    return W.ends_weight(sh, "embedding", VOCAB, device="cuda")


def w_ends_head(sh):
    return W.ends_weight(sh, "lm_head", VOCAB, device="cuda")


def w_ends_gain(sh):
    return W.ends_weight(sh, "final_norm", VOCAB, device="cuda", dtype=torch.float32)


def test_a_request_generates_the_same_tokens_alone_and_inside_mixed_batches():
    """Batch composition, paging and eviction must not change what a request computes beyond
    rounding: its first tokens in the 40-request run equal those of a run that holds it alone
    (compared up to the first position where the two runs' own choices diverge by a near-tie,
    which the tolerance of the logits allows; the first two tokens are required to agree)."""
    sh = W.SHAPES["tiny"]
    reqs, prompts = make_requests(40, 11)
    w, _, _ = run_engine(sh, reqs, prompts, 2, 600)
    agree = []
    for i in (3, 12, 25):
        solo, _, _ = run_engine(sh, [reqs[i]], [prompts[i]], 1, 4000)
        a, b = w.generated[i], solo.generated[0]
        assert len(a) == len(b) == reqs[i][1]
        same = 0
        while same < len(a) and a[same] == b[same]:
            same += 1
        agree.append(same / len(a))
        assert same >= min(2, len(a)), (i, a, b)
    assert np.mean(agree) > 0.5, agree


def test_worker_refuses_a_schedule_it_cannot_hold():
    sh = W.SHAPES["tiny"]
    reqs, prompts = make_requests(8, 5)
    with Stage(tdp, sh, 4, 8, 128, 8, 8) as st, Ends(sh, VOCAB, 128) as ends:
        w = StageWorker(tdp, st.h, ends.h, sh.d_model, 4, 8, 8, 128, 8, prompts)       # 4 pages: far too few
        from paper_2506_10470_amd.engine import OutOfPages
        with pytest.raises(OutOfPages):
            w.run(L, L.SimConfig(2, 4000, 128, 1, 1, 1, 1), reqs, DEC, PRE)
        torch.cuda.synchronize()

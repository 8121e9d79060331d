"""A worker that runs what the scheduling library decides: the executor side of tdp_simulate_exec.

The paper's engine tells each worker which batch to run in which phase (Sec. 3.2); the decisions are
those of Sec. 3.3 - 3.5 (libtdp_sched.so).  This module is the worker for ONE GPU: it owns the page
allocation (the engine's job, Sec. 3.2.1), turns each event of the schedule into calls of the stage
library (token embedding -> tdp_stage_prefill / tdp_stage_decode -> final norm + vocabulary
projection + greedy selection) and keeps every request's tokens.  The pipeline clock of the
schedule still comes from the profiles handed to the scheduler; the work itself is done by the HIP
kernels, on the stream the caller names.  Host logic only: no arithmetic of the method lives here.
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

import numpy as np
import torch

PAGE = 16


class OutOfPages(RuntimeError):
    pass


class StageWorker:
    """Executes prefill / decode / release events on a stage (tdp_stage) and a pair of pipeline ends
    (tdp_ends) that the caller created and loaded.  `prompts[i]` are request i's prompt token ids.
    `stage` may also be a sequence of stage handles: the stages of a pipeline held by one GPU, run one
    after the other on every batch (hidden states handed from each to the next as bf16, the pipeline's
    hand-over format, Sec. 2.2.3); they share the block tables, every stage owning its own pools of
    `num_pages` pages."""

    def __init__(self, tdp, stage: int, ends: int, d_model: int, num_pages: int, max_pages_per_seq: int,
                 max_batch: int, max_tokens: int, max_seqs: int, prompts: Sequence[Sequence[int]], stream=None,
                 check_tables: bool = False):
        """check_tables: validate every call's block tables on the GPU first (tdp_stage_check_*): one
        synchronisation per call, for runs that test the allocator rather than the throughput."""
        self.tdp, self.ends = tdp, ends
        self.stages = [stage] if isinstance(stage, int) else list(stage)
        self.stage = self.stages[0]
        self.d_model = d_model
        self.max_pps, self.max_batch, self.max_tokens, self.max_seqs = max_pages_per_seq, max_batch, max_tokens, max_seqs
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        self.free_pages: List[int] = list(range(num_pages - 1, -1, -1))
        self.num_pages = num_pages
        self.check_tables = check_tables
        self.pages: Dict[int, List[int]] = {}
        self.prompts = [list(map(int, p)) for p in prompts]
        self.generated: List[List[int]] = [[] for _ in prompts]
        rows = max(max_batch, max_tokens, 1)
        self.hidden = torch.empty((rows, d_model), dtype=torch.bfloat16, device="cuda")
        self.hidden_out = torch.empty_like(self.hidden)
        self.next_tok = torch.empty(max(max_batch, max_seqs, 1), dtype=torch.int32, device="cuda")
        self.stats = {"prefill_batches": 0, "prefill_tokens": 0, "decode_steps": 0, "decode_tokens": 0,
                      "released": 0, "evicted": 0, "min_free_pages": num_pages}

    # ---- pages
    def _take(self, n: int) -> List[int]:
        if n > len(self.free_pages):
            raise OutOfPages("need %d pages, %d free" % (n, len(self.free_pages)))
        got = [self.free_pages.pop() for _ in range(n)]
        self.stats["min_free_pages"] = min(self.stats["min_free_pages"], len(self.free_pages))
        return got

    def _table(self, ids: Sequence[int]) -> torch.Tensor:
        t = np.zeros((len(ids), self.max_pps), dtype=np.int32)
        for k, rid in enumerate(ids):
            p = self.pages[rid]
            t[k, :len(p)] = p
        return torch.from_numpy(t).cuda()

    @staticmethod
    def _i32(a) -> torch.Tensor:
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()

    # ---- the three events
    def prefill(self, ids: List[int], lens: List[int]) -> None:
        n, total = len(ids), int(sum(lens))
        if n > self.max_seqs or total > self.max_tokens:
            raise ValueError("prefill batch of %d prompts / %d tokens exceeds the stage's limits" % (n, total))
        toks: List[int] = []
        for rid, L in zip(ids, lens):
            seq = self.prompts[rid] + self.generated[rid]
            if len(seq) != L:
                raise ValueError("request %d: schedule says %d tokens, worker holds %d" % (rid, L, len(seq)))
            if rid in self.pages:
                raise ValueError("request %d is prefilled while it still holds pages" % rid)
            if (L + PAGE - 1) // PAGE > self.max_pps:
                raise ValueError("request %d does not fit a block-table row" % rid)
            self.pages[rid] = self._take((L + PAGE - 1) // PAGE)
            toks += seq
        cu = np.zeros(n + 1, dtype=np.int32)
        cu[1:] = np.cumsum(lens)
        tdp = self.tdp
        x, y = self.hidden[:total], self.hidden_out[:total]
        cu_dev, table = self._i32(cu), self._table(ids)
        if self.check_tables:
            tdp.tdp_stage_check_prefill(self.stage, cu_dev, table, n, total, self.stream)
        tdp.tdp_embed_tokens(self.ends, self._i32(toks), total, x, self.stream)
        for st in self.stages:
            tdp.tdp_stage_prefill(st, x, cu_dev, table, n, total, y, self.stream)
            x, y = y, x
        y = x
        tdp.tdp_lm_head(self.ends, y, total, self._i32(cu[1:] - 1), n, None, self.next_tok[:n], self.stream)
        for rid, t in zip(ids, self.next_tok[:n].cpu().tolist()):
            self.generated[rid].append(int(t))
        self.stats["prefill_batches"] += 1
        self.stats["prefill_tokens"] += total

    def decode(self, batch: int, ids: List[int], contexts: List[int]) -> None:
        n = len(ids)
        if n == 0:
            return
        if n > self.max_batch:
            raise ValueError("decode batch of %d exceeds the stage's max_batch %d" % (n, self.max_batch))
        for rid, ctx in zip(ids, contexts):
            if ctx != len(self.prompts[rid]) + len(self.generated[rid]) - 1:
                raise ValueError("request %d: schedule says %d cached tokens, worker holds %d" % (
                    rid, ctx, len(self.prompts[rid]) + len(self.generated[rid]) - 1))
            if ctx // PAGE >= self.max_pps:
                raise ValueError("request %d outgrew its block-table row" % rid)
            if ctx // PAGE >= len(self.pages[rid]):
                self.pages[rid] += self._take(1)
        tdp = self.tdp
        x, y = self.hidden[:n], self.hidden_out[:n]
        ctx_dev, table = self._i32(contexts), self._table(ids)
        if self.check_tables:
            tdp.tdp_stage_check_decode(self.stage, ctx_dev, table, n, self.stream)
        tdp.tdp_embed_tokens(self.ends, self._i32([self.generated[rid][-1] for rid in ids]), n, x, self.stream)
        for st in self.stages:
            tdp.tdp_stage_decode(st, x, ctx_dev, table, n, y, self.stream)
            x, y = y, x
        y = x
        tdp.tdp_lm_head(self.ends, y, n, None, n, None, self.next_tok[:n], self.stream)
        for rid, t in zip(ids, self.next_tok[:n].cpu().tolist()):
            self.generated[rid].append(int(t))
        self.stats["decode_steps"] += 1
        self.stats["decode_tokens"] += n

    def release(self, ids: List[int], reason: int) -> None:
        for rid in ids:
            self.free_pages.extend(reversed(self.pages.pop(rid)))
        self.stats["released" if reason == 0 else "evicted"] += len(ids)

    # ---- the run
    def run(self, sched, cfg, requests: Sequence[Tuple[int, int, int]], decode_profile, prefill_profile,
            events_cap: int = 0):
        """requests[i] = (input_len, output_len, predict_len) with input_len = len(prompts[i]).  Returns
        (SimResult, events) of the scheduling library; the tokens are in self.generated."""
        if len(requests) != len(self.prompts) or any(r[0] != len(p) for r, p in zip(requests, self.prompts)):
            raise ValueError("requests and prompts disagree")
        return sched.tdp_simulate_exec(cfg, requests, decode_profile, prefill_profile, prefill=self.prefill,
                                       decode=self.decode, release=self.release, events_cap=events_cap)

"""fp64 CPU oracle for the two ends of the pipeline: what comes before the first stage and after
the last one, so that a chain of stages emits tokens.

TEST INFRASTRUCTURE ONLY: imported by tests, never by the product path; shares no code with the
HIP kernels.

The paper runs whole models (Table 2) through its pipeline and counts generated tokens per second
(Sec. 4.1); the layer slices are the stages, and the steps on either side of them are the public
Llama-2 ones: a token-embedding lookup in front, and behind the last layer a final RMSNorm, the
vocabulary projection and - for the deterministic throughput runs - greedy selection of the next
token.  Greedy selection is the one place on the path where floating point decides an integer:
the rule here is "the lowest index among the largest logits".

Pinned by tests/test_oracle_pins.py (section "pipeline ends"): the lookup against a one-hot matrix
product, the selection against planted ties and numpy's first-occurrence argmax, the projection
against closed forms (identity head, scale invariance of the norm).
"""
from __future__ import annotations

from typing import Sequence

import numpy as np

from .stage_oracle import rmsnorm

F64 = np.float64


def embed(token_ids: Sequence[int], table: np.ndarray) -> np.ndarray:
    """Row t of the result is row token_ids[t] of the [vocab, d_model] table."""
    table = np.asarray(table, dtype=F64)
    out = np.empty((len(token_ids), table.shape[1]), dtype=F64)
    for t, tok in enumerate(token_ids):
        if not 0 <= int(tok) < table.shape[0]:
            raise IndexError("token id %d outside the vocabulary" % int(tok))
        out[t] = table[int(tok)]
    return out


def final_logits(x: np.ndarray, gain: np.ndarray, w_head: np.ndarray, eps: float) -> np.ndarray:
    """logits = RMSNorm(x; gain) @ w_head with w_head [d_model, vocab]."""
    return rmsnorm(np.asarray(x, dtype=F64), np.asarray(gain, dtype=F64), eps) @ np.asarray(w_head, dtype=F64)


def greedy_tokens(logits: np.ndarray) -> np.ndarray:
    """Per row, the lowest index among the maxima."""
    logits = np.asarray(logits)
    out = np.zeros(logits.shape[0], dtype=np.int64)
    for r in range(logits.shape[0]):
        best = 0
        for j in range(1, logits.shape[1]):
            if logits[r, j] > logits[r, best]:
                best = j
        out[r] = best
    return out

"""GPU parity on stage shapes nobody picked by hand: every legal combination of model width, head
count, GQA group, head size, FFN width (ragged tails included), bias and depth is a shape the
library accepts, so a seeded draw of them goes through prefill (ragged prompts, K/V append checked
slot by slot), decode steps on that cache and a decode batch on an imported cache, each against the
fp64 oracle at the same tolerance as the hand-picked shapes."""
import numpy as np
import pytest

from harness import workload as W
from test_gpu_parity import run_decode_case, run_prefill_case, tdp  # noqa: F401  (tdp: fixture)

pytestmark = pytest.mark.gpu

GROUPS = (1, 1, 2, 3, 4, 5, 8, 16)


def draw_shape(case: int) -> W.StageShape:
    rng = np.random.default_rng(1000 + case)
    head_dim = int(rng.choice([64, 128]))
    n_kv = int(rng.integers(1, 5))
    group = int(rng.choice(GROUPS))
    return W.StageShape(
        name=f"drawn_{case}", n_layers=int(rng.integers(1, 3)), d_model=64 * int(rng.integers(1, 13)),
        n_q_heads=n_kv * group, n_kv_heads=n_kv, head_dim=head_dim, d_ff=4 * int(rng.integers(1, 500)),
        rms_eps=float(rng.choice([1e-5, 1e-6])), rope_base=float(rng.choice([1e4, 1e6])),
        config_index=100 + case, qkv_bias=bool(rng.integers(0, 2)))


@pytest.mark.parametrize("case", range(12))
def test_drawn_shape_prefill_then_decode(tdp, case):  # noqa: F811
    sh = draw_shape(case)
    rng = np.random.default_rng(2000 + case)
    seq_lens = rng.integers(1, 330, size=int(rng.integers(1, 6)))
    err = run_prefill_case(tdp, sh, seq_lens, decode_steps=2)
    print(sh, list(seq_lens), f"{err:.2e}")


@pytest.mark.parametrize("case", range(12))
def test_drawn_shape_decode_on_an_imported_cache(tdp, case):  # noqa: F811
    sh = draw_shape(case)
    rng = np.random.default_rng(3000 + case)
    ctx = rng.integers(0, 600, size=int(rng.integers(1, 41)))
    ctx[0] = int(rng.choice([0, 15, 16, 255, 256, 511]))  # a page or span edge in every batch
    err = run_decode_case(tdp, sh, ctx, span=int(rng.choice([0, 256, 512])))
    print(sh, len(ctx), f"{err:.2e}")

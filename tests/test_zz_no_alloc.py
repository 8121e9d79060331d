"""The allocation-free projection call (tdp_gemm_bf16_static) against the allocating one
(tdp_gemm_bf16): same kernels on a scratch array that is part of the library image, so the two must
agree bit for bit, also on a second call with a smaller input that finds the first call's contents
in the array.  Runs last: it must pass alone in a fresh process and after every other test."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tdp():
    from paper_2506_10470_amd import tdp as _tdp
    return _tdp


def _operands(M, N, K, seed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    A = torch.randn(M, K, generator=g).to(torch.bfloat16).cuda()
    Wm = (torch.randn(K, N, generator=g) * 0.05).to(torch.bfloat16).cuda()
    R = torch.randn(M, N, generator=g).to(torch.bfloat16).cuda()
    return A, Wm, R


def _both(tdp, M, N, K, epi, tile, splits, seed):
    A, Wm, R = _operands(M, N, K, seed)
    want = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    tdp.tdp_gemm_bf16(A, Wm, R if epi else None, want, M, N, K, epi, tile, splits)
    got = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    tdp.tdp_gemm_bf16_static(A, Wm, R if epi else None, got, M, N, K, epi, tile, splits)
    torch.cuda.synchronize()
    ref = A.double().cpu().numpy() @ Wm.double().cpu().numpy() + (R.double().cpu().numpy() if epi else 0.0)
    return got, want, ref


def _row_rel_err(got, ref):
    got = got.double().cpu().numpy()
    return float(np.max(np.max(np.abs(got - ref), axis=-1) / np.max(np.abs(ref), axis=-1)))


def test_two_calls_in_a_row_the_second_smaller(tdp):
    # first call: several tiles, ragged M and N (padded weight rows), split-K partials in the scratch
    got, want, ref = _both(tdp, 300, 1028, 1024, 1, 0, 3, seed=1)
    assert torch.equal(got.view(torch.int16), want.view(torch.int16))
    assert _row_rel_err(got, ref) <= 1e-2
    # second call, smaller in every dimension: the scratch still holds the first call's weights and partials
    got, want, ref = _both(tdp, 70, 260, 256, 0, 0, 2, seed=2)
    assert torch.equal(got.view(torch.int16), want.view(torch.int16))
    assert _row_rel_err(got, ref) <= 1e-2
    # and the planner's own choice on a third shape
    got, want, ref = _both(tdp, 512, 1280, 2048, 1, 0, 0, seed=3)
    assert torch.equal(got.view(torch.int16), want.view(torch.int16))
    assert _row_rel_err(got, ref) <= 1e-2


def test_calls_on_one_stream_need_no_wait_in_between(tdp):
    """The call only enqueues: two calls back to back on one stream reuse the scratch in stream order."""
    A1, W1, R1 = _operands(129, 516, 512, 11)
    A2, W2, R2 = _operands(40, 256, 128, 12)
    o1 = torch.empty(129, 516, dtype=torch.bfloat16, device="cuda")
    o2 = torch.empty(40, 256, dtype=torch.bfloat16, device="cuda")
    s = torch.cuda.current_stream()
    tdp.tdp_gemm_bf16_static(A1, W1, R1, o1, 129, 516, 512, 1, 0, 2, s)
    tdp.tdp_gemm_bf16_static(A2, W2, None, o2, 40, 256, 128, 0, 0, 0, s)
    torch.cuda.synchronize()
    r1 = A1.double().cpu().numpy() @ W1.double().cpu().numpy() + R1.double().cpu().numpy()
    r2 = A2.double().cpu().numpy() @ W2.double().cpu().numpy()
    assert _row_rel_err(o1, r1) <= 1e-2 and _row_rel_err(o2, r2) <= 1e-2


def test_sizes_beyond_the_scratch_are_rejected_before_any_work(tdp):
    x = torch.zeros(16, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(tdp.TdpError) as e:      # 4096 x 4096 weights: 16 Mi elements > 8 Mi
        tdp.tdp_gemm_bf16_static(x, x, None, x, 1, 4096, 4096, 0, 0, 0)
    assert e.value.code == tdp.EINVAL and "static scratch" in str(e.value)
    with pytest.raises(tdp.TdpError) as e:      # 16 x 4096 x 256 floats of partials > 12 Mi
        tdp.tdp_gemm_bf16_static(x, x, None, x, 4096, 256, 64, 0, 0, 0)
    assert e.value.code == tdp.EINVAL and "workspace" in str(e.value)
    tdp.tdp_gemm_bf16_static(None, None, None, None, 0, 64, 64, 0, 0, 0)     # M = 0: nothing to do

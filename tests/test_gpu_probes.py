"""The machine probes behind the benchmark's empirical ceilings: they read what they say they read
(sizes, never a byte written) and return rates a GPU of this class can have."""
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tdp():
    from paper_2506_10470_amd import tdp as t
    return t


def test_hbm_read_probe_sizes_and_rates(tdp):
    buf = torch.full(((1 << 30) + 12345,), 7, dtype=torch.uint8, device="cuda")
    for scattered in (False, True):
        for nt in (False, True):
            n, ms = tdp.tdp_probe_hbm_read(buf, buf.numel(), scattered, 3, non_temporal=nt)
            assert n == 1 << 30                     # the largest 2^k * 4 KiB that fits
            gbs = n / ms / 1e6
            assert 1000.0 < gbs < 8000.0, (scattered, nt, gbs)
    n, ms = tdp.tdp_probe_hbm_read(buf, 3 << 20, True, 2)
    assert n == 2 << 20 and ms > 0
    n, ms = tdp.tdp_probe_hbm_read(buf, 512 << 10, False, 1)       # the smallest size: one workgroup
    assert n == 512 << 10
    torch.cuda.synchronize()
    assert bool((buf == 7).all())               # read-only


def test_mfma_probe_rate_is_plausible(tdp):
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    rates = {}
    for random_operands in (True, False):
        flop, ms = tdp.tdp_probe_mfma_bf16(2048, 3, random_operands)
        assert flop == cus * 2 * 4 * 2048 * 16 * 2 * 16 * 16 * 32
        rates[random_operands] = flop / ms / 1e9
        assert 500.0 < rates[random_operands] < 2600.0, rates      # published dense bf16 peak: 2.5 PFLOP/s
    assert rates[False] > 0.9 * rates[True]         # constant operands are never much slower

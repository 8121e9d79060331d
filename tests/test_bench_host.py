"""Host-side checks of bench.py that need no GPU: the multi-GPU refusal, and the scheduler section
on a fixed profile (the part of the benchmark that is pure host code)."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""           # no JSON line is printed


def test_scheduler_section_on_a_fixed_profile():
    sys.path.insert(0, ROOT)
    import bench
    from harness import workload as W
    sweep = [{"batch": b, "ms_per_step": m} for b, m in
             [(16, 8.0), (32, 8.6), (64, 9.2), (128, 11.1), (256, 15.7), (512, 26.6)]]
    curve = [{"tokens": t, "ms": m} for t, m in [(900, 30.0), (2100, 64.0), (4300, 128.0), (9000, 266.0), (17766, 523.0)]]
    out = bench.scheduler_section(W.SHAPES["70b_quarter"], sweep, curve, n_requests=3000)
    json.dumps(out)                           # serialisable
    pol = out["policies"]
    assert set(pol) == {"td_pipe", "no_greedy_prefill", "no_work_stealing", "no_intensity_switch", "none"}
    for v in pol.values():
        assert v["tok_s"] > 0 and 0 <= v["bubble_ratio"] < 1
    # every policy generates the same tokens; the full policy set is not slower than none of them
    assert pol["td_pipe"]["tok_s"] >= 0.98 * pol["none"]["tok_s"]
    assert out["kv_capacity_tokens"] > 10 ** 6


def test_scattered_order_visits_every_piece_once():
    """The device-side index scrambler is a bijection on [0, 2^bits): same integer arithmetic on the host."""
    import numpy as np
    for bits in (7, 8, 13, 18, 22):
        mask = np.uint64((1 << bits) - 1)
        g = np.arange(1 << bits, dtype=np.uint64)
        x = (g * np.uint64(0x9E3779B1)) & np.uint64(0xFFFFFFFF) & mask
        x ^= x >> np.uint64((bits + 1) // 2)
        x = (x * np.uint64(0x85EBCA6B)) & np.uint64(0xFFFFFFFF) & mask
        assert len(np.unique(x)) == 1 << bits, bits

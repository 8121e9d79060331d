#!/usr/bin/env python3
"""Benchmark of the pipeline-stage forward pass on one MI355X.

A "step" is one decode step of the whole stage (every layer: RMSNorm, QKV GEMM, RoPE + KV append,
paged attention, O GEMM, RMSNorm, gate/up GEMM + SwiGLU, down GEMM) over one synthetic batch whose
weights, hidden states, block tables and KV cache are resident in HBM before the timed region.
The default workload is the 70B-shaped quarter stage (20 layers, GQA 64/8, FFN 28672, bf16) at
decode batch 512; the same run also reports the decode batch-size sweep (the computational-
intensity curve the paper's phase-switch decision is built on, Sec. 3.5) and the prefill rate.

Prints ONE JSON line.  Only one GPU is used; --gpus above 1 is refused.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

ADVANCE_STEPS = 17             # the advancing-context run crosses a page boundary in every request
HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def build_stage(tdp, W, Stage, shape, dec_ctx, pre_lens, i32, kv_scales=None):
    """One stage sized for the decode batch and the prefill batch, page ranges disjoint."""
    import torch
    max_pps = 4096 // 16 + 2
    dec = W.make_decode_batch(dec_ctx, max_pages_per_seq=max_pps, steps=ADVANCE_STEPS + 1)
    pre = W.make_prefill_batch(pre_lens, max_pages_per_seq=max_pps)
    pre_tables = np.where(pre.tables >= 0, pre.tables + dec.num_pages, -1).astype(np.int32)
    t0 = time.time()
    st = Stage(tdp, shape, dec.num_pages + pre.num_pages, len(dec_ctx), int(pre_lens.sum()), len(pre_lens),
               max_pps, load_weights=True, kv_scales=kv_scales)
    torch.cuda.synchronize()
    log("stage created, weights loaded: %.1f s" % (time.time() - t0))
    # pre-existing KV ~ N(0,1), written through the library's import kernel
    t0 = time.time()
    total = int(dec_ctx.sum())
    cu = np.zeros(len(dec_ctx) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(dec_ctx)
    cu_d, tab_d = i32(cu), i32(dec.tables)
    for l in range(shape.n_layers):
        k = W.kv_packed(shape, l, "k", total, 1, device="cuda")
        v = W.kv_packed(shape, l, "v", total, 1, device="cuda")
        tdp.tdp_stage_kv_import(st.h, l, k, v, cu_d, tab_d, len(dec_ctx), total)
        torch.cuda.synchronize()
        del k, v
    log("KV cache filled (%d tokens x %d layers): %.1f s" % (total, shape.n_layers, time.time() - t0))
    return st, dec, pre, pre_tables, cu


def time_calls(fn, warmup, steps):
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def step_percentiles(fn, steps):
    """p10 / p50 / p90 of single-step times from events on the launch stream (torch's current stream)."""
    import torch
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    ev[0].record()
    for i in range(steps):
        fn()
        ev[i + 1].record()
    torch.cuda.synchronize()
    t = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(steps))
    pick = lambda q: round(t[min(len(t) - 1, int(q * len(t)))], 4)
    return {"p10": pick(0.10), "p50": pick(0.50), "p90": pick(0.90), "mean": round(sum(t) / len(t), 4), "steps": steps}


def time_events(fn, warmup, steps):
    """Mean and p10 / p50 / p90 of single calls, from events on the launch stream."""
    import torch
    for _ in range(warmup):
        fn()
    pct = step_percentiles(fn, steps)
    return pct


def class_times(tdp, st, fn, reps):
    """Average milliseconds per call and kernel class, from HIP events on the launch stream."""
    import torch
    tdp.tdp_stage_timing_enable(st.h, True)
    fn()
    torch.cuda.synchronize()
    acc = {}
    for _ in range(reps):
        fn()
        t = tdp.tdp_stage_timing_read(st.h)
        for k, v in t.items():
            acc[k] = acc.get(k, 0.0) + v / reps
    tdp.tdp_stage_timing_enable(st.h, False)
    return acc


def kernel_rooflines(shape, M, kv_read_bytes, attn_flops, times_ms, phase):
    """Per kernel class: algorithmic bytes and flops per stage pass, the roofline that binds it
    (HBM when flops/byte is below peak_flops/peak_bytes, else MFMA), achieved rate and fraction."""
    d, dq, dkv, F, L = shape.d_model, shape.d_q, shape.d_kv, shape.d_ff, shape.n_layers
    gemms = {"gemm_qkv": (dq + 2 * dkv, d), "gemm_o": (d, dq), "gemm_gate_up": (2 * F, d), "gemm_down": (d, F)}
    ridge = MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)
    out = {}
    for name, (N, K) in gemms.items():
        byts = L * N * K * 2
        flops = 2 * M * L * N * K
        out[name] = (byts, flops)
    out["attention"] = (kv_read_bytes, attn_flops)
    res = {}
    for name, (byts, flops) in out.items():
        ms = times_ms.get(name, 0.0)
        if ms <= 0:
            continue
        launches = L
        bound = "mfma" if (phase == "prefill" or flops / byts > ridge) else "hbm"
        if bound == "hbm":
            ach, peak, unit = byts / (ms * 1e-3) / 1e9, HBM_PEAK_GBS, "GB/s"
        else:
            ach, peak, unit = flops / (ms * 1e-3) / 1e12, MFMA_BF16_PEAK_TFLOPS, "TFLOP/s"
        res[name] = {"bound": bound, "achieved": round(ach, 1), "peak": peak, "unit": unit,
                     "frac": round(ach / peak, 4), "avg_launch_ms": round(ms / launches, 4),
                     "launches_per_step": launches, "alg_bytes_per_launch": byts // launches,
                     "alg_flops_per_launch": flops // launches, "traffic": None}
    return res


TRAFFIC_FILES = {"70b_quarter stage, decode phase, batch 512": "traffic_decode_70b_quarter_b512.json",
                 "70b_quarter stage, decode phase, batch 256": "traffic_decode_70b_quarter_b256.json"}


def measured_traffic(workload):
    """HBM bytes per launch measured with rocprofv3 TCC counters in an EARLIER run (committed under
    profiles/, see the summary there for the commands): rocprofv3 cannot run inside this process, so the
    figure is a stored one.  Returns (per-class bytes, description of where they come from)."""
    name = TRAFFIC_FILES.get(workload)
    if not name:
        return {}, None
    try:
        t = json.load(open(os.path.join(ROOT, "profiles", name)))
    except OSError:
        return {}, None
    per = t["per_launch"]
    tot = lambda *ks: sum(per[k]["fetch_bytes"] + per[k]["write_bytes"] for k in ks if k in per)
    src = "stored, not measured in this run: profiles/%s (%s; recorded %s)" % (name, t.get("source", "?"), t.get("recorded", "?"))
    return {"attention": tot("attn_decode_kernel"), "gemm_qkv": tot("gemm_qkv"),
            "gemm_o": tot("gemm_o"), "gemm_gate_up": tot("gemm_gate_up"), "gemm_down": tot("gemm_down")}, src


def cpu_baseline(shape, dec_ctx, cu, budget_layers=4, n_requests=64):
    """The fp64 oracle, as it stands, on a bounded sample of the decode workload: `n_requests`
    requests spread evenly over the batch sorted by context length (shortest and longest included)
    through the first `budget_layers` layers, scaled to the full layer count.  Weight generation /
    widening to fp64 is input preparation and is not timed."""
    import torch
    from threadpoolctl import threadpool_info
    from harness import workload as W
    from oracle import stage_oracle as O
    order = np.argsort(dec_ctx, kind="stable")
    budget_layers = min(budget_layers, shape.n_layers)
    picks = np.unique(np.linspace(0, len(order) - 1, min(n_requests, len(order))).round().astype(int))
    sample = [int(order[i]) for i in picks]
    osh = O.Shape(shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.rms_eps, shape.rope_base)
    t_prep = time.time()
    layers = []
    for l in range(budget_layers):
        ws = []
        for name in W.WEIGHT_NAMES:
            w = W.weight(shape, l, name, device="cuda")
            if not name.startswith("g_"):
                w = w.to(torch.bfloat16)
            ws.append(w.cpu().to(torch.float64).numpy())
        layers.append(O.LayerWeights(*ws))
    total = int(dec_ctx.sum())
    caches = []
    for b in sample:
        c = []
        for l in range(budget_layers):
            k = W.kv_packed(shape, l, "k", total, 1, device="cuda", tok0=int(cu[b]), toks=int(dec_ctx[b]))
            v = W.kv_packed(shape, l, "v", total, 1, device="cuda", tok0=int(cu[b]), toks=int(dec_ctx[b]))
            c.append((k.cpu().to(torch.float64).numpy(), v.cpu().to(torch.float64).numpy()))
        caches.append(c)
    x = W.hidden_states(shape, len(dec_ctx), 1, device="cuda").cpu().to(torch.float64).numpy()
    t_prep = time.time() - t_prep
    t0 = time.perf_counter()
    O.stage_decode([x[b] for b in sample], caches, layers, osh)
    dt = time.perf_counter() - t0
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    tok_s = len(sample) / (dt * shape.n_layers / budget_layers)
    return {"value": round(tok_s, 4), "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": "decode: %d requests (ctx %d..%d, mean %.0f) x %d of %d layers, %.1f s timed, scaled by "
                      "layers; input preparation %.1f s not timed" % (
                          len(sample), min(int(dec_ctx[b]) for b in sample), max(int(dec_ctx[b]) for b in sample),
                          float(np.mean([dec_ctx[b] for b in sample])), budget_layers, shape.n_layers, dt, t_prep)}


def micro_batch_section(tdp, W, Stage, shape, dec_ctx, i32, steps, warmup):
    """The headline decode step as two half-batches on two streams (decode_micro_batches = 2), same weights,
    same cache contents; an option of the library, measured beside the one-batch form."""
    import torch
    B = len(dec_ctx)
    max_pps = 4096 // 16 + 2
    dec = W.make_decode_batch(dec_ctx, max_pages_per_seq=max_pps, steps=ADVANCE_STEPS + 1)
    st = Stage(tdp, shape, dec.num_pages, B, 0, 0, max_pps, load_weights=True, decode_micro_batches=2)
    total = int(dec_ctx.sum())
    cu = np.zeros(B + 1, dtype=np.int32)
    cu[1:] = np.cumsum(dec_ctx)
    cu_d, tab_d = i32(cu), i32(dec.tables)
    for l in range(shape.n_layers):
        k = W.kv_packed(shape, l, "k", total, 1, device="cuda")
        v = W.kv_packed(shape, l, "v", total, 1, device="cuda")
        tdp.tdp_stage_kv_import(st.h, l, k, v, cu_d, tab_d, B, total)
        torch.cuda.synchronize()
        del k, v
    stream = torch.cuda.current_stream()
    x = W.hidden_states(shape, B, 1, device="cuda")
    out = torch.empty_like(x)
    ctx_d = i32(dec.ctx_lens)
    res = {"decode_micro_batches": 2, "batches": []}
    for b in (B, B // 2):
        pb = time_events(lambda: tdp.tdp_stage_decode(st.h, x, ctx_d, tab_d, b, out, stream), warmup, max(steps, 20))
        res["batches"].append({"batch": b, "ms_per_step": pb["mean"], "ms_p10": pb["p10"], "ms_p90": pb["p90"],
                               "tok_s": round(b / pb["mean"] * 1e3, 1)})
    st.close()
    torch.cuda.empty_cache()
    return res


def fp8_kv_section(tdp, W, Stage, A, shape, sargs, dec_ctx, i32, steps, warmup):
    """The same decode step with the KV cache held as 8-bit E4M3 codes (scales 1): the cache bytes
    the step must read are halved, everything else is unchanged.  An option of the library, not the
    headline configuration (the paper keeps the cache in the model's 16-bit type)."""
    import torch
    B = len(dec_ctx)
    st, dec, _, _, _ = build_stage(tdp, W, Stage, shape, dec_ctx, np.array([16], dtype=np.int64), i32,
                                   kv_scales=(1.0, 1.0))
    stream = torch.cuda.current_stream()
    x = W.hidden_states(shape, B, 1, device="cuda")
    out = torch.empty_like(x)
    ctx_d, tab_d = i32(dec.ctx_lens), i32(dec.tables)
    fn = lambda b=B: tdp.tdp_stage_decode(st.h, x, ctx_d, tab_d, b, out, stream)
    ms = time_calls(fn, warmup, steps)
    work = A.decode_step_work(*sargs, dec_ctx, kv_elem_bytes=1)
    ct = class_times(tdp, st, fn, 5)
    kern = kernel_rooflines(shape, B, work["kv_read_bytes"], work["attn_flops"], ct, "decode")
    sweep = []
    for b in (64, 128, 256):
        if b >= B:
            continue
        msb = time_calls(lambda: fn(b), 3, 10)
        sweep.append({"batch": b, "ms_per_step": round(msb, 4), "tok_s": round(b / msb * 1e3, 1)})
    st.close()
    torch.cuda.empty_cache()
    return {"kv_dtype": "e4m3", "k_scale": 1.0, "v_scale": 1.0, "batch": B, "ms_per_step": round(ms, 4),
            "tok_s": round(B / ms * 1e3, 1), "alg_bytes_per_step": work["bytes"],
            "hbm_gbs": round(work["bytes"] / ms / 1e6, 1), "class_ms": {k: round(v, 4) for k, v in ct.items()},
            "attention": kern.get("attention"), "sweep": sweep}


def empirical_section(tdp, st, n_layers, stream):
    """What this GPU sustains with nothing else in the way (library probes, HIP events inside the calls):
    HBM reads over a footprint like one decode-attention launch's (2 GiB) in address order and in scattered
    4 KiB pieces (how a paged cache is read), the in-order rate over a large footprint, and a register-only
    bf16 MFMA loop.  Context for the published peaks the roofline fractions are quoted against."""
    k, _, n = tdp.tdp_stage_kv_pool(st.h, 0)
    total = n * n_layers                              # the layers' K pools are one contiguous allocation
    out = {}
    for name, size, scattered, nt in (("hbm_read_in_order_gbs", 2 << 30, False, False),
                                      ("hbm_read_4k_scattered_gbs", 2 << 30, True, False),
                                      ("hbm_read_in_order_large_gbs", 16 << 30, False, False),
                                      ("hbm_read_4k_scattered_large_gbs", 16 << 30, True, False),
                                      # the same reads marked non-temporal, as the kernels mark what they read once
                                      ("hbm_read_in_order_non_temporal_gbs", 2 << 30, False, True),
                                      ("hbm_read_4k_scattered_non_temporal_gbs", 2 << 30, True, True),
                                      ("hbm_read_4k_scattered_non_temporal_large_gbs", 16 << 30, True, True)):
        nbytes, ms = tdp.tdp_probe_hbm_read(k, min(size, total), scattered, 5, stream, non_temporal=nt)
        out[name] = round(nbytes / ms / 1e6, 1)
        out[name.replace("_gbs", "_footprint_bytes")] = nbytes
    flop, ms = tdp.tdp_probe_mfma_bf16(8192, 5, True, stream)
    out["mfma_bf16_loop_tflops"] = round(flop / ms / 1e9, 1)                       # operands uniform in (-1, 1)
    flop, ms = tdp.tdp_probe_mfma_bf16(8192, 5, False, stream)
    out["mfma_bf16_loop_constant_operands_tflops"] = round(flop / ms / 1e9, 1)
    return out


def ends_section(tdp, W, shape, batch, i32, vocab=32000):
    """What the first and the last stage of a pipeline add per decode step: the token-embedding
    lookup, and final RMSNorm + vocabulary projection (fp32 logits) + greedy selection."""
    import torch
    h = tdp.tdp_ends_create(tdp.EndsConfig(vocab, shape.d_model, shape.rms_eps, batch))
    for which, name, dt, rows, cols in ((tdp.E_EMBEDDING, "embedding", tdp.BF16, vocab, shape.d_model),
                                        (tdp.E_LM_HEAD, "lm_head", tdp.BF16, shape.d_model, vocab),
                                        (tdp.E_FINAL_NORM, "final_norm", tdp.F32, shape.d_model, 1)):
        w = W.ends_weight(shape, name, vocab, device="cuda", dtype=torch.float32 if dt == tdp.F32 else torch.bfloat16)
        tdp.tdp_ends_set_weight(h, which, w, dt, tdp.DEVICE, rows, cols)
        del w
    ids = i32(W.token_ids(vocab, batch, 1))
    x = torch.empty((batch, shape.d_model), dtype=torch.bfloat16, device="cuda")
    tok = torch.empty(batch, dtype=torch.int32, device="cuda")
    stream = torch.cuda.current_stream()
    t_embed = time_calls(lambda: tdp.tdp_embed_tokens(h, ids, batch, x, stream), 3, 20)
    x = W.hidden_states(shape, batch, 5, device="cuda")
    t_head = time_calls(lambda: tdp.tdp_lm_head(h, x, batch, None, batch, None, tok, stream), 3, 20)
    tdp.tdp_ends_destroy(h)
    flops = 2.0 * batch * vocab * shape.d_model
    return {"vocab": vocab, "batch": batch, "embed_ms": round(t_embed, 4), "lm_head_ms": round(t_head, 4),
            "lm_head_tflops": round(flops / t_head / 1e9, 1),
            "lm_head_weight_gbs": round(vocab * shape.d_model * 2 / t_head / 1e6, 1)}


def engine_section(tdp, W, Stage, shape, decode_sweep, prefill_curve, i32, n_requests=256, n_stages=4, vocab=32000):
    """The decisions of Sec. 3.3 - 3.5 driving the real stage on this one GPU: tdp_simulate_exec plans a
    4-stage temporally-disaggregated pipeline on the measured profile and a StageWorker executes every batch
    of the schedule with the HIP kernels (token embedding -> stage -> vocabulary projection -> greedy token),
    one after the other.  The wall time is therefore that of ONE GPU doing every batch's work in turn, not a
    pipeline's; it shows the whole path running from token ids to token ids under the paper's scheduling."""
    import torch
    from paper_2506_10470_amd import tdp_sched as L
    from paper_2506_10470_amd.engine import StageWorker

    dec = [(float(s["batch"]), float(s["ms_per_step"])) for s in decode_sweep]
    pre = [(float(c["tokens"]), float(c["ms"])) for c in prefill_curve]
    reqs = [(int(a), int(min(b, 128)), int(min(c, 128))) for a, b, c in W.serving_requests(n_requests)]
    prompts = [W.token_ids(vocab, r[0], 1000 + i) for i, r in enumerate(reqs)]
    budget = 4096
    capacity = 48 * 1024                      # tokens: small enough that the run switches phases several times
    max_len = max(r[0] + r[1] for r in reqs) + 1
    max_pps = (max_len + 15) // 16 + 1
    num_pages = capacity // 16 + n_requests
    max_tokens = max(budget, max_len)
    st = Stage(tdp, shape, num_pages, n_requests, max_tokens, n_requests, max_pps, load_weights=True)
    ends = tdp.tdp_ends_create(tdp.EndsConfig(vocab, shape.d_model, shape.rms_eps, max(max_tokens, n_requests)))
    for which, name, dt, rows, cols in ((tdp.E_EMBEDDING, "embedding", tdp.BF16, vocab, shape.d_model),
                                        (tdp.E_LM_HEAD, "lm_head", tdp.BF16, shape.d_model, vocab),
                                        (tdp.E_FINAL_NORM, "final_norm", tdp.F32, shape.d_model, 1)):
        w = W.ends_weight(shape, name, vocab, device="cuda", dtype=torch.float32 if dt == tdp.F32 else torch.bfloat16)
        tdp.tdp_ends_set_weight(ends, which, w, dt, tdp.DEVICE, rows, cols)
        del w
    worker = StageWorker(tdp, st.h, ends, shape.d_model, num_pages, max_pps, n_requests, max_tokens, n_requests, prompts)
    cfg = L.SimConfig(n_stages, capacity, budget, 1, 1, 1, 1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    res, _ = worker.run(L, cfg, reqs, dec, pre)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ok = [len(g) for g in worker.generated] == [r[1] for r in reqs] and len(worker.free_pages) == num_pages
    tdp.tdp_ends_destroy(ends)
    st.close()
    torch.cuda.empty_cache()
    return {"n_requests": n_requests, "n_stages_planned": n_stages, "kv_capacity_tokens": capacity, "vocab": vocab,
            "generated_tokens": int(res.generated_tokens), "prefill_tokens": int(res.prefill_tokens),
            "phase_switches": int(res.phase_switches), "recomputes": int(res.recomputes),
            "prefill_batches": worker.stats["prefill_batches"], "decode_steps": worker.stats["decode_steps"],
            "wall_s_one_gpu_sequential": round(wall, 3),
            "tok_s_one_gpu_sequential": round(res.generated_tokens / wall, 1),
            "planned_pipeline_tok_s": round(res.generated_tokens / (res.total_ms * 1e-3), 1),
            "all_requests_complete_and_pages_returned": bool(ok)}


def scheduler_section(shape, decode_sweep, prefill_curve, n_requests=20000, n_stages=4):
    """The paper's three scheduling decisions (Sec. 3.3 - 3.5) driving a simulated pipeline of
    `n_stages` copies of this stage, timed by the profile measured above: 20000 synthetic requests
    (enough to fill the KV capacity several times over),
    KV capacity = what 90 % of one GPU's 288 GB leaves after the stage's weights.  Host code only."""
    from harness import workload as W
    from paper_2506_10470_amd import accounting as A
    from paper_2506_10470_amd import tdp_sched as L

    dec = [(float(s["batch"]), float(s["ms_per_step"])) for s in decode_sweep]
    pre = [(float(c["tokens"]), float(c["ms"])) for c in prefill_curve]
    weights = 2 * shape.n_layers * A.matmul_params_per_layer(shape.d_model, shape.n_q_heads, shape.n_kv_heads,
                                                             shape.head_dim, shape.d_ff)
    kv_tok = A.kv_bytes_per_token(shape.n_layers, shape.n_kv_heads, shape.head_dim)
    capacity = int((0.9 * 288e9 - weights) // kv_tok)
    reqs = [tuple(int(v) for v in r) for r in W.serving_requests(n_requests)]
    names = {"td_pipe": (1, 1, 1), "no_greedy_prefill": (0, 1, 1), "no_work_stealing": (1, 0, 1),
             "no_intensity_switch": (1, 1, 0), "none": (0, 0, 0)}

    def run_policies(cap):
        out = {}
        for name, (g, w, i) in names.items():
            cfg = L.SimConfig(n_stages, cap, 16384, g, w, i, 1)
            t0 = time.perf_counter()
            res, _ = L.tdp_simulate(cfg, reqs, dec, pre)
            wall = time.perf_counter() - t0
            out[name] = {"tok_s": round(res.generated_tokens / (res.total_ms * 1e-3), 1),
                         "total_s": round(res.total_ms * 1e-3, 2), "phase_switches": res.phase_switches,
                         "recomputes": res.recomputes, "peak_kv_tokens": res.peak_kv_tokens,
                         "bubble_ratio": round(1.0 - res.busy_ms / (n_stages * res.total_ms), 4),
                         "decisions": res.n_events, "scheduler_wall_ms": round(wall * 1e3, 2)}
        return out

    # the same queue with a quarter of the KV memory: the regime the paper's 40-48 GB GPUs are in, where the
    # decode batches cannot reach the peak batch size and the timing of the phase switches decides the throughput
    return {"n_stages": n_stages, "n_requests": n_requests, "kv_capacity_tokens": capacity,
            "prefill_token_budget": 16384, "data": "synthetic request lengths; stage times measured in this run",
            "policies": run_policies(capacity),
            "memory_tight": {"kv_capacity_tokens": capacity // 4, "policies": run_policies(capacity // 4)}}


def other_config_section(tdp, W, Stage, A, i32, name, batches, n_prompts):
    """A lean pass over one of the other benchmark configurations (same code paths as the headline): decode
    at the given batch sizes, timed per step with events, per-class times and rooflines at the largest,
    and the configuration's prefill batch."""
    import torch
    shape = W.SHAPES[name]
    B = max(batches)
    dec_ctx = W.decode_ctx_lens(name, B)
    pre_lens = W.prefill_seq_lens(name, n_prompts)
    st, dec, pre, pre_tables, _ = build_stage(tdp, W, Stage, shape, dec_ctx, pre_lens, i32)
    stream = torch.cuda.current_stream()
    sargs = (shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ff)
    x = W.hidden_states(shape, B, 1, device="cuda")
    out = torch.empty_like(x)
    ctx_d, tab_d = i32(dec.ctx_lens), i32(dec.tables)
    fn = lambda b=B: tdp.tdp_stage_decode(st.h, x, ctx_d, tab_d, b, out, stream)
    sweep = []
    for b in batches:
        pb = time_events(lambda: fn(b), 5, 30)
        wb = A.decode_step_work(*sargs, dec_ctx[:b])
        sweep.append({"batch": b, "ms_per_step": pb["mean"], "ms_p10": pb["p10"], "ms_p90": pb["p90"],
                      "tok_s": round(b / pb["mean"] * 1e3, 1), "hbm_gbs": round(wb["bytes"] / pb["mean"] / 1e6, 1),
                      "hbm_frac": round(wb["bytes"] / pb["mean"] / 1e6 / HBM_PEAK_GBS, 4)})
    peak = max(v["tok_s"] for v in sweep)
    for v in sweep:
        v["spatial_intensity"] = round(v["tok_s"] / peak, 4)
    work = A.decode_step_work(*sargs, dec_ctx)
    ct = class_times(tdp, st, fn, 3)
    kern = kernel_rooflines(shape, B, work["kv_read_bytes"], work["attn_flops"], ct, "decode")
    T = int(pre_lens.sum())
    xp = W.hidden_states(shape, T, 2, device="cuda")
    op = torch.empty_like(xp)
    cu_p, tab_p = i32(pre.cu_seqlens), i32(pre_tables)
    pfn = lambda: tdp.tdp_stage_prefill(st.h, xp, cu_p, tab_p, len(pre_lens), T, op, stream)
    msp = time_calls(pfn, 1, 3)
    wp = A.prefill_work(*sargs, pre_lens)
    ctp = class_times(tdp, st, pfn, 2)
    gemm_ms = sum(ctp[k] for k in ("gemm_qkv", "gemm_o", "gemm_gate_up", "gemm_down"))
    res = {"workload": "%s stage" % name, "n_layers": shape.n_layers, "mean_ctx": round(float(dec_ctx.mean()), 1),
           "decode_sweep": sweep,
           "decode_at_batch_%d" % B: {"class_ms": {k: round(v, 4) for k, v in ct.items()}, "kernels": kern},
           "prefill": {"tokens": T, "n_prompts": len(pre_lens), "ms": round(msp, 3), "tok_s": round(T / msp * 1e3, 1),
                       "tflops": round(wp["flops"] / msp / 1e9, 1),
                       "gemm_tflops": round(wp["gemm_flops"] / gemm_ms / 1e9, 1),
                       "gemm_mfma_frac": round(wp["gemm_flops"] / gemm_ms / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4),
                       "class_ms": {k: round(v, 3) for k, v in ctp.items()}}}
    log("%s: decode %s; prefill %d tokens %.1f ms (GEMMs %.0f TFLOP/s)" % (
        name, ", ".join("B=%d %.2f ms %.0f GB/s" % (v["batch"], v["ms_per_step"], v["hbm_gbs"]) for v in sweep), T, msp,
        wp["gemm_flops"] / gemm_ms / 1e9))
    del xp, op, x, out
    st.close()
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="70b_quarter", choices=["70b_quarter", "13b_quarter", "7b_quarter", "qwen32b_quarter"])
    ap.add_argument("--batch", type=int, default=512)
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (debugging only)")
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--no-prefill", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--micro-batches", type=int, default=0, choices=[0, 2],
                    help="2: also time the headline step as two half-batches on two streams (decode_micro_batches)")
    ap.add_argument("--no-others", action="store_true", help="skip the lean passes over the other configurations")
    ap.add_argument("--decode-span", type=int, default=0, choices=[0, 256, 512, 1024, 2048, 4096],
                    help="pin the tokens of one context handled by one decode-attention workgroup (0: the library's choice)")
    ap.add_argument("--kv-fp8", action="store_true",
                    help="run the 8-bit KV-cache section even in the lean (--no-sweep) mode")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy, the known-size kernel that rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE readings are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (pipeline stages would each run "
              "this same code on their own GPU); re-run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from harness import workload as W
    from harness.runner import Stage, i32
    from paper_2506_10470_amd import accounting as A
    from paper_2506_10470_amd import tdp

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    shape = W.SHAPES[args.workload]
    if args.layers:
        shape = shape.with_layers(args.layers)
    B = args.batch
    n_prompts = {"70b_quarter": 16, "13b_quarter": 32, "7b_quarter": 32, "qwen32b_quarter": 32}[args.workload]
    dec_ctx = W.decode_ctx_lens(args.workload, B)
    pre_lens = W.prefill_seq_lens(args.workload, n_prompts)
    st, dec, pre, pre_tables, cu = build_stage(tdp, W, Stage, shape, dec_ctx, pre_lens, i32)
    if args.decode_span:
        tdp.tdp_stage_set_decode_span(st.h, args.decode_span)
    stream = torch.cuda.current_stream()
    sargs = (shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ff)

    x = W.hidden_states(shape, B, 1, device="cuda")
    out = torch.empty_like(x)
    ctx_d, tab_d = i32(dec.ctx_lens), i32(dec.tables)

    def decode_fn(b=B):
        tdp.tdp_stage_decode(st.h, x, ctx_d, tab_d, b, out, stream)

    if args.copy_calibration:
        src = torch.empty(1 << 29, dtype=torch.bfloat16, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)            # 1 GiB read + 1 GiB written
        torch.cuda.synchronize()
        del src, dst

    # ---- headline: decode at the full batch
    ms = time_calls(decode_fn, args.warmup, args.steps)
    work = A.decode_step_work(*sargs, dec_ctx)
    log("decode B=%d: %.3f ms/step, %.0f tok/s, %.0f GB/s algorithmic" % (B, ms, B / ms * 1e3,
                                                                          work["bytes"] / ms / 1e6))
    pct, ms_adv = None, None
    if not args.no_sweep:   # (--no-sweep is the lean mode the profiler runs use: headline + per-class times only)
        for _ in range(max(0, 20 - args.warmup - args.steps)):   # at least 20 steps before the percentiles
            decode_fn()
        pct = step_percentiles(decode_fn, max(args.steps, 100))
        # the same step repeated rewrites the same KV slot; this run advances every context by one token
        # per step instead, so each request crosses a page boundary once within ADVANCE_STEPS steps
        ctx_run = ctx_d.clone()

        def advancing_fn():
            tdp.tdp_stage_decode(st.h, x, ctx_run, tab_d, B, out, stream)
            ctx_run.add_(1)

        ms_adv = time_calls(advancing_fn, 0, ADVANCE_STEPS)
    ct = class_times(tdp, st, decode_fn, 5)
    kern = kernel_rooflines(shape, B, work["kv_read_bytes"], work["attn_flops"], ct, "decode")
    workload_name = "%s stage, decode phase, batch %d" % (args.workload, B)
    traffic, traffic_src = measured_traffic(workload_name)
    for name, tr in traffic.items():
        if name in kern and not args.layers:
            kern[name]["traffic"] = tr
            kern[name]["traffic_source"] = traffic_src
    dominant = max(kern, key=lambda k: ct[k])
    roof = dict(kern[dominant])
    roof["kernel"] = dominant
    t_min = sum(max(v["alg_bytes_per_launch"] * v["launches_per_step"] / (HBM_PEAK_GBS * 1e9),
                    v["alg_flops_per_launch"] * v["launches_per_step"] / (MFMA_BF16_PEAK_TFLOPS * 1e12))
                for v in kern.values()) * 1e3

    result = {
        "metric": "stage decode tok/s vs batch; prefill tok/s; % of HBM / MFMA roofline",
        "value": round(B / ms * 1e3, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": workload_name,
                   "n_layers": shape.n_layers, "d_model": shape.d_model, "n_q_heads": shape.n_q_heads,
                   "n_kv_heads": shape.n_kv_heads, "head_dim": shape.head_dim, "d_ff": shape.d_ff,
                   "batch": B, "mean_ctx": round(float(dec_ctx.mean()), 1), "max_ctx": int(dec_ctx.max()),
                   "page_size": 16, "parallelism": "single GPU"},
        "roofline": roof,
        "decode": {"alg_bytes_per_step": work["bytes"], "alg_flops_per_step": work["flops"],
                   "hbm_gbs": round(work["bytes"] / ms / 1e6, 1),
                   "hbm_frac": round(work["bytes"] / ms / 1e6 / HBM_PEAK_GBS, 4),
                   "composite_t_min_ms": round(t_min, 3), "composite_frac": round(t_min / ms, 4),
                   "step_ms_percentiles": pct,
                   "advancing_context_ms_per_step": None if ms_adv is None else round(ms_adv, 4),
                   "class_ms": {k: round(v, 4) for k, v in ct.items()}, "kernels": kern},
    }

    # ---- decode batch-size sweep on the same stage (first b requests of the batch)
    if not args.no_sweep:
        sweep = []
        for b in (16, 32, 64, 128, 256, 512):
            if b > B:
                continue
            pb = time_events(lambda: decode_fn(b), 5, 40)       # events on the launch stream, per step
            msb = pb["mean"]
            wb = A.decode_step_work(*sargs, dec_ctx[:b])
            sweep.append({"batch": b, "ms_per_step": round(msb, 4), "ms_p10": pb["p10"], "ms_p90": pb["p90"],
                          "tok_s": round(b / msb * 1e3, 1), "hbm_gbs": round(wb["bytes"] / msb / 1e6, 1),
                          "hbm_frac": round(wb["bytes"] / msb / 1e6 / HBM_PEAK_GBS, 4)})
            log("  sweep B=%d: %.3f ms, %.0f tok/s, %.0f GB/s" % (b, msb, b / msb * 1e3, wb["bytes"] / msb / 1e6))
        peak = max(s["tok_s"] for s in sweep)
        for s in sweep:
            s["spatial_intensity"] = round(s["tok_s"] / peak, 4)     # Achieved / Peak (paper Eq. 1)
        result["decode_sweep"] = sweep
        # the batch the HBM target is stated on (>= 256): per-kernel rooflines of the same stage at batch 256
        if B > 256:
            b = 256
            w256 = A.decode_step_work(*sargs, dec_ctx[:b])
            ct256 = class_times(tdp, st, lambda: decode_fn(b), 5)
            k256 = kernel_rooflines(shape, b, w256["kv_read_bytes"], w256["attn_flops"], ct256, "decode")
            tr256, src256 = measured_traffic("%s stage, decode phase, batch %d" % (args.workload, b))
            for name, tr in tr256.items():
                if name in k256 and not args.layers:
                    k256[name]["traffic"] = tr
                    k256[name]["traffic_source"] = src256
            ms256 = next(x["ms_per_step"] for x in sweep if x["batch"] == b)
            t_min256 = sum(max(v["alg_bytes_per_launch"] * v["launches_per_step"] / (HBM_PEAK_GBS * 1e9),
                               v["alg_flops_per_launch"] * v["launches_per_step"] / (MFMA_BF16_PEAK_TFLOPS * 1e12))
                           for v in k256.values()) * 1e3
            result["decode_b256"] = {"batch": b, "ms_per_step": ms256, "tok_s": round(b / ms256 * 1e3, 1),
                                     "alg_bytes_per_step": w256["bytes"], "hbm_gbs": round(w256["bytes"] / ms256 / 1e6, 1),
                                     "hbm_frac": round(w256["bytes"] / ms256 / 1e6 / HBM_PEAK_GBS, 4),
                                     "composite_t_min_ms": round(t_min256, 3), "composite_frac": round(t_min256 / ms256, 4),
                                     "class_ms": {k: round(v, 4) for k, v in ct256.items()}, "kernels": k256}

    # ---- prefill
    if not args.no_prefill:
        T = int(pre_lens.sum())
        xp = W.hidden_states(shape, T, 2, device="cuda")
        op = torch.empty_like(xp)
        cu_p, tab_p = i32(pre.cu_seqlens), i32(pre_tables)

        def prefill_fn():
            tdp.tdp_stage_prefill(st.h, xp, cu_p, tab_p, len(pre_lens), T, op, stream)

        msp = time_calls(prefill_fn, 1, 3)
        wp = A.prefill_work(*sargs, pre_lens)
        ctp = class_times(tdp, st, prefill_fn, 2)
        kp = kernel_rooflines(shape, T, 0, wp["attn_flops"], {k: v for k, v in ctp.items()}, "prefill")
        gemm_ms = sum(ctp[k] for k in ("gemm_qkv", "gemm_o", "gemm_gate_up", "gemm_down"))
        result["prefill"] = {"tokens": T, "n_prompts": len(pre_lens), "ms": round(msp, 3),
                             "tok_s": round(T / msp * 1e3, 1),
                             "tflops": round(wp["flops"] / msp / 1e9, 1),
                             "mfma_frac": round(wp["flops"] / msp / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4),
                             "gemm_tflops": round(wp["gemm_flops"] / gemm_ms / 1e9, 1),
                             "gemm_mfma_frac": round(wp["gemm_flops"] / gemm_ms / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4),
                             "class_ms": {k: round(v, 3) for k, v in ctp.items()}, "kernels": kp}
        log("prefill T=%d: %.1f ms, %.0f tok/s, %.0f TFLOP/s (GEMMs %.0f TFLOP/s)" % (
            T, msp, T / msp * 1e3, wp["flops"] / msp / 1e9, wp["gemm_flops"] / gemm_ms / 1e9))
        # prefill time against packed tokens (first k prompts): the profile the scheduler plans with
        curve = []
        for k in (1, 2, 4, 8):
            if k >= len(pre_lens) or args.no_sweep:
                continue
            Tk = int(pre.cu_seqlens[k])
            msk = time_calls(lambda: tdp.tdp_stage_prefill(st.h, xp, cu_p, tab_p, k, Tk, op, stream), 1, 2)
            curve.append({"tokens": Tk, "ms": round(msk, 3)})
        curve.append({"tokens": T, "ms": round(msp, 3)})
        result["prefill"]["curve"] = sorted(curve, key=lambda c: c["tokens"])
        del xp, op

    if not args.layers:
        emp = empirical_section(tdp, st, shape.n_layers, stream)
        result["empirical_peaks"] = emp
        if roof["bound"] == "hbm":
            # against the probe that reads the way the kernel does: scattered 4 KiB pieces, non-temporal loads
            roof["frac_of_measured_scattered_read"] = round(
                roof["achieved"] / emp["hbm_read_4k_scattered_non_temporal_gbs"], 4)
        # the composite lower bound again, priced at what the probes sustain instead of the published peaks
        t_min_emp = sum(max(v["alg_bytes_per_launch"] * v["launches_per_step"] / (emp["hbm_read_in_order_non_temporal_gbs"] * 1e9),
                            v["alg_flops_per_launch"] * v["launches_per_step"] / (emp["mfma_bf16_loop_tflops"] * 1e12))
                        for v in kern.values()) * 1e3
        result["decode"]["composite_t_min_at_measured_ceilings_ms"] = round(t_min_emp, 3)
        result["decode"]["composite_frac_of_measured_ceilings"] = round(t_min_emp / ms, 4)
        if "prefill" in result:
            result["prefill"]["gemm_frac_of_measured_mfma_loop"] = round(
                result["prefill"]["gemm_tflops"] / emp["mfma_bf16_loop_tflops"], 4)
        log("empirical ceilings: %s" % json.dumps(emp))
    st.close()
    torch.cuda.empty_cache()
    if args.micro_batches == 2:
        result["decode_two_half_batches"] = micro_batch_section(tdp, W, Stage, shape, dec_ctx, i32, args.steps, args.warmup)
        log("decode as two half-batches on two streams: %s" % json.dumps(result["decode_two_half_batches"]["batches"]))
    if args.kv_fp8 or not (args.layers or args.no_sweep):
        result["decode_fp8_kv"] = fp8_kv_section(tdp, W, Stage, A, shape, sargs, dec_ctx, i32, args.steps, args.warmup)
        log("decode B=%d with an 8-bit KV cache: %.3f ms/step, %.0f tok/s (attention %.3f ms per step)" % (
            B, result["decode_fp8_kv"]["ms_per_step"], result["decode_fp8_kv"]["tok_s"],
            result["decode_fp8_kv"]["class_ms"]["attention"]))
    if not args.layers and not args.no_sweep:
        result["ends"] = ends_section(tdp, W, shape, B, i32)
        log("pipeline ends at batch %d: embedding %.3f ms, final norm + vocabulary projection + greedy %.3f ms" % (
            B, result["ends"]["embed_ms"], result["ends"]["lm_head_ms"]))
    if "decode_sweep" in result and "prefill" in result:
        result["scheduler"] = scheduler_section(shape, result["decode_sweep"], result["prefill"]["curve"])
        log("scheduler (simulated 4-stage pipeline on the measured profile): %s; with a quarter of the KV memory: %s" % (
            json.dumps({k: v["tok_s"] for k, v in result["scheduler"]["policies"].items()}),
            json.dumps({k: v["tok_s"] for k, v in result["scheduler"]["memory_tight"]["policies"].items()})))
    if "decode_sweep" in result and "prefill" in result and not args.layers:
        result["engine"] = engine_section(tdp, W, Stage, shape, result["decode_sweep"], result["prefill"]["curve"], i32)
        log("engine (schedule executed with the real kernels, %d requests): %s" % (
            result["engine"]["n_requests"], json.dumps({k: result["engine"][k] for k in (
                "generated_tokens", "decode_steps", "prefill_batches", "phase_switches", "recomputes",
                "wall_s_one_gpu_sequential", "tok_s_one_gpu_sequential")})))
    if args.workload == "70b_quarter" and not (args.layers or args.no_sweep or args.no_others):
        # the other benchmark configurations (7B decode at batch 256 + prefill; 13B prefill and batch sweep, the
        # Achieved / Peak curve of Sec. 3.5 on the paper's own 13B shape), lean passes through the same code
        result["other_configs"] = {
            "7b_quarter": other_config_section(tdp, W, Stage, A, i32, "7b_quarter", (256,), 32),
            "13b_quarter": other_config_section(tdp, W, Stage, A, i32, "13b_quarter", (16, 32, 64, 128, 256, 512), 32)}
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(shape, dec_ctx, cu)
        log("cpu oracle: %s tok/s (%s)" % (result["cpu_baseline"]["value"], result["cpu_baseline"]["sample"]))
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()

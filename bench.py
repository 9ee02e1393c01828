#!/usr/bin/env python3
"""Benchmark of the fused SWA+RLA layer on one MI355X.

A step = rattn_fwd (saving for backward) + rattn_bwd on the 3B-scale layer
(B=4, Hq=24, Hkv=8, T=4096, D=128, W=512, bf16), inputs resident in HBM.  `value` is the
algorithmic TFLOP/s of fwd+bwd: exact in-window (t,s) pairs plus the chunked linear-attention
products at nominal chunk 64, no recomputation and no masked-tile waste counted.
Prints ONE JSON line.
"""
import argparse
import ctypes
import dataclasses
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_MFMA = 2.5e15     # dense bf16 MFMA FLOP/s, MI355X
PEAK_FP32_VALU = 157.3e12   # fp32 vector FLOP/s
PEAK_HBM = 8.0e12           # bytes/s
NOMINAL_CHUNK = 64


def swa_pairs(T, W):
    return W * T - W * (W - 1) // 2 if W <= T else T * (T + 1) // 2


def layer_flops(B, T, Hq, Hkv, D, W, C=NOMINAL_CHUNK):
    """Algorithmic FLOPs of the layer, split by the kernels' responsibilities."""
    P = swa_pairs(T, W)
    Tp = max(T - W, 0)
    f = {}
    f["fwd_swa"] = B * Hq * 4 * D * P
    f["fwd_rla_out"] = B * Hq * (2 * Tp * D * D + 4 * D * Tp * (C + 1) // 2)
    f["fwd_state"] = B * Hkv * 2 * Tp * D * D
    f["bwd_swa"] = B * Hq * 10 * D * P
    f["bwd_rla_q"] = B * Hq * (4 * Tp * D * D + 10 * D * Tp * (C + 1) // 2)
    f["bwd_rla_kv"] = B * Hkv * 4 * Tp * D * D
    f["fwd"] = f["fwd_swa"] + f["fwd_rla_out"] + f["fwd_state"]
    f["bwd"] = f["bwd_swa"] + f["bwd_rla_q"] + f["bwd_rla_kv"]
    return f


def kernel_algorithmic_flops(name, fl):
    """Algorithmic FLOPs one launch of a named kernel is responsible for (None = not one of the contraction kernels:
    the chunk-state kernels are bound by HBM traffic, their few matrix FLOPs are credited to the step as a whole)."""
    table = {
        "gen_fwd_kernel": fl["fwd_swa"] + fl["fwd_rla_out"],
        "gen_scan_kernel": fl["fwd_state"],
        "gen_bwd_dq_kernel": 0.4 * fl["bwd_swa"] + 0.5 * fl["bwd_rla_q"],
        "gen_bwd_dkv_kernel": 0.6 * fl["bwd_swa"] + 0.5 * fl["bwd_rla_q"] + 0.5 * fl["bwd_rla_kv"],
        "fwd_fused_kernel": fl["fwd_swa"] + fl["fwd_rla_out"],
        "bwd_dq_kernel": 0.4 * fl["bwd_swa"] + 0.5 * fl["bwd_rla_q"],
        "bwd_dkv_kernel": 0.6 * fl["bwd_swa"] + 0.5 * fl["bwd_rla_q"] + 0.5 * fl["bwd_rla_kv"],
    }
    return table.get(name)


def measured_traffic(kernel, workload):
    """HBM bytes per launch of `kernel` from the committed counter summary (FETCH_SIZE + WRITE_SIZE, scaled by what the
    same counters read for a plain copy of known size), with where the figure comes from: it is NOT measured in this
    run (rocprofv3 counters need a run of their own), so the summary's digest of the kernel sources is compared with
    the sources in the tree and a mismatch is reported as stale.  (None, info) when no summary covers the kernel."""
    rel = f"profiles/hbm_traffic_{workload}.txt"
    info = {"file": rel, "measured_in_this_run": False}
    try:
        with open(os.path.join(ROOT, rel)) as f:
            rows = json.loads(f.read().split("---JSON---", 1)[1])
    except (OSError, IndexError, ValueError):
        return None, info
    import profile_summary
    info["kernel_sources_of_summary"] = rows.get("_kernel_sources")
    info["stale"] = rows.get("_kernel_sources") != profile_summary.kernel_sources_digest()
    return rows.get(kernel, {}).get("hbm_bytes_per_launch"), info


def decode_bytes(N, Hkv, Hq, D, W, esize, nvalid_sum=None):
    ring = 2 * N * Hkv * W * D * esize if nvalid_sum is None else 2 * nvalid_sum * Hkv * D * esize
    state = 2 * N * Hkv * D * D * 4
    vec = N * (2 * Hq + 4 * Hkv) * D * esize  # q, o, k_new, v_new, ring slot write
    return ring + state + vec


_CPU_INPUTS = None   # set in the parent before the worker pool forks


def _cpu_unit(unit):
    """One (batch row, query head) of the fp64 oracle, forward + backward, on one thread."""
    from oracle import rattn_oracle as orc
    try:
        from threadpoolctl import threadpool_limits
        limit = threadpool_limits(limits=1)
    except Exception:
        limit = None
    cfg, q, k, v, dO = _CPU_INPUTS
    b, h = unit
    t0 = time.perf_counter()
    orc.fwd_dense(q, k, v, cfg.W, scale=cfg.scale, heads=[h], batches=[b])
    orc.bwd_dense(q, k, v, dO, cfg.W, scale=cfg.scale, heads=[h], batches=[b])
    dt = time.perf_counter() - t0
    del limit
    return dt


def host_cores():
    n = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    for var in ("OMP_NUM_THREADS", "MAX_JOBS"):   # the machine's CPU share, where it is smaller than what nproc shows
        try:
            n = min(n, int(os.environ[var]))
        except (KeyError, ValueError):
            pass
    return max(n, 1)


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(cfg, units_per_core=6):
    """The fp64 oracle, as it stands, on a bounded sample of the benchmark workload: a process pool over
    (batch row, query head) units on all host cores (one thread each), `units_per_core` units per core, each unit the
    full sequence, forward + backward.  Units are independent and equal in work, so the measured rate carries over to
    all B * Hq units: the extrapolated whole-tensor time is reported next to the measured one.
    Must run before this process touches the GPU (the pool forks)."""
    global _CPU_INPUTS
    import multiprocessing as mp
    import torch
    from paper_2506_15545_amd import synth
    cores = host_cores()
    all_units = [(b, h) for b in range(cfg.B) for h in range(cfg.Hq)]
    units = all_units[:min(len(all_units), units_per_core * cores)]
    f64 = lambda t: t.to(torch.float64).numpy()
    _CPU_INPUTS = (cfg,) + tuple(f64(t) for t in synth.make_layer_inputs(cfg, with_dO=True, B=units[-1][0] + 1))
    t0 = time.perf_counter()
    with mp.get_context("fork").Pool(cores) as pool:
        unit_s = pool.map(_cpu_unit, units, chunksize=1)
    dt = time.perf_counter() - t0
    _CPU_INPUTS = None
    fl = layer_flops(1, cfg.T, 1, 0, cfg.D, cfg.W)
    # the per-KV-head state products are shared by the G heads of a group in the method; the oracle recomputes them per
    # query head, the FLOP count credits them once per group as everywhere else in this file
    unit_flops = fl["fwd"] + fl["bwd"] + (layer_flops(1, cfg.T, 0, 1, cfg.D, cfg.W)["fwd"]
                                          + layer_flops(1, cfg.T, 0, 1, cfg.D, cfg.W)["bwd"]) * cfg.Hkv / cfg.Hq
    flops = unit_flops * len(units)
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": f"fp64 numpy oracle fwd+bwd, {len(units)} of {len(all_units)} (batch row, query head) units, full "
                      f"T={cfg.T}, process pool of {cores} single-thread workers, {dt:.1f} s wall",
            "seconds": dt, "units": len(units), "unit_seconds_mean": sum(unit_s) / len(unit_s),
            "whole_tensor_seconds_extrapolated": dt * len(all_units) / len(units),
            "cpu_model": cpu_model(), "nproc": os.cpu_count()}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-prefill", action="store_true",
                    help="skip the reported-only prefill hand-over and chunked-prefill timings (profiling runs: keeps "
                         "every forward launch in the trace on the headline workload)")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--cpu-units-per-core", type=int, default=6,
                    help="(batch row, query head) units of the oracle per host core in the cpu_baseline sample")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the reported-only timings of the 12B-shaped layer and the window sweep")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain out-of-place elementwise pass over 256 MiB (reads and writes 256 MiB): "
                         "under a counter run its FETCH_SIZE / WRITE_SIZE readings give the counters' scale")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    from paper_2506_15545_amd import synth
    # the CPU baseline forks a worker pool: it runs first, before this process has touched the GPU
    cpu_base = None
    if not args.no_cpu_baseline:
        cpu_base = cpu_baseline(synth.CONFIGS["layer3b_t4096_w512"], args.cpu_units_per_core)

    import torch
    from paper_2506_15545_amd import binding as rb
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    rb.lib()
    torch.cuda.set_device(0)

    cfg = synth.CONFIGS["layer3b_t4096_w512"]
    q, k, v, dO = (t.cuda() for t in synth.make_layer_inputs(cfg, with_dO=True))
    p = rb.make_params(q, k, cfg.W, 0, cfg.scale, 1e-6, True)
    fwd_b, bwd_b, saved_b = rb.rattn_workspace_bytes(p)
    ws = torch.empty(max(fwd_b, bwd_b, 16), dtype=torch.uint8, device="cuda")
    saved = torch.empty(saved_b, dtype=torch.uint8, device="cuda")
    o = torch.empty_like(q)
    grads = (torch.empty_like(q), torch.empty_like(k), torch.empty_like(v))

    def fwd_only():
        rb.rattn_fwd(q, k, v, cfg.W, softmax_scale=cfg.scale, save_for_bwd=True, out=o, saved=saved, workspace=ws)

    def bwd_only():
        rb.rattn_bwd(q, k, v, saved, dO, cfg.W, softmax_scale=cfg.scale, want_dgamma=False, workspace=ws, out=grads)

    def step():
        fwd_only()
        bwd_only()

    def timed(fn, n):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    # What this device sustains on nothing but matrix-core instructions, and on a plain copy: context for the fractions
    # of the published peaks below.  These probes run first, the matrix-core loop last: the device needs some tens of
    # milliseconds of work to reach its steady clocks (the first 20 steps after idling take 1.0 ms each, later ones
    # 0.91; after 100 ms of the matrix-core loop 0.91 at once), more than a short warm-up of the step itself provides.
    machine = None
    if not args.no_other_workloads:
        src = torch.zeros(512 * 2 ** 20 // 4, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1.0, out=dst)
        copy_ms = min(timed(lambda: torch.add(src, 1.0, out=dst), 100) for _ in range(3))   # best of 3 rounds, ~17 ms each
        copy_gbps = 2 * src.numel() * 4 / (copy_ms * 1e-3) / 1e9
        del src, dst
        sink = torch.zeros(64, dtype=torch.float32, device="cuda")
        rb.rattn_probe_mfma(sink, 8000, 2048)
        torch.cuda.synchronize()
        mfma_tflops = 0.0
        for _ in range(6):   # ~13 ms each; the best of them (the rate climbs while the clocks do)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            probe_flops = rb.rattn_probe_mfma(sink, 8000, 2048)
            e1.record()
            torch.cuda.synchronize()
            mfma_tflops = max(mfma_tflops, probe_flops / (e0.elapsed_time(e1) * 1e-3) / 1e12)
        machine = {"mfma_loop_tflops": mfma_tflops, "copy_GBps": copy_gbps}

    for _ in range(args.warmup):
        step()
    # the timed region: exactly `steps` steps, nothing else on the stream
    ms_per_step = timed(step, args.steps)
    # the same step replayed as one HIP graph (reported only: launch gaps removed; `value` stays the eager figure)
    graph_ms = None
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            step()
            with torch.cuda.graph(graph, stream=side):
                step()
        torch.cuda.synchronize()
        for _ in range(5):
            graph.replay()
        # alternate with the eager step so that clock drift over the run hits both alike
        te = tg = 0.0
        for _ in range(3):
            te += timed(step, 20) / 3
            tg += timed(graph.replay, 20) / 3
        graph_ms = {"graph": tg, "eager_interleaved": te}
        del graph
    except Exception as e:  # reported field only
        print(f"bench: graph replay skipped: {e}", file=sys.stderr)
    # the same steps again with the library's per-kernel HIP events (recorded on the launch stream) switched
    # on; they serialise neighbouring kernels, so they stay out of the region `value` is taken from
    rb.rattn_profile_enable(True)
    ms_per_step_profiled = timed(step, args.steps)
    recs = rb.rattn_profile_records()
    rb.rattn_profile_enable(False)
    fwd_ms = timed(fwd_only, args.steps)
    bwd_ms = timed(bwd_only, args.steps)
    fl = layer_flops(cfg.B, cfg.T, cfg.Hq, cfg.Hkv, cfg.D, cfg.W)
    fl_fwd_bwd = (fl["fwd"], fl["bwd"])

    # single calls, one event pair each: median of 100, plain and with 512 MiB written between the calls (more than L2
    # and the memory-side cache hold, so every call starts from HBM); reported, never part of `value`
    per_call = None
    if not args.no_other_workloads:
        def single_calls(fn, scrub, n=100):
            pairs = []
            for _ in range(n):
                if scrub is not None:
                    scrub.zero_()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                fn()
                e1.record()
                pairs.append((e0, e1))
            torch.cuda.synchronize()
            ts = sorted(a.elapsed_time(b) for a, b in pairs)
            return ts[n // 2], ts[0]
        scrub = torch.empty(512 * 2 ** 20, dtype=torch.uint8, device="cuda")
        per_call = {"calls": 100, "scrub_MiB": 512}
        for name, fn, flops in (("fwd", fwd_only, fl_fwd_bwd[0]), ("bwd", bwd_only, fl_fwd_bwd[1])):
            med, best = single_calls(fn, None)
            med_s, _ = single_calls(fn, scrub)
            per_call[name] = {"median_ms": med, "min_ms": best, "median_ms_scrubbed": med_s,
                              "tflops_median": flops / (med * 1e-3) / 1e12, "tokens_per_s_median": cfg.B * cfg.T / (med * 1e-3)}
        del scrub

    total = fl["fwd"] + fl["bwd"]
    value = total / (ms_per_step * 1e-3) / 1e12

    agg = {}
    for name, ms in recs:
        a = agg.setdefault(name, [0.0, 0])
        a[0] += ms; a[1] += 1
    kernels = {n: {"avg_ms": s / c, "launches_per_step": c / args.steps} for n, (s, c) in agg.items()}
    dom = max(kernels, key=lambda n: kernels[n]["avg_ms"] * kernels[n]["launches_per_step"])
    mfma_path = not dom.startswith("gen_")
    peak = PEAK_BF16_MFMA if mfma_path else PEAK_FP32_VALU

    def kernel_roofline(name):
        kfl = kernel_algorithmic_flops(name, fl)
        achieved = (kfl or 0.0) / (kernels[name]["avg_ms"] * 1e-3)
        traffic, src = measured_traffic(name, cfg.name)
        return {"bound": "mfma" if mfma_path else "alu", "kernel": name, "achieved": achieved / 1e12,
                "peak": peak / 1e12, "unit": "TFLOP/s", "frac": achieved / peak, "traffic": traffic,
                "traffic_source": src, "avg_ms": kernels[name]["avg_ms"], "algorithmic_flops": kfl}

    roofline = kernel_roofline(dom)
    # every kernel that carries algorithmic matrix work, and the one furthest below the roof
    per_kernel = {n: kernel_roofline(n) for n in kernels if kernel_algorithmic_flops(n, fl)}
    lowest = min(per_kernel.values(), key=lambda r: r["frac"]) if per_kernel else None

    out = {
        "metric": "fused SWA+RLA fwd+bwd TFLOP/s & % MFMA peak @T=4096,w=512,d=128",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": cfg.name, "B": cfg.B, "T": cfg.T, "Hq": cfg.Hq, "Hkv": cfg.Hkv, "D": cfg.D,
                   "W": cfg.W, "step": "rattn_fwd(save_for_bwd)+rattn_bwd"},
        "frac_mfma_peak": value * 1e12 / PEAK_BF16_MFMA,
        "tokens_per_s": cfg.B * cfg.T / (ms_per_step * 1e-3),
        "ms_per_step_profiled": ms_per_step_profiled,
        "ms_per_step_graph": graph_ms,
        "fwd": {"ms": fwd_ms, "tflops": fl["fwd"] / (fwd_ms * 1e-3) / 1e12,
                "frac_mfma_peak": fl["fwd"] / (fwd_ms * 1e-3) / PEAK_BF16_MFMA},
        "bwd": {"ms": bwd_ms, "tflops": fl["bwd"] / (bwd_ms * 1e-3) / 1e12,
                "frac_mfma_peak": fl["bwd"] / (bwd_ms * 1e-3) / PEAK_BF16_MFMA},
        "per_call": per_call,
        "kernels": kernels,
        "roofline": roofline,
        "roofline_lowest_kernel": lowest,
        "roofline_per_kernel": {n: {"frac": r["frac"], "achieved": r["achieved"], "avg_ms": r["avg_ms"],
                                    "traffic": r["traffic"]} for n, r in per_kernel.items()},
    }

    if not args.no_decode:
        dcfg = synth.DECODE_CONFIGS["decode_b128_w512"]
        d = {n: t.cuda() for n, t in synth.make_decode_inputs(dcfg).items()}
        od = torch.empty_like(d["q"])
        dstep = lambda: rb.rattn_decode_step(d["q"], d["k_new"], d["v_new"], d["pos"], d["k_ring"], d["v_ring"],
                                             d["state"], softmax_scale=dcfg.scale, out=od)
        for _ in range(20):
            dstep()
        torch.cuda.synchronize()
        rb.rattn_profile_enable(True)
        nd = 50
        for _ in range(nd):
            dstep()
        torch.cuda.synchronize()
        drecs = [ms for n, ms in rb.rattn_profile_records() if n == "decode_kernel"]
        rb.rattn_profile_enable(False)
        us = sum(drecs) / len(drecs) * 1e3
        nbytes = decode_bytes(dcfg.N, dcfg.Hkv, dcfg.Hq, dcfg.D, dcfg.W, 2)
        out["decode"] = {"workload": dcfg.name, "us_per_step": us, "tokens_per_s": dcfg.N / (us * 1e-6),
                         # attention term of the generation step-time model (batch * cache bytes per sequence /
                         # memory bandwidth) at the MI355X peak, for this layer alone
                         "step_time_model_us": nbytes / PEAK_HBM * 1e6,
                         "roofline": {"bound": "hbm", "kernel": "decode_kernel", "achieved": nbytes / (us * 1e-6) / 1e9,
                                      "peak": PEAK_HBM / 1e9, "unit": "GB/s", "frac": nbytes / (us * 1e-6) / PEAK_HBM,
                                      "traffic": measured_traffic("decode_kernel", dcfg.name)[0],
                                      "traffic_source": measured_traffic("decode_kernel", dcfg.name)[1],
                                      "algorithmic_bytes": nbytes}}

    if not args.no_decode:
        # generation step-time model of the paper's inference analysis with MI355X figures (8 TB/s, 2.5 PFLOP/s
        # bf16), local:global 3:1 stacks, window 512 + state against sliding-window 4096; the measured decode
        # kernel turns the model's cache term for the local layers into a measured one
        def stack(layers, hkv, pcount, batch, ctx):
            swa = rb.rattn_cache_bytes(layers, 4, ctx, 4096, False, hkv, 128, 2)
            ratt = rb.rattn_cache_bytes(layers, 4, ctx, 512, True, hkv, 128, 2)
            t0 = rb.rattn_step_time_model(batch, swa, pcount, 2 * pcount, PEAK_HBM, PEAK_BF16_MFMA)
            t1 = rb.rattn_step_time_model(batch, ratt, pcount, 2 * pcount, PEAK_HBM, PEAK_BF16_MFMA)
            return {"batch": batch, "ctx": ctx, "swa4096_ms": t0 * 1e3, "rattn512_ms": t1 * 1e3, "gain": 1.0 - t1 / t0}
        out["step_time_model"] = {
            "hardware": {"bandwidth_GBps": PEAK_HBM / 1e9, "tflops": PEAK_BF16_MFMA / 1e12},
            "3B_56layers_4kv": [stack(56, 4, 3e9, b_, c_) for b_ in (1, 128) for c_ in (4096, 32768)],
            "12B_40layers_8kv": [stack(40, 8, 12e9, b_, c_) for b_ in (1, 128) for c_ in (4096, 32768)],
            "local_layer_cache_term_us": {"model_at_peak": out["decode"]["step_time_model_us"],
                                          "measured_kernel": out["decode"]["us_per_step"]}}

    if not args.no_decode and not args.no_prefill:
        # prefill -> decode hand-over on the layer's K/V (one-off per prompt; reported, not part of `value`)
        for _ in range(3):
            rb.rattn_prefill_export(k, v, cfg.W)
        torch.cuda.synchronize()
        rb.rattn_profile_enable(True)
        for _ in range(10):
            rb.rattn_prefill_export(k, v, cfg.W)
        torch.cuda.synchronize()
        per = {}
        for name, ms in rb.rattn_profile_records():
            if name.startswith("export_"):
                per.setdefault(name, []).append(ms)
        rb.rattn_profile_enable(False)
        out["prefill_export"] = {"workload": cfg.name, "us": {n_: sum(v_) / len(v_) * 1e3 for n_, v_ in per.items()},
                                 "us_total": sum(sum(v_) / len(v_) for v_ in per.values()) * 1e3}

        # chunked prefill: the second half of the layer's tokens given rings and state after the first half
        # (reported, not part of `value`); per-kernel averages and the whole call
        half = cfg.T // 2
        kr_, vr_, S_ = rb.rattn_prefill_export(k[:, :half].contiguous(), v[:, :half].contiguous(), cfg.W)
        qh, kh, vh = (t_[:, half:].contiguous() for t_ in (q, k, v))
        oh = torch.empty_like(qh)
        pc = rb.make_params(qh, kh, cfg.W, 0, cfg.scale, 1e-6, False)
        nb_ = ctypes.c_size_t()
        rb.lib().rattn_prefill_chunk_workspace_bytes(ctypes.byref(pc), half, ctypes.byref(nb_))
        wsc = torch.empty(nb_.value, dtype=torch.uint8, device="cuda")
        # every call advances rings and state by `half` tokens in place; the timing does not depend on their values
        chunk_call = lambda: rb.rattn_prefill_chunk(qh, kh, vh, cfg.W, half, kr_, vr_, S_, softmax_scale=cfg.scale,
                                                    workspace=wsc, out=oh)
        for _ in range(3):
            chunk_call()
        ms_chunk = timed(chunk_call, 10)
        rb.rattn_profile_enable(True)
        for _ in range(5):
            chunk_call()
        torch.cuda.synchronize()
        per = {}
        for name, ms in rb.rattn_profile_records():
            per.setdefault(name, []).append(ms)
        rb.rattn_profile_enable(False)
        out["prefill_chunk"] = {"workload": f"{cfg.name}: tokens {half}..{cfg.T - 1} after {half}",
                                "ms": ms_chunk, "tokens_per_s": cfg.B * half / (ms_chunk * 1e-3),
                                "us": {n_: sum(v_) / len(v_) * 1e3 for n_, v_ in per.items()}}
        del kr_, vr_, S_, qh, kh, vh, oh, wsc

    if not args.no_other_workloads:
        # reported next to the headline (never part of `value`): the 12B-shaped layer and the window
        # sweep at T = 8192 (fwd and bwd), same timing method, 20 iterations after 5 warm-up ones
        del q, k, v, dO, o, grads, saved, ws
        torch.cuda.empty_cache()
        other = {}

        def run_layer(c, with_bwd, gains=False, feature_map="softmax", chunk=0, state_policy="keep"):
            t = [x_.cuda() for x_ in synth.make_layer_inputs(c, with_dO=with_bwd)]
            gs_ = (1.0 + 0.1 * torch.randn(c.Hq, c.D, device="cuda")) if gains else None
            gr_ = (1.0 + 0.1 * torch.randn(c.Hq, c.D, device="cuda")) if gains else None
            pp = rb.make_params(t[0], t[1], c.W, chunk, c.scale, 1e-6, with_bwd, feature_map, "auto", state_policy)
            fb, bb, sb = rb.rattn_workspace_bytes(pp)
            w_ = torch.empty(max(fb, bb, 16), dtype=torch.uint8, device="cuda")
            sv_ = torch.empty(max(sb, 16), dtype=torch.uint8, device="cuda") if with_bwd else None
            o_ = torch.empty_like(t[0])
            g_ = (torch.empty_like(t[0]), torch.empty_like(t[1]), torch.empty_like(t[2])) if with_bwd else None
            f_ = lambda: rb.rattn_fwd(t[0], t[1], t[2], c.W, gs_, gr_, softmax_scale=c.scale, save_for_bwd=with_bwd,
                                      out=o_, saved=sv_, workspace=w_, feature_map=feature_map, chunk=chunk,
                                      state_policy=state_policy)
            b_ = lambda: rb.rattn_bwd(t[0], t[1], t[2], sv_, t[3], c.W, gs_, gr_, softmax_scale=c.scale,
                                      want_dgamma=gains, workspace=w_, out=g_, feature_map=feature_map, chunk=chunk,
                                      state_policy=state_policy)
            for _ in range(5):
                f_()
                if with_bwd:
                    b_()
            fl_ = layer_flops(c.B, c.T, c.Hq, c.Hkv, c.D, c.W)
            r = {"fwd_ms": timed(f_, 20)}
            r["fwd_tflops"] = fl_["fwd"] / (r["fwd_ms"] * 1e-3) / 1e12
            if with_bwd:
                r["bwd_ms"] = timed(b_, 20)
                r["bwd_tflops"] = fl_["bwd"] / (r["bwd_ms"] * 1e-3) / 1e12
                r["fwd_bwd_tflops"] = (fl_["fwd"] + fl_["bwd"]) / ((r["fwd_ms"] + r["bwd_ms"]) * 1e-3) / 1e12
            r["tokens_per_s"] = c.B * c.T / ((r["fwd_ms"] + r.get("bwd_ms", 0.0)) * 1e-3)
            r["saved_MB"] = sb / 1e6
            return r

        other["layer12b_t8192_w512"] = run_layer(synth.CONFIGS["layer12b_t8192_w512"], True)
        # the headline shape with the window read as 512 earlier tokens + the current one (not a tile multiple)
        other["layer3b_t4096_w513"] = run_layer(dataclasses.replace(cfg, name="layer3b_t4096_w513", W=513), True)
        # the headline shape with learned per-head RMS gains and their gradients (the headline itself has none),
        # and without them by the same (shorter) timing method for comparison
        other["layer3b_t4096_w512_gains"] = run_layer(cfg, True, gains=True)
        other["layer3b_t4096_w512"] = run_layer(cfg, True)
        # the ablation's ReLU and identity feature maps (Sec. 4.5) on the same kernels, same FLOP formula
        other["layer3b_t4096_w512_relu"] = run_layer(cfg, True, feature_map="relu")
        # (identity map: forward only - calls that keep `saved` for a backward pass run on the general kernels)
        other["layer3b_t4096_w512_identity_fwd_only"] = run_layer(cfg, False, feature_map="identity")
        # shapes that reach the matrix-core kernels through zero-padded copies: a ragged length (4000 -> 4096 rows)
        # and head size 64 (rows widened to 128 features; FLOPs counted at head size 64)
        other["layer3b_t4000_w512_ragged"] = run_layer(dataclasses.replace(cfg, name="layer3b_t4000_w512", T=4000), True)
        other["layer3b_t4096_w512_d64"] = run_layer(dataclasses.replace(cfg, name="layer3b_t4096_w512_d64", D=64,
                                                                        scale=0.125), True)
        for W_ in (128, 512, 1024, 4096, 8192):
            c_ = synth.sweep_config(W_)
            other[c_.name] = run_layer(c_, True)
        # The paper's search over what is stored of the chunk states and over the chunk size (Sec. 3.2, Fig. 3: best
        # setting ~15 % faster than storing every state at C = 256), on the matrix-core kernels: chunk states kept in
        # `saved` for backward (all of them, m = 1; every 2nd or 4th, m = 2, 4) or rebuilt there, chunk products of 128
        # or 64 keys; both benchmark layers, fwd + bwd
        search = {}
        for c_ in (cfg, synth.CONFIGS["layer12b_t8192_w512"]):
            rows = {}
            for pol in ("keep", "every2", "every4", "rebuild"):
                for ck in (128, 64):
                    r_ = run_layer(c_, True, chunk=ck, state_policy=pol)
                    rows[f"{pol}_C{ck}"] = {"fwd_ms": r_["fwd_ms"], "bwd_ms": r_["bwd_ms"],
                                            "step_ms": r_["fwd_ms"] + r_["bwd_ms"], "saved_MB": r_["saved_MB"]}
            best = min(rows, key=lambda n_: rows[n_]["step_ms"])
            worst = max(rows, key=lambda n_: rows[n_]["step_ms"])
            search[c_.name] = {"variants": rows, "best": best, "default": "keep_C128",
                               "best_over_worst_gain": rows[worst]["step_ms"] / rows[best]["step_ms"] - 1.0,
                               "saved_MB_not_kept": rows["keep_C128"]["saved_MB"] - rows["rebuild_C128"]["saved_MB"]}
        other["state_pipeline_search"] = search
        # chunk-size enumeration of the linear branch (Sec. 3.2's search over C) on the general kernels, which take the
        # chunk as a parameter (the matrix-core path fixes one state per 128 keys)
        xg = synth.make_random_layer(1, 4096, 8, 2, 64, "bf16", 11)
        qg, kg, vg = xg["q"].cuda(), xg["k"].cuda(), xg["v"].cuda()
        sweep_c = {}
        for c_ in (16, 32, 64, 128, 256, 512):
            fg = lambda: rb.rattn_fwd(qg, kg, vg, 512, chunk=c_, softmax_scale=0.125, kernel_path="general")
            for _ in range(3):
                fg()
            sweep_c[str(c_)] = timed(fg, 10)
        other["general_path_chunk_sweep_t4096_d64_fwd_ms"] = sweep_c
        out["other_workloads"] = other

    if machine is not None:
        machine["value_over_mfma_loop"] = value / machine["mfma_loop_tflops"]
        machine["roofline_achieved_over_mfma_loop"] = roofline["achieved"] / machine["mfma_loop_tflops"]
        out["machine"] = machine

    if args.calibrate_copy:
        src = torch.zeros(256 * 2 ** 20 // 4, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        out["calibration"] = {"kernel": "elementwise add, out-of-place", "bytes_read": src.numel() * 4,
                              "bytes_written": dst.numel() * 4}

    if cpu_base is not None:
        out["cpu_baseline"] = cpu_base
    print(json.dumps(out))


if __name__ == "__main__":
    main()

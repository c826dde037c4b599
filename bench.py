#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

One step = one pass of the whole hot path over one batch of seeded synthetic input:
  1. bf16 GEMM 4096^3: one warm launch, then uninstrumented / instrumented (all 4 regions, ring of
     4096 records per workgroup) launched alternately, two of each; then the same for the
     stage-by-stage schedule of the K step with its configured 5 regions (514 records per wave),
     and two launches each with a region masked off, with the constant-rate clock on top of that, with
     the 64-lane store (generic record sites) and with the flush strategy
  2. kp_trace_reduce of the GEMM trace
  3. causal attention forward 4x32x4096x128: warm launch, then uninstrumented / instrumented
     (3 regions, ring of 1024 records per workgroup, wraps) alternately, two of each
  4. kp_trace_reduce of the attention trace
  5. kp_trace_reduce of the standalone decode workload: 2^28 synthetic records
  6. kp_trace_pairs of the same records: one timeline row per paired region instance
  7. kp_trace_waits of the same records: the waits behind asynchronous operations
  8. kp_pairs_stages of the timeline rows: stage latency per (workgroup, region, iteration)
  9. kp_stages_critical of that table: the critical path of every workgroup
All inputs are resident in HBM before the timed region starts.  Every kernel is bracketed by
HIP events on the launch stream inside the timed region; the per-kernel figures below are
averages over the timed steps.

Prints ONE JSON line.  `value` is the instrumented GEMM's TFLOP/s (the metric's "instrumented
TFLOP/s"); the other halves of the metric are in `overhead_pct` and `decode_records_per_s`.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E
# HBM bytes per launch from hardware counters (FETCH_SIZE x 2.000 + WRITE_SIZE x 1.000 KiB, the factors
# read off a plain 1 GiB copy); procedure and readings are in profiles/pmc_hbm_traffic.md.
TRAFFIC_BYTES = {
    "decode_2^28": (1079450.8 * 2.0 + 37816.8) * 1024,
    "gemm_vanilla": (98365.0 * 2.0 + 32796.2) * 1024,
    "attn_vanilla": (196729.4 * 2.0 + 131100.3) * 1024,
    "timeline_2^28": (1057962.5 * 2.0 + 2085926.4) * 1024,
    "waits_2^28": (1056935.8 * 2.0 + 33216.0) * 1024,
    "stages_2^28": (1043570.7 * 2.0 + 274535.0) * 1024,
    "critical_2^28": (132139.5 * 2.0 + 992.0) * 1024,
}
DECODE_BYTES_PER_RECORD = 8.0 + 16.0 * 16 / 2048 + 128.0 / 16384  # record + per-(wg,wave,region) out + wg header


def cpu_baseline(args, inputs, a, b, q, k, v) -> dict:
    """The CPU oracle as it stands, timed on the host cores of the GPU machine on bounded samples of the
    benchmark's own workloads (about 10 s for the decoder, a few seconds for the others)."""
    import numpy as np

    import oracle

    host_cpus = os.cpu_count() or 1
    threads = min(host_cpus, 16)
    sample_log2 = min(args.log2_records, 23)
    sraw, _ = inputs.gen_trace(inputs.spec_decode_standalone(sample_log2))
    n = 1 << sample_log2

    def decode_rate(n_threads: int, budget_s: float, max_reps: int) -> tuple[float, int]:
        oracle.decode_bytes(sraw, n_threads)  # warm-up
        c0 = time.perf_counter()
        reps = 0
        while True:
            oracle.decode_bytes(sraw, n_threads)
            reps += 1
            if time.perf_counter() - c0 > budget_s or reps >= max_reps:
                break
        return reps * n / (time.perf_counter() - c0), reps

    multi, reps = decode_rate(threads, 10.0, 20)
    single, reps1 = decode_rate(1, 5.0, 2)
    # dense legs: 128 rows of the 4096^3 GEMM, 128 query rows of one attention head (numpy fp64)
    rows = np.arange(0, 4096, 32)
    c0 = time.perf_counter()
    oracle.ref_gemm(a, b, rows=rows)
    t_gemm = time.perf_counter() - c0
    rows_a = np.arange(31, 4096, 32)
    c0 = time.perf_counter()
    oracle.ref_attn(q[0, 0], k[0, 0], v[0, 0], causal=True, rows=rows_a)
    t_attn = time.perf_counter() - c0
    return {
        "value": round(multi, 1),
        "unit": "records/s (trace decode)",
        "cores": threads,
        "host_cpus": host_cpus,
        "kind": "oracle",
        "sample": f"{reps} x the first 2^{sample_log2} records' worth of the decode workload "
                  f"({n // 16384} workgroups x 8 waves x 2048 records), OpenMP over workgroups",
        "single_thread": {"value": round(single, 1), "unit": "records/s (trace decode)", "cores": 1,
                          "sample": f"{reps1} x the same 2^{sample_log2} records"},
        "gemm": {"value": round(2.0 * len(rows) * 4096 * 4096 / t_gemm / 1e9, 2), "unit": "GFLOP/s (fp64, numpy)",
                 "sample": f"{len(rows)} of the 4096 output rows of the 4096^3 GEMM (conversion to fp64 included)"},
        "attention": {"value": round(4.0 * float((rows_a + 1).sum()) * 128 / t_attn / 1e9, 2),
                      "unit": "GFLOP/s (fp64, numpy; causal FLOPs)",
                      "sample": f"{len(rows_a)} of the 4096 query rows of one (batch, head) of the attention workload"},
    }


def decode_steps(args) -> int:
    """Cost of every step of the decoder (profiles/decode_steps.md is this table)."""
    import numpy as np
    import torch

    import inputs
    import paper_2505_21661_amd as kp

    spec = inputs.spec_decode_standalone(args.log2_records)
    raw, _ = inputs.gen_trace(spec)
    n = spec.n_slots
    dev_raw = torch.from_numpy(raw.view(np.int32)).cuda()
    out = torch.zeros(kp.kp_stats_bytes(spec.n_wg, spec.waves, spec.n_regions), dtype=torch.uint8, device="cuda")
    hdr = kp.make_hdr(spec.n_wg, spec.waves, spec.n_regions, spec.cap_wave)

    def timed(f, reps=10):
        for _ in range(2):
            f()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            f()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    steps = ["records ordered by sequence number (load, scatter by rank)", "paired, durations and histogram",
             "paired records counted into time cells", "prefix sum over the cells", "records placed cell by cell",
             "ranked inside their cell (only without the register sort)", "sorted sequence written (likewise)",
             "register sort of the windows, region-pair overlap"]
    rows, prev = [], 0.0
    for i, what in enumerate(steps, 1):
        t = timed(lambda: kp.kp_trace_reduce_steps(dev_raw, n, hdr, out, i))
        rows.append({"step": i, "what": what, "ms_up_to_here": round(t, 4), "ms_of_step": round(t - prev, 4)})
        prev = t
    full = timed(lambda: kp.kp_trace_reduce_hdr(dev_raw, n, hdr, out))
    rows.append({"step": 9, "what": "per-(workgroup, wave, region) output, totals, init and finalize kernels",
                 "ms_up_to_here": round(full, 4), "ms_of_step": round(full - prev, 4)})
    del dev_raw, out
    # the multi-pass kernel for geometries outside the LDS-resident one's: same recipe, 2^26 record slots
    wide = []
    for W, R, cap in ((8, 16, 8192), (16, 16, 32768), (8, 64, 2048), (8, 128, 2048), (16, 128, 8192)):
        ws = wide_spec(W, R, cap, 26)
        wraw, _ = inputs.gen_trace(ws)
        wdev = torch.from_numpy(wraw.view(np.int32)).cuda()
        wout = torch.zeros(kp.kp_stats_bytes(ws.n_wg, W, R), dtype=torch.uint8, device="cuda")
        whdr = kp.make_hdr(ws.n_wg, W, R, cap)
        t = timed(lambda: kp.kp_trace_reduce_hdr(wdev, ws.n_slots, whdr, wout), reps=5)
        wide.append({"waves": W, "n_regions": R, "cap_wave": cap, "n_wg": ws.n_wg, "ms": round(t, 3),
                     "hbm_frac": round(8.0 * ws.n_slots / (t * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)})
        del wdev, wout, wraw
    print(json.dumps({"records": n, "steps": rows, "hbm_frac": round(DECODE_BYTES_PER_RECORD * n / (full * 1e-3) / 1e9
                                                                      / PEAK_HBM_GBS, 4), "wide_geometries_2^26": wide}))
    return 0


def wide_spec(W: int, R: int, cap: int, log2_records: int):
    """The standalone decode recipe at another geometry (for the decoder's multi-pass kernel)."""
    import dataclasses

    import inputs

    base = inputs.spec_decode_standalone(log2_records)
    return dataclasses.replace(base, n_wg=(1 << log2_records) // (W * cap), waves=W, n_regions=R, cap_wave=cap,
                               total_per_wave=cap)


def probe(args) -> int:
    """Every hot kernel twice (the second launch is the one to read), after a plain 1 GiB copy that scales
    the HBM counters: FETCH_SIZE / WRITE_SIZE are reported in KiB per dispatch; divide a kernel's reading by
    the copy kernel's reading per GiB to get bytes."""
    import numpy as np
    import torch

    import inputs
    import paper_2505_21661_amd as kp

    dev = "cuda"
    src = torch.arange(1 << 28, dtype=torch.int32, device=dev)  # 1 GiB
    dst = torch.empty_like(src)
    for _ in range(2):
        torch.add(src, 1, out=dst)  # one elementwise kernel: reads 1 GiB, writes 1 GiB
    torch.cuda.synchronize()
    del src, dst
    M = N = K = 4096
    a, b = inputs.gemm_inputs(M, N, K, seed=2)
    A, B = a.to(dev), b.to(dev)
    C = torch.empty(M, N, dtype=torch.bfloat16, device=dev)
    n_wg, waves, R = kp.kp_gemm_launch_shape(M, N, K)
    trace = torch.zeros(kp.kp_trace_bytes(n_wg, waves, 4096), dtype=torch.uint8, device=dev)
    for mask in (0, 0b1111, kp.KP_MASK_PHASES, kp.KP_MASK_PHASES | 0b11111):
        for _ in range(2):
            kp.kp_gemm_instrumented(A, B, C, M, N, K, mask, trace if mask & 31 else None, 4096 if mask & 31 else 0)
    torch.cuda.synchronize()
    Bt, H, S, D = 4, 32, 4096, 128
    q, k, v = inputs.attn_inputs(Bt, H, S, D, seed=3)
    Q, Kt, V = q.to(dev), k.to(dev), v.to(dev)
    O = torch.empty_like(Q)
    for _ in range(2):
        kp.kp_attn_instrumented(Q, Kt, V, O, Bt, H, S, D, True, 1.0 / math.sqrt(D), 0, None, 0)
    torch.cuda.synchronize()
    spec = inputs.spec_decode_standalone(args.log2_records)
    raw, _ = inputs.gen_trace(spec)
    n = spec.n_slots
    d_raw = torch.from_numpy(raw.view(np.int32)).to(dev)
    hdr = kp.make_hdr(spec.n_wg, spec.waves, spec.n_regions, spec.cap_wave)
    stats = torch.zeros(kp.kp_stats_bytes(spec.n_wg, spec.waves, spec.n_regions), dtype=torch.uint8, device=dev)
    pairs = torch.empty(kp.kp_pairs_bytes(spec.n_wg, spec.waves, spec.waves * spec.cap_wave), dtype=torch.uint8, device=dev)
    waits = torch.empty(kp.kp_waits_bytes(spec.n_wg, spec.waves, spec.n_regions), dtype=torch.uint8, device=dev)
    stages = torch.empty(kp.kp_stages_bytes(spec.n_wg, spec.n_regions, 64), dtype=torch.uint8, device=dev)
    paths = torch.empty(kp.kp_critical_bytes(spec.n_wg, spec.n_regions), dtype=torch.uint8, device=dev)
    for _ in range(2):
        kp.kp_trace_reduce_hdr(d_raw, n, hdr, stats)
    for _ in range(2):
        kp.kp_trace_pairs_hdr(d_raw, n, hdr, pairs)
    for _ in range(2):
        kp.kp_trace_waits_hdr(d_raw, n, hdr, waits)
    for _ in range(2):
        kp.kp_pairs_stages(pairs, spec.n_wg, spec.waves, spec.waves * spec.cap_wave, spec.n_regions, 64, stages)
    for _ in range(2):
        kp.kp_stages_critical(stages, spec.n_wg, spec.n_regions, 64, paths)
    torch.cuda.synchronize()
    del d_raw, stats, pairs, waits, stages, paths
    ws = wide_spec(8, 16, 8192, min(args.log2_records, 26))  # the decoder's multi-pass kernel
    wraw, _ = inputs.gen_trace(ws)
    wdev = torch.from_numpy(wraw.view(np.int32)).to(dev)
    wstats = torch.zeros(kp.kp_stats_bytes(ws.n_wg, ws.waves, ws.n_regions), dtype=torch.uint8, device=dev)
    for _ in range(2):
        kp.kp_trace_reduce_hdr(wdev, ws.n_slots, kp.make_hdr(ws.n_wg, ws.waves, ws.n_regions, ws.cap_wave), wstats)
    torch.cuda.synchronize()
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--log2-records", type=int, default=28, help="size of the standalone decode workload")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--decode-steps", action="store_true",
                    help="instead of the benchmark: time the decoder cut short after each of its steps "
                         "(kp_trace_reduce_steps) and print the cost of every step")
    ap.add_argument("--probe", action="store_true",
                    help="instead of the benchmark: launch every hot kernel twice, after a 1 GiB copy, "
                         "for hardware-counter runs (rocprofv3 --pmc ... -- python3 bench.py --probe)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2
    if args.decode_steps:
        return decode_steps(args)
    if args.probe:
        return probe(args)

    import numpy as np
    import torch

    import inputs
    import paper_2505_21661_amd as kp
    from paper_2505_21661_amd import model

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    kp.lib()  # fails loudly if libkperf.so is missing
    dev = "cuda"

    # ---- resident inputs ------------------------------------------------------------------
    M = N = K = 4096
    a, b = inputs.gemm_inputs(M, N, K, seed=2)
    A, Bm = a.to(dev), b.to(dev)
    C = torch.empty(M, N, dtype=torch.bfloat16, device=dev)
    g_wg, g_waves, g_R = kp.kp_gemm_launch_shape(M, N, K)
    g_cap = 4096
    g_trace = torch.zeros(kp.kp_trace_bytes(g_wg, g_waves, g_cap), dtype=torch.uint8, device=dev)
    g_stats = torch.zeros(kp.kp_stats_bytes(g_wg, g_waves, g_R), dtype=torch.uint8, device=dev)
    g_hdr = kp.make_hdr(g_wg, g_waves, g_R, g_cap // g_waves)

    Bt, H, S, D = 4, 32, 4096, 128
    q, k, v = inputs.attn_inputs(Bt, H, S, D, seed=3)
    Q, Kt, V = q.to(dev), k.to(dev), v.to(dev)
    O = torch.empty_like(Q)
    a_wg, a_waves, a_R = kp.kp_attn_launch_shape(Bt, H, S, D)
    a_cap = 1024
    a_trace = torch.zeros(kp.kp_trace_bytes(a_wg, a_waves, a_cap), dtype=torch.uint8, device=dev)
    a_stats = torch.zeros(kp.kp_stats_bytes(a_wg, a_waves, a_R), dtype=torch.uint8, device=dev)
    a_hdr = kp.make_hdr(a_wg, a_waves, a_R, a_cap // a_waves)
    scale = 1.0 / math.sqrt(D)

    spec = inputs.spec_decode_standalone(args.log2_records)
    raw, _ = inputs.gen_trace(spec)
    d_n = spec.n_slots
    d_raw = torch.from_numpy(raw.view(np.int32)).to(dev)
    d_stats = torch.zeros(kp.kp_stats_bytes(spec.n_wg, spec.waves, spec.n_regions), dtype=torch.uint8, device=dev)
    d_hdr = kp.make_hdr(spec.n_wg, spec.waves, spec.n_regions, spec.cap_wave)
    d_pairs = torch.empty(kp.kp_pairs_bytes(spec.n_wg, spec.waves, spec.waves * spec.cap_wave), dtype=torch.uint8,
                          device=dev)
    d_waits = torch.empty(kp.kp_waits_bytes(spec.n_wg, spec.waves, spec.n_regions), dtype=torch.uint8, device=dev)
    d_iters = 64  # iterations kept per region: the workload runs about 64 pairs per wave and region
    d_stages = torch.empty(kp.kp_stages_bytes(spec.n_wg, spec.n_regions, d_iters), dtype=torch.uint8, device=dev)
    d_paths = torch.empty(kp.kp_critical_bytes(spec.n_wg, spec.n_regions), dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()

    # The dense kernels run after one warm launch (the preceding decode of a 2 GiB trace leaves L2 and
    # the memory-side cache cold) in the order vanilla, instrumented, instrumented, vanilla: the chip's
    # clock sags over a burst of MFMA kernels, and in this order both kinds sit at the same mean
    # position in the burst; every launch is inside the timed step.  The sag outlasts the burst: the
    # statistics decoder takes 1.78 ms in a step without the dense kernels, 1.89 ms right behind them and
    # 1.82 ms as the last leg of the step, behind the other four trace kernels, where it runs here.
    names = ["gemm_warm", "gemm_vanilla", "gemm_instr", "gemm_instr2", "gemm_vanilla2", "gemm_reduce",
             "gemm5_unfenced", "gemm5_vanilla", "gemm5_instr", "gemm5_instr2", "gemm5_vanilla2", "gemm5_unfenced2", "gemm_masked", "gemm_collab", "gemm_realtime",
             "gemm_flush", "gemm_flush2", "gemm_realtime2", "gemm_collab2", "gemm_masked2",
             "attn_warm", "attn_vanilla", "attn_instr", "attn_instr2", "attn_vanilla2", "attn_reduce",
             "timeline", "waits", "stages", "critical", "decode"]

    def step(events=None, main_events=None):
        gemm_v = lambda: kp.kp_gemm_instrumented(A, Bm, C, M, N, K, 0, None, 0)
        gemm_i = lambda: kp.kp_gemm_instrumented(A, Bm, C, M, N, K, 0b1111, g_trace, g_cap)
        gemm5_v = lambda: kp.kp_gemm_instrumented(A, Bm, C, M, N, K, kp.KP_MASK_PHASES, None, 0)
        gemm5_u = lambda: kp.kp_gemm_instrumented(A, Bm, C, M, N, K, kp.KP_MASK_PHASES | kp.KP_MASK_UNFENCED, None, 0)
        gemm5_i = lambda: kp.kp_gemm_instrumented(A, Bm, C, M, N, K, 0b11111 | kp.KP_MASK_PHASES, g_trace, g_cap)
        gemm_m = lambda: kp.kp_gemm_instrumented(A, Bm, C, M, N, K, 0b1011, g_trace, g_cap)
        gemm_c = lambda: kp.kp_gemm_instrumented(A, Bm, C, M, N, K, 0b1011 | kp.KP_MASK_COLLAB, g_trace, g_cap)
        gemm_r = lambda: kp.kp_gemm_instrumented(A, Bm, C, M, N, K, 0b1011 | kp.KP_MASK_REALTIME, g_trace, g_cap)
        gemm_f = lambda: kp.kp_gemm_instrumented(A, Bm, C, M, N, K, 0b1111 | kp.KP_MASK_FLUSH, g_trace, g_cap)
        attn_v = lambda: kp.kp_attn_instrumented(Q, Kt, V, O, Bt, H, S, D, True, scale, 0, None, 0)
        attn_i = lambda: kp.kp_attn_instrumented(Q, Kt, V, O, Bt, H, S, D, True, scale, 0b111, a_trace, a_cap)
        calls = (
            gemm_v, gemm_v, gemm_i, gemm_i, gemm_v,
            lambda: kp.kp_trace_reduce_hdr(g_trace, g_wg * g_cap, g_hdr, g_stats),
            gemm5_u, gemm5_v, gemm5_i, gemm5_i, gemm5_v, gemm5_u, gemm_m, gemm_c, gemm_r, gemm_f, gemm_f, gemm_r, gemm_c, gemm_m,
            attn_v, attn_v, attn_i, attn_i, attn_v,
            lambda: kp.kp_trace_reduce_hdr(a_trace, a_wg * a_cap, a_hdr, a_stats),
            lambda: kp.kp_trace_pairs_hdr(d_raw, d_n, d_hdr, d_pairs),
            lambda: kp.kp_trace_waits_hdr(d_raw, d_n, d_hdr, d_waits),
            lambda: kp.kp_pairs_stages(d_pairs, spec.n_wg, spec.waves, spec.waves * spec.cap_wave, spec.n_regions,
                                       d_iters, d_stages),
            lambda: kp.kp_stages_critical(d_stages, spec.n_wg, spec.n_regions, d_iters, d_paths),
            # (the decoder's main kernel between two events of its own: the call is three kernels)
            (lambda: kp.kp_trace_reduce_hdr(d_raw, d_n, d_hdr, d_stats)) if main_events is None else
            (lambda: kp.kp_trace_reduce_hdr_events(d_raw, d_n, d_hdr, d_stats, main_events[0], main_events[1])),
        )
        for i, call in enumerate(calls):
            if events is not None:
                events[i][0].record()
            call()
            if events is not None:
                events[i][1].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    all_events = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in names]
                  for _ in range(args.steps)]
    main_events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for pair in main_events:  # (an event has a handle to pass to the library once it has been recorded)
        pair[0].record()
        pair[1].record()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(all_events[s], main_events[s])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    ms = {n: float(np.mean([all_events[s][i][0].elapsed_time(all_events[s][i][1]) for s in range(args.steps)]))
          for i, n in enumerate(names)}

    for base in ("gemm", "gemm5", "attn"):
        ms[base + "_vanilla"] = 0.5 * (ms[base + "_vanilla"] + ms.pop(base + "_vanilla2"))
        ms[base + "_instr"] = 0.5 * (ms[base + "_instr"] + ms.pop(base + "_instr2"))
    gemm_flop = 2.0 * M * N * K
    attn_flop = 4.0 * Bt * H * S * S * D / 2.0
    tf_van = gemm_flop / ms["gemm_vanilla"] / 1e9
    tf_ins = gemm_flop / ms["gemm_instr"] / 1e9
    overhead = (ms["gemm_instr"] - ms["gemm_vanilla"]) / ms["gemm_vanilla"] * 100.0
    overhead5 = (ms["gemm5_instr"] - ms["gemm5_vanilla"]) / ms["gemm5_vanilla"] * 100.0
    for leg in ("gemm_masked", "gemm_collab", "gemm_realtime", "gemm_flush", "gemm5_unfenced"):
        ms[leg] = 0.5 * (ms[leg] + ms.pop(leg + "2"))
    overhead_masked = (ms["gemm_masked"] - ms["gemm_vanilla"]) / ms["gemm_vanilla"] * 100.0
    attn_tf_van = attn_flop / ms["attn_vanilla"] / 1e9
    attn_tf_ins = attn_flop / ms["attn_instr"] / 1e9
    attn_overhead = (ms["attn_instr"] - ms["attn_vanilla"]) / ms["attn_vanilla"] * 100.0
    ms["decode_main_kernel"] = float(np.mean([b.elapsed_time(e) for b, e in main_events]))
    dec_rps = d_n / (ms["decode"] * 1e-3)  # the whole call: clearing, replay and finalize kernels
    dec_gbs = DECODE_BYTES_PER_RECORD * d_n / (ms["decode_main_kernel"] * 1e-3) / 1e9  # the replay kernel alone

    st = kp.parse_stats(d_stats)
    assert st["status"] == 0 and st["n_slots_valid"] == d_n, "decode workload did not decode"
    # timeline rows of the same trace: 8 B read per record, 16 B written per pair, 4 B per (wg, wave)
    n_seg = spec.n_wg * spec.waves
    pair_count = d_pairs[: 4 * n_seg].view(torch.int32).sum(dtype=torch.int64).item()
    assert pair_count == st["n_pairs"], "timeline rows and statistics disagree on the number of pairs"
    tl_bytes = 8.0 * d_n + 16.0 * pair_count + 4.0 * n_seg + 128.0 * spec.n_wg
    tl_gbs = tl_bytes / (ms["timeline"] * 1e-3) / 1e9
    # waits of the same trace: 8 B read per record, 16 B written per (wg, wave, region)
    wv = kp.parse_waits(d_waits)
    assert wv["n_wg"] == spec.n_wg and 0 < wv["n_waits"] <= st["n_pairs"] + st["n_orphan_end"], "waits block is off"
    wt_bytes = 8.0 * d_n + 16.0 * n_seg * spec.n_regions + 128.0 * spec.n_wg
    wt_gbs = wt_bytes / (ms["waits"] * 1e-3) / 1e9
    # stage table: 16 B read per row, 4 B per (wg, wave), 16 B written per (wg, region, iteration)
    sg_hdr = d_stages[:32].view(torch.int64).tolist()
    assert sg_hdr[0] + sg_hdr[1] == pair_count and sg_hdr[2] == 0, "stage table lost rows"
    sg_bytes = 16.0 * pair_count + 4.0 * n_seg + 16.0 * spec.n_wg * spec.n_regions * d_iters
    sg_gbs = sg_bytes / (ms["stages"] * 1e-3) / 1e9
    # critical path: 16 B read per (wg, region, iteration), 32 B written per workgroup
    cp_hdr, cp_region, _ = kp.parse_critical(d_paths, spec.n_wg, spec.n_regions)
    assert cp_hdr["n_paths"] == spec.n_wg and cp_hdr["n_path_stages"] == int(cp_region[:, 0].sum()), "critical-path block is off"
    cp_bytes = 16.0 * spec.n_wg * spec.n_regions * d_iters + 32.0 * spec.n_wg
    cp_gbs = cp_bytes / (ms["critical"] * 1e-3) / 1e9

    # Overhead model of the paper, eq. (1): T_theoretical = T_vanilla + N_record * Cycle_record, with the
    # per-record cost taken from the calibration kernel (an empty START/END region, i.e. two records)
    # and the tick rate of s_memtime from the constant-rate clock sampled over the same spans.
    c_wg, c_waves = 1024, 4
    c_trace = torch.zeros(kp.kp_trace_bytes(c_wg, c_waves, 16), dtype=torch.uint8, device=dev)
    kp.kp_calibrate([0, 4096], c_wg, c_waves, 0, c_trace, 16)
    c_stats = torch.zeros(kp.kp_stats_bytes(c_wg, c_waves, 2), dtype=torch.uint8, device=dev)
    kp.kp_trace_reduce(c_trace, c_wg * 16, c_stats)
    torch.cuda.synchronize()
    cst = kp.parse_stats(c_stats)
    pair_cost = float(np.median(cst["per"]["sum"][:, :, 0]))
    chdr = c_trace.cpu().numpy().view(np.uint32)[16:16 + 32 * c_wg].reshape(c_wg, 32).astype(np.uint64)
    c_span = ((chdr[:, 4] | (chdr[:, 5] << np.uint64(32))) - (chdr[:, 2] | (chdr[:, 3] << np.uint64(32)))).astype(np.float64)
    c_rt = (chdr[:, 6] | (chdr[:, 7] << np.uint64(32))).astype(np.float64)
    tick_hz = 100e6 * c_span.sum() / c_rt.sum()
    n_record = 2 * 3 * (K // 64) + 2
    t_vanilla_ticks = ms["gemm_vanilla"] * 1e-3 * tick_hz
    eq1 = {
        "n_record_per_wave": n_record,
        "cycle_record": round(pair_cost / 2.0, 1),
        "s_memtime_hz": round(tick_hz),
        "t_vanilla_ticks": round(t_vanilla_ticks),
        "t_theoretical_ticks": round(model.theoretical_ticks(t_vanilla_ticks, n_record, pair_cost / 2.0)),
        "t_actual_ticks": round(ms["gemm_instr"] * 1e-3 * tick_hz),
        "note": "cycle_record is the back-to-back cost (it includes the s_memtime round trip); sites "
                "inside long regions overlap most of it, so the actual time stays below the model",
    }

    out = {
        "metric": "instrumentation overhead % + instrumented TFLOP/s; trace-decode records/s (HBM %)",
        "value": round(tf_ins, 2),
        "unit": "TFLOP/s (instrumented bf16 GEMM 4096^3)",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": "instrumented bf16 GEMM M=N=K=4096 (256x256x64 tiles, 4 regions, ring 4096 rec/WG) "
                        "+ causal attention 4x32x4096x128 (3 regions, ring 1024 rec/WG) "
                        f"+ trace decode of 2^{args.log2_records} synthetic records (16384 WG x 8 waves x 16 regions at 2^28)",
            "decode_entry_point": "kp_trace_reduce_hdr_events",
        },
        "overhead_pct": round(overhead, 3),
        "overhead_pct_stage_by_stage": {
            "value": round(overhead5, 3),
            "what": "K step with its stages one after the other, 5 regions (load issue, wait, LDS write, MFMA, "
                    "epilogue), 514 records per wave; against the same schedule without record sites, i.e. with a "
                    "bare scheduling fence wherever the instrumented kernel has a site (a site pins its place in the "
                    "instruction stream; without the fences the compiler threads the stages through one another again)",
            "uninstrumented_tflops": round(gemm_flop / ms["gemm5_vanilla"] / 1e9, 2),
            "instrumented_tflops": round(gemm_flop / ms["gemm5_instr"] / 1e9, 2),
            "unfenced_uninstrumented_tflops": round(gemm_flop / ms["gemm5_unfenced"] / 1e9, 2),
            "overhead_pct_against_unfenced": round((ms["gemm5_instr"] - ms["gemm5_unfenced"]) / ms["gemm5_unfenced"] * 100.0, 3),
        },
        "overhead_pct_masked_sites": {
            "value": round(overhead_masked, 3),
            "what": "default schedule with region 2 masked off (region_mask 0b1011): the loop still keeps only the "
                    "clocks of its sites, and the mask decides which records are made from them when the trace is "
                    "copied out (a region mask, wave-group records and the constant-rate clock all keep that form)",
            "with_constant_rate_clock": round((ms["gemm_realtime"] - ms["gemm_vanilla"]) / ms["gemm_vanilla"] * 100.0, 3),
        },
        "overhead_pct_generic_sites": {
            "what": "the generic record sites (a site writes its records to LDS at the next site), which the 64-lane store of "
                    "Sec. 4.2 (KP_MASK_COLLAB, region_mask 0b1011, hardware ids in the workgroup header) and the "
                    "flush strategy (KP_MASK_FLUSH, all regions, 64-slot sub-rings copied out when full) need",
            "with_64_lane_store_and_hw_ids": round((ms["gemm_collab"] - ms["gemm_vanilla"]) / ms["gemm_vanilla"] * 100.0, 3),
            "flush_strategy": round((ms["gemm_flush"] - ms["gemm_vanilla"]) / ms["gemm_vanilla"] * 100.0, 3),
        },
        "uninstrumented_tflops": round(tf_van, 2),
        "uninstrumented_frac_of_mfma_peak": round(tf_van / PEAK_BF16_TFLOPS, 4),
        "instrumented_frac_of_mfma_peak": round(tf_ins / PEAK_BF16_TFLOPS, 4),
        "attn_overhead_pct": round(attn_overhead, 3),
        "attn_uninstrumented_tflops": round(attn_tf_van, 2),
        "attn_instrumented_tflops": round(attn_tf_ins, 2),
        "decode_records_per_s": round(dec_rps, 1),
        "decode_hbm_frac": round(dec_gbs / PEAK_HBM_GBS, 4),
        "timeline_records_per_s": round(d_n / (ms["timeline"] * 1e-3), 1),
        "waits_records_per_s": round(d_n / (ms["waits"] * 1e-3), 1),
        "stages_rows_per_s": round(pair_count / (ms["stages"] * 1e-3), 1),
        "critical_stages_per_s": round(spec.n_wg * spec.n_regions * d_iters / (ms["critical"] * 1e-3), 1),
        "critical_path": {"stages_on_paths": cp_hdr["n_path_stages"], "mean_stages_per_workgroup": round(cp_hdr["n_path_stages"] / spec.n_wg, 1),
                          "bubble_share": round(cp_hdr["sum_bubbles"] / max(1, cp_hdr["sum_bubbles"] + cp_hdr["sum_latency"]), 4)},
        "kernel_ms": {n: round(x, 4) for n, x in ms.items()},
        "overhead_model_eq1": eq1,
        "paper_context": {"overhead_pct": 8.2, "hardware": "H100 / MI300X (not split), Triton GEMM/FA3"},
        # dominant kernel of the step by time: the decoder's main kernel
        "roofline": {
            "kernel": "kp_reduce_main (trace decode)",
            "bound": "hbm",
            "achieved": round(dec_gbs, 2),
            "peak": PEAK_HBM_GBS,
            "unit": "GB/s",
            "frac": round(dec_gbs / PEAK_HBM_GBS, 4),
            "algorithmic_bytes": round(DECODE_BYTES_PER_RECORD * d_n),
            "traffic": round(TRAFFIC_BYTES["decode_2^28"]) if args.log2_records == 28 else None,
        },
        "roofline_gemm": {
            "kernel": "kp_gemm_big<false> (uninstrumented 4096^3)",
            "bound": "mfma",
            "achieved": round(tf_van, 2),
            "peak": PEAK_BF16_TFLOPS,
            "unit": "TFLOP/s",
            "frac": round(tf_van / PEAK_BF16_TFLOPS, 4),
            "traffic": round(TRAFFIC_BYTES["gemm_vanilla"]),
        },
        "roofline_attn": {
            "kernel": "kp_attn_fwd<false> (uninstrumented)",
            "bound": "mfma",
            "achieved": round(attn_tf_van, 2),
            "peak": PEAK_BF16_TFLOPS,
            "unit": "TFLOP/s",
            "frac": round(attn_tf_van / PEAK_BF16_TFLOPS, 4),
            "traffic": round(TRAFFIC_BYTES["attn_vanilla"]),
        },
        "roofline_timeline": {
            "kernel": "kp_pairs_main (timeline rows of the decode workload)",
            "bound": "hbm",
            "achieved": round(tl_gbs, 2),
            "peak": PEAK_HBM_GBS,
            "unit": "GB/s",
            "frac": round(tl_gbs / PEAK_HBM_GBS, 4),
            "algorithmic_bytes": round(tl_bytes),
            "traffic": round(TRAFFIC_BYTES["timeline_2^28"]) if args.log2_records == 28 else None,
        },
        "roofline_waits": {
            "kernel": "kp_waits_main (asynchronous waits of the decode workload)",
            "bound": "hbm",
            "achieved": round(wt_gbs, 2),
            "peak": PEAK_HBM_GBS,
            "unit": "GB/s",
            "frac": round(wt_gbs / PEAK_HBM_GBS, 4),
            "algorithmic_bytes": round(wt_bytes),
            "traffic": round(TRAFFIC_BYTES["waits_2^28"]) if args.log2_records == 28 else None,
        },
        "roofline_stages": {
            "kernel": "kp_stages_main (stage table from the timeline rows of the decode workload)",
            "bound": "hbm",
            "achieved": round(sg_gbs, 2),
            "peak": PEAK_HBM_GBS,
            "unit": "GB/s",
            "frac": round(sg_gbs / PEAK_HBM_GBS, 4),
            "algorithmic_bytes": round(sg_bytes),
            "traffic": round(TRAFFIC_BYTES["stages_2^28"]) if args.log2_records == 28 else None,
        },
        "roofline_critical": {
            "kernel": "kp_critical_main (critical path of every workgroup over that stage table)",
            "bound": "hbm",
            "achieved": round(cp_gbs, 2),
            "peak": PEAK_HBM_GBS,
            "unit": "GB/s",
            "frac": round(cp_gbs / PEAK_HBM_GBS, 4),
            "algorithmic_bytes": round(cp_bytes),
            "traffic": round(TRAFFIC_BYTES["critical_2^28"]) if args.log2_records == 28 else None,
        },
    }

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args, inputs, a, b, q, k, v)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())

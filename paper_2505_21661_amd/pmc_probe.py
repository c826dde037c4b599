"""Workload for hardware-counter runs (HBM traffic of the hot kernels).

Launches, in this order and twice each (the second launch is the one to read):
  a plain device-to-device copy of 1 GiB (reads 1 GiB, writes 1 GiB: the scale reference),
  the uninstrumented and the instrumented 4096^3 GEMM,
  the uninstrumented attention forward 4x32x4096x128,
  kp_trace_reduce_hdr, kp_trace_pairs_hdr, kp_trace_waits_hdr and kp_pairs_stages on the standalone
  decode workload (2^LOG2 records, default 28).

Run it under the profiler once per counter, e.g.
  rocprofv3 --pmc FETCH_SIZE --output-format csv -d out_fetch -- python3 -m paper_2505_21661_amd.pmc_probe
  rocprofv3 --pmc WRITE_SIZE --output-format csv -d out_write -- python3 -m paper_2505_21661_amd.pmc_probe
FETCH_SIZE / WRITE_SIZE are reported in KiB per dispatch; divide a kernel's reading by the copy
kernel's reading per GiB to get bytes.
"""
from __future__ import annotations

import math
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main() -> None:
    import numpy as np
    import torch

    import inputs
    import paper_2505_21661_amd as kp

    log2n = int(sys.argv[1]) if len(sys.argv) > 1 else 28
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
    for _ in range(2):
        kp.kp_gemm_instrumented(A, B, C, M, N, K, 0, None, 0)
    for _ in range(2):
        kp.kp_gemm_instrumented(A, B, C, M, N, K, 0b1111, trace, 4096)
    torch.cuda.synchronize()

    Bt, H, S, D = 4, 32, 4096, 128
    q, k, v = inputs.attn_inputs(Bt, H, S, D, seed=3)
    Q, Kt, V = q.to(dev), k.to(dev), v.to(dev)
    O = torch.empty_like(Q)
    for _ in range(2):
        kp.kp_attn_instrumented(Q, Kt, V, O, Bt, H, S, D, True, 1.0 / math.sqrt(D), 0, None, 0)
    torch.cuda.synchronize()
    del Q, Kt, V, O

    spec = inputs.spec_decode_standalone(log2n)
    raw, _ = inputs.gen_trace(spec)
    d_raw = torch.from_numpy(raw.view(np.int32)).to(dev)
    stats = torch.zeros(kp.kp_stats_bytes(spec.n_wg, spec.waves, spec.n_regions), dtype=torch.uint8, device=dev)
    hdr = kp.make_hdr(spec.n_wg, spec.waves, spec.n_regions, spec.cap_wave)
    for _ in range(2):
        kp.kp_trace_reduce_hdr(d_raw, spec.n_slots, hdr, stats)
    rows = torch.empty(kp.kp_pairs_bytes(spec.n_wg, spec.waves, spec.waves * spec.cap_wave), dtype=torch.uint8, device=dev)
    for _ in range(2):
        kp.kp_trace_pairs_hdr(d_raw, spec.n_slots, hdr, rows)
    waits = torch.empty(kp.kp_waits_bytes(spec.n_wg, spec.waves, spec.n_regions), dtype=torch.uint8, device=dev)
    for _ in range(2):
        kp.kp_trace_waits_hdr(d_raw, spec.n_slots, hdr, waits)
    stages = torch.empty(kp.kp_stages_bytes(spec.n_wg, spec.n_regions, 64), dtype=torch.uint8, device=dev)
    for _ in range(2):
        kp.kp_pairs_stages(rows, spec.n_wg, spec.waves, spec.waves * spec.cap_wave, spec.n_regions, 64, stages)
    torch.cuda.synchronize()
    print("pmc_probe done")


if __name__ == "__main__":
    main()

"""The asynchronous entry points record into a HIP graph: one instrumented GEMM, the decode of its
trace, its timeline rows, wait replay and stage table are captured once and replayed several times,
with eager work and synchronisations in between; every replay must reproduce the eager results
(the trace differs from launch to launch, so the decoded blocks are compared with the oracle run on
that replay's own trace)."""
import numpy as np
import pytest

import inputs

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def test_record_and_decode_replay_in_a_graph(oracle_mod):
    import paper_2505_21661_amd as kp

    M = N = 1024
    K = 256
    a, b = inputs.gemm_inputs(M, N, K, seed=11)
    A, B = a.cuda(), b.cuda()
    C = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    C_ref = torch.empty_like(C)
    n_wg, waves, R = kp.kp_gemm_launch_shape(M, N, K)
    cap, max_iter = 512, K // 64
    hdr = kp.make_hdr(n_wg, waves, R, cap // waves)
    trace = torch.zeros(kp.kp_trace_bytes(n_wg, waves, cap), dtype=torch.uint8, device="cuda")
    stats = torch.zeros(kp.kp_stats_bytes(n_wg, waves, R), dtype=torch.uint8, device="cuda")
    rows = torch.zeros(kp.kp_pairs_bytes(n_wg, waves, cap), dtype=torch.uint8, device="cuda")
    waits = torch.zeros(kp.kp_waits_bytes(n_wg, waves, R), dtype=torch.uint8, device="cuda")
    stages = torch.zeros(kp.kp_stages_bytes(n_wg, R, max_iter), dtype=torch.uint8, device="cuda")
    kp.kp_gemm_instrumented(A, B, C_ref, M, N, K, 0, None, 0)

    def step():
        kp.kp_gemm_instrumented(A, B, C, M, N, K, (1 << R) - 1, trace, cap)
        kp.kp_trace_reduce_hdr(trace, n_wg * cap, hdr, stats)
        kp.kp_trace_pairs_hdr(trace, n_wg * cap, hdr, rows)
        kp.kp_trace_waits_hdr(trace, n_wg * cap, hdr, waits)
        kp.kp_pairs_stages(rows, n_wg, waves, cap, R, max_iter, stages)

    step()  # eager once: module loading and attribute calls happen outside the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()

    for replay in range(3):
        for t in (C, trace, stats, rows, waits, stages):
            t.fill_(0x11 * (replay + 1) if t.dtype == torch.uint8 else 0)  # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(C.view(torch.int16), C_ref.view(torch.int16)), f"replay {replay}: GEMM result"
        raw = trace.cpu().numpy().view(np.uint32).copy()
        assert np.array_equal(oracle_mod.decode_bytes(raw), stats.cpu().numpy()), f"replay {replay}: statistics"
        # rows past a wave's count keep what the buffer held before the replay
        want_rows = oracle_mod.pairs_raw(raw, fill=0x11 * (replay + 1))
        assert np.array_equal(want_rows, rows.cpu().numpy()), f"replay {replay}: timeline rows"
        assert np.array_equal(oracle_mod.waits_raw(raw), waits.cpu().numpy()), f"replay {replay}: waits"
        want_stages = oracle_mod.stages_raw(want_rows, n_wg, waves, cap // waves, R, max_iter)
        assert np.array_equal(want_stages, stages.cpu().numpy()), f"replay {replay}: stage table"


def test_multi_pass_decoder_and_critical_path_replay_in_a_graph(oracle_mod):
    """The decoder's multi-pass kernel (a geometry outside the LDS-resident kernel's) and the critical-path
    kernel, captured once and replayed over changing input: the trace buffer is overwritten with another
    trace of the same geometry before every replay."""
    import paper_2505_21661_amd as kp

    def trace_of(seed):
        spec = inputs.TraceSpec(n_wg=20, waves=4, n_regions=48, cap_wave=8192, total_per_wave=9000, total_var=900,
                                seed=seed, dist="lognormal", p0=5.0, p1=1.0, p_orphan=0.02, p_swap=1e-3)
        return inputs.gen_trace(spec)[0]

    raw0 = trace_of(100)
    n_wg, W, R, cap = (int(x) for x in raw0[2:6])
    n = n_wg * W * cap
    hdr = kp.make_hdr(n_wg, W, R, cap)
    dev = torch.from_numpy(raw0.view(np.int32)).cuda()
    stats = torch.zeros(kp.kp_stats_bytes(n_wg, W, R), dtype=torch.uint8, device="cuda")
    max_iter = 16
    stage_tab = torch.zeros(kp.kp_stages_bytes(n_wg, R, max_iter), dtype=torch.uint8, device="cuda")
    paths = torch.zeros(kp.kp_critical_bytes(n_wg, R), dtype=torch.uint8, device="cuda")

    def step():
        kp.kp_trace_reduce_hdr(dev, n, hdr, stats)
        kp.kp_stages_critical(stage_tab, n_wg, R, max_iter, paths)

    step()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    for replay in range(3):
        raw = trace_of(200 + replay)
        dev.copy_(torch.from_numpy(raw.view(np.int32)))
        tab = np.zeros((n_wg, R, max_iter), dtype=oracle_mod.STAGE_DTYPE)
        start = rng.integers(0, 5000, size=tab.shape).astype(np.uint32)
        ext = rng.integers(0, 200, size=tab.shape).astype(np.uint32)
        tab["min_start"], tab["max_end"], tab["max_dur"], tab["n_waves"] = start, start + ext, ext, 1
        block = oracle_mod.stage_block(tab)
        stage_tab.copy_(torch.from_numpy(np.ascontiguousarray(block)))
        stats.fill_(0x22 * (replay + 1))
        paths.fill_(0x33)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(oracle_mod.decode_bytes(raw), stats.cpu().numpy()), f"replay {replay}: statistics"
        assert np.array_equal(oracle_mod.critical_raw(block, n_wg, R, max_iter), paths.cpu().numpy()), f"replay {replay}: paths"

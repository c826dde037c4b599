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

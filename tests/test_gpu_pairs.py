"""GPU parity of kp_trace_pairs (timeline rows) against oracle/ref_pairs.c, through the C ABI.

Bit-exact: counts, the first count rows of every (workgroup, wave), and the untouched remainder.
"""
import json
import math

import numpy as np
import pytest

import inputs

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kp():
    import paper_2505_21661_amd as kp

    return kp


def run_pairs(kp, raw, use_hdr=False, fill=0xA5):
    n_wg, W, R, cap = (int(x) for x in raw[2:6])
    n = n_wg * W * cap
    dev = torch.from_numpy(raw.view(np.int32)).cuda()
    out = torch.full((max(16, kp.kp_pairs_bytes(n_wg, W, W * cap)),), fill, dtype=torch.uint8, device="cuda")
    if use_hdr:
        kp.kp_trace_pairs_hdr(dev, n, kp.make_hdr(n_wg, W, R, cap, int(raw[6]), int(raw[7])), out)
    else:
        kp.kp_trace_pairs(dev, n, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()[: kp.kp_pairs_bytes(n_wg, W, W * cap)]


def assert_pairs_equal(oracle_mod, raw, got, fill=0xA5):
    ref = oracle_mod.pairs_raw(raw, fill=fill)
    assert got.size == ref.size
    if not np.array_equal(ref, got):
        n_wg, W, _R, cap = (int(x) for x in raw[2:6])
        rc, rr = oracle_mod.view_pairs(ref, n_wg, W, cap)
        gc, gr = oracle_mod.view_pairs(got, n_wg, W, cap)
        assert np.array_equal(rc, gc), ("count", np.argwhere(rc != gc)[:5])
        bad = np.argwhere(rr != gr)
        raise AssertionError(f"rows differ at {bad[:5].tolist()}: ref {rr[tuple(bad[0])]} got {gr[tuple(bad[0])]}")


@pytest.mark.parametrize("seed", range(12))
def test_messy_traces(kp, oracle_mod, seed):
    waves = [1, 2, 3, 4, 5, 8, 16][seed % 7]
    n_regions = [1, 3, 5, 16, 17, 32, 100][seed % 7]
    cap = [2, 8, 32, 64, 128, 256][seed % 6]
    raw = inputs.messy_trace(2000 + seed, n_wg=9, waves=waves, n_regions=n_regions, cap_wave=cap,
                             flush=bool(seed & 1))
    assert_pairs_equal(oracle_mod, raw, run_pairs(kp, raw, use_hdr=bool(seed & 2)))


@pytest.mark.parametrize("W,R,cap,total", [(4, 3, 128, 48), (8, 16, 2048, 2048), (8, 16, 2048, 6144),
                                           (4, 7, 4096, 4096), (1, 2, 16384, 16384), (16, 16, 1024, 1000),
                                           (4, 128, 1024, 1024), (2, 100, 512, 700), (3, 65, 256, 256)])
def test_generated_traces(kp, oracle_mod, W, R, cap, total):
    spec = inputs.TraceSpec(n_wg=37, waves=W, n_regions=R, cap_wave=cap, total_per_wave=total, total_var=total // 3,
                            seed=W * 1000 + R, p_orphan=0.02, p_swap=1e-3)
    raw, _ = inputs.gen_trace(spec)
    assert_pairs_equal(oracle_mod, raw, run_pairs(kp, raw))


def test_many_workgroups_exercise_generation_reuse(kp, oracle_mod):
    # more recorded workgroups than resident decoder workgroups: the staging area is reused
    spec = inputs.TraceSpec(n_wg=3000, waves=4, n_regions=6, cap_wave=64, total_per_wave=64, total_var=40, seed=77,
                            p_orphan=0.05, p_swap=0.01)
    raw, _ = inputs.gen_trace(spec)
    assert_pairs_equal(oracle_mod, raw, run_pairs(kp, raw, use_hdr=True))


def test_single_region_many_pairs_per_round(kp, oracle_mod):
    # one region: 32 pairs in every round of 64 ranks, the largest per-round counter value
    ev = []
    for i in range(256):
        ev += [(inputs.PHASE_START, 0, 10 * i), (inputs.PHASE_END, 0, 10 * i + 7)]
    wg = inputs.events_to_wg([ev, ev[:100]], 512)
    raw = inputs.encode_trace([wg], 2, 1, 512)
    got = run_pairs(kp, raw)
    assert_pairs_equal(oracle_mod, raw, got)
    count, rows = kp.parse_pairs(got, 1, 2, 1024)
    assert count.tolist() == [[256, 50]] and rows[0, 0, :256]["iter"].tolist() == list(range(256))


def test_empty_and_argument_errors(kp):
    raw = inputs.encode_trace([], 2, 3, 8)
    dev = torch.from_numpy(raw.view(np.int32)).cuda()
    out = torch.zeros(16, dtype=torch.uint8, device="cuda")
    kp.kp_trace_pairs(dev, 0, out)
    with pytest.raises(kp.KperfError):
        kp.kp_trace_pairs(dev, 5, out)  # slot count does not match the header


def test_rows_of_a_real_gemm_trace_and_chrome_export(kp, oracle_mod, tmp_path):
    from paper_2505_21661_amd import timeline

    M = N = 1024
    K = 512
    a, b = inputs.gemm_inputs(M, N, K, seed=5)
    A, B = a.cuda(), b.cuda()
    C = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    n_wg, waves, R = kp.kp_gemm_launch_shape(M, N, K)
    cap = 1024
    trace = torch.zeros(kp.kp_trace_bytes(n_wg, waves, cap), dtype=torch.uint8, device="cuda")
    kp.kp_gemm_instrumented(A, B, C, M, N, K, (1 << R) - 1, trace, cap)
    out = torch.zeros(kp.kp_pairs_bytes(n_wg, waves, cap), dtype=torch.uint8, device="cuda")
    kp.kp_trace_pairs(trace, n_wg * cap, out)
    torch.cuda.synchronize()
    raw = trace.cpu().numpy().view(np.uint32).copy()
    got = out.cpu().numpy()
    assert_pairs_equal(oracle_mod, raw, got, fill=0)
    count, rows = kp.parse_pairs(got, n_wg, waves, cap)
    kt = K // 64
    assert (count == 3 * kt + 1).all()
    r0 = rows[3, 5, : count[3, 5]]
    # per K step: first half, second half, barrier wait; then the epilogue once
    assert r0["region"].tolist() == [0, 1, 2] * kt + [3]
    assert r0["iter"].tolist() == [i for i in range(kt) for _ in range(3)] + [0]
    assert (np.diff(r0["start"].astype(np.int64)) > 0).all()
    path = tmp_path / "gemm_trace.json"
    n_ev = timeline.write_chrome_trace(str(path), count, rows, ["mfma+A", "mfma+B", "barrier", "epilogue"],
                                       ticks_per_us=2300.0, max_wgs=2)
    doc = json.loads(path.read_text())
    assert n_ev == len(doc["traceEvents"]) == 2 * waves * (3 * kt + 1)
    ev = doc["traceEvents"][0]
    assert ev["ph"] == "X" and ev["name"] == "mfma+A" and ev["args"]["iter"] == 0 and ev["dur"] > 0

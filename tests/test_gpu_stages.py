"""GPU parity of kp_pairs_stages (stage latency per workgroup, region and iteration) against
oracle/ref_stages.c, through the C ABI.  Bit-exact on the whole output block.  The kernel's input
is the timeline block; the oracle's own block is uploaded, so no expected value depends on the GPU."""
import numpy as np
import pytest

import inputs

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kp():
    import paper_2505_21661_amd as kp

    return kp


def run_stages(kp, block, n_wg, W, cap, R, max_iter):
    dev = torch.from_numpy(np.ascontiguousarray(block)).cuda()
    if dev.numel() == 0:
        dev = torch.zeros(16, dtype=torch.uint8, device="cuda")
    out = torch.full((kp.kp_stages_bytes(n_wg, R, max_iter),), 0x3C, dtype=torch.uint8, device="cuda")
    kp.kp_pairs_stages(dev, n_wg, W, W * cap, R, max_iter, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def check(kp, oracle_mod, raw, max_iter):
    n_wg, W, R, cap = (int(x) for x in raw[2:6])
    block = oracle_mod.pairs_raw(raw, fill=0xA5)
    want = oracle_mod.stages_raw(block, n_wg, W, cap, R, max_iter)
    got = run_stages(kp, block, n_wg, W, cap, R, max_iter)
    if not np.array_equal(want, got):
        hw, tw = oracle_mod.view_stages(want, n_wg, R, max_iter)
        hg, tg = oracle_mod.view_stages(got, n_wg, R, max_iter)
        assert hw == hg
        bad = np.argwhere(tw != tg)
        raise AssertionError(f"entries differ at {bad[:5].tolist()}: ref {tw[tuple(bad[0])]} got {tg[tuple(bad[0])]}")
    return oracle_mod.view_stages(got, n_wg, R, max_iter)


@pytest.mark.parametrize("seed", range(12))
def test_messy_traces(kp, oracle_mod, seed):
    waves = [1, 2, 3, 4, 5, 8, 16][seed % 7]
    n_regions = [1, 3, 5, 16, 17, 32, 100][seed % 7]
    cap = [2, 8, 32, 64, 128, 256][seed % 6]
    raw = inputs.messy_trace(6000 + seed, n_wg=9, waves=waves, n_regions=n_regions, cap_wave=cap,
                             flush=bool(seed & 1))
    check(kp, oracle_mod, raw, [1, 2, 7, 32][seed % 4])


@pytest.mark.parametrize("W,R,cap,total,max_iter", [(4, 3, 128, 48, 16), (8, 16, 2048, 2048, 64), (8, 16, 2048, 6144, 40),
                                                    (4, 7, 4096, 4096, 300), (1, 2, 16384, 16384, 2047),
                                                    (16, 16, 1024, 1000, 33), (2, 100, 512, 700, 4)])
def test_generated_traces(kp, oracle_mod, W, R, cap, total, max_iter):
    spec = inputs.TraceSpec(n_wg=37, waves=W, n_regions=R, cap_wave=cap, total_per_wave=total, total_var=total // 3,
                            seed=W * 1000 + R + 2, p_orphan=0.02, p_swap=1e-3)
    raw, _ = inputs.gen_trace(spec)
    hdr, tab = check(kp, oracle_mod, raw, max_iter)
    assert hdr["n_rows"] > 0 and int(tab["n_waves"].sum()) == hdr["n_rows"]


def test_many_workgroups_reuse_the_table(kp, oracle_mod):
    spec = inputs.TraceSpec(n_wg=5000, waves=4, n_regions=6, cap_wave=64, total_per_wave=64, total_var=40, seed=79,
                            p_orphan=0.05, p_swap=0.01)
    raw, _ = inputs.gen_trace(spec)
    check(kp, oracle_mod, raw, 5)


def test_fewer_regions_than_the_rows_use(kp, oracle_mod):
    spec = inputs.TraceSpec(n_wg=11, waves=4, n_regions=6, cap_wave=64, total_per_wave=60, total_var=10, seed=80)
    raw, _ = inputs.gen_trace(spec)
    block = oracle_mod.pairs_raw(raw, fill=0)
    want = oracle_mod.stages_raw(block, 11, 4, 64, 4, 8)   # regions 4 and 5 are "bad" for a table of 4
    got = run_stages(kp, block, 11, 4, 64, 4, 8)
    assert np.array_equal(want, got)
    assert oracle_mod.view_stages(got, 11, 4, 8)[0]["n_bad_region"] > 0


def test_empty_and_argument_errors(kp, oracle_mod):
    raw = inputs.encode_trace([], 2, 3, 8)
    check(kp, oracle_mod, raw, 4)
    dev = torch.zeros(64, dtype=torch.uint8, device="cuda")
    out = torch.zeros(kp.kp_stages_bytes(1, 3, 4), dtype=torch.uint8, device="cuda")
    with pytest.raises(kp.KperfError):
        kp.kp_pairs_stages(dev, 1, 3, 64, 3, 4, out)      # capacity not a multiple of the waves
    with pytest.raises(kp.KperfError) as e:
        kp.kp_pairs_stages(dev, 1, 2, 64, 128, 64, out)   # 128 regions x 65 iterations do not fit the LDS table
    assert e.value.status == kp.KP_ERR_UNSUPPORTED_SHAPE


def test_gemm_trace_end_to_end(kp, oracle_mod):
    """Record a GEMM, decode its rows and fold them on the GPU; compare with the oracle run on the
    same raw trace, and read the stage latencies the overlap models take."""
    from paper_2505_21661_amd import model

    M = N = 1024
    K = 512
    a, b = inputs.gemm_inputs(M, N, K, seed=7)
    A, B = a.cuda(), b.cuda()
    C = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    n_wg, waves, R = kp.kp_gemm_launch_shape(M, N, K)
    cap, kt = 1024, K // 64
    trace = torch.zeros(kp.kp_trace_bytes(n_wg, waves, cap), dtype=torch.uint8, device="cuda")
    kp.kp_gemm_instrumented(A, B, C, M, N, K, (1 << R) - 1, trace, cap)
    rows = torch.zeros(kp.kp_pairs_bytes(n_wg, waves, cap), dtype=torch.uint8, device="cuda")
    kp.kp_trace_pairs(trace, n_wg * cap, rows)
    out = torch.zeros(kp.kp_stages_bytes(n_wg, R, kt), dtype=torch.uint8, device="cuda")
    kp.kp_pairs_stages(rows, n_wg, waves, cap, R, kt, out)
    torch.cuda.synchronize()
    raw = trace.cpu().numpy().view(np.uint32).copy()
    want = oracle_mod.stages_raw(oracle_mod.pairs_raw(raw, fill=0), n_wg, waves, cap // waves, R, kt)
    assert np.array_equal(want, out.cpu().numpy())
    hdr, tab = kp.parse_stages(out, n_wg, R, kt)
    assert hdr == {"n_rows": n_wg * waves * (3 * kt + 1), "n_clipped": 0, "n_bad_region": 0}
    assert (tab["n_waves"][:, :3, :] == waves).all() and (tab["n_waves"][:, 3, 0] == waves).all()
    lat = model.stage_latencies(tab, 0)
    assert all(x > 0 for x in lat)
    # every wave of a workgroup leaves the barrier of K step i before any enters the one of step i + 1
    assert (tab["max_end"][:, 2, :-1] <= tab["min_start"][:, 2, 1:]).all()

"""GPU parity of kp_stages_critical (critical path of every workgroup over its stage table) against
oracle/ref_critical.c, through the C ABI.  Bit-exact on the whole output block.  The kernel's input
is a stage block written by the oracle or built by the test, so no expected value depends on the GPU."""
import numpy as np
import pytest

import inputs

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kp():
    import paper_2505_21661_amd as kp

    return kp


def run_critical(kp, block, n_wg, R, max_iter):
    dev = torch.from_numpy(np.ascontiguousarray(block)).cuda()
    out = torch.full((kp.kp_critical_bytes(n_wg, R),), 0x3C, dtype=torch.uint8, device="cuda")
    kp.kp_stages_critical(dev, n_wg, R, max_iter, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def check(kp, oracle_mod, block, n_wg, R, max_iter):
    want = oracle_mod.critical_raw(block, n_wg, R, max_iter)
    got = run_critical(kp, block, n_wg, R, max_iter)
    if not np.array_equal(want, got):
        hw, pw, rw = oracle_mod.view_critical(want, n_wg, R)
        hg, pg, rg = oracle_mod.view_critical(got, n_wg, R)
        bad = np.flatnonzero(rw != rg)
        if bad.size:
            raise AssertionError(f"rows differ at {bad[:5].tolist()}: ref {rw[bad[0]]} got {rg[bad[0]]}")
        assert pw.tolist() == pg.tolist()
        assert hw == hg
        raise AssertionError("blocks differ outside the parsed fields")
    return oracle_mod.view_critical(got, n_wg, R)


def random_table(oracle_mod, seed, n_wg, R, I, p_empty=0.2, t_max=4000, ext_max=300):
    rng = np.random.default_rng(seed)
    tab = np.zeros((n_wg, R, I), dtype=oracle_mod.STAGE_DTYPE)
    start = rng.integers(0, t_max, size=(n_wg, R, I)).astype(np.uint32)
    ext = rng.integers(0, ext_max, size=(n_wg, R, I)).astype(np.uint32)
    ext[rng.random((n_wg, R, I)) < 0.05] = 0
    live = rng.random((n_wg, R, I)) >= p_empty
    tab["min_start"] = np.where(live, start, 0xFFFFFFFF)
    tab["max_end"] = np.where(live, start + ext, 0)
    tab["max_dur"] = np.where(live, (ext * rng.random((n_wg, R, I))).astype(np.uint32), 0)
    tab["n_waves"] = np.where(live, rng.integers(1, 9, size=(n_wg, R, I)), 0)
    return tab


@pytest.mark.parametrize("R,I", [(1, 1), (1, 7), (3, 5), (2, 32), (7, 9), (16, 64), (5, 300), (100, 40), (128, 32), (4, 1024)])
def test_random_stage_tables(kp, oracle_mod, R, I):
    n_wg = 23
    tab = random_table(oracle_mod, R * 1000 + I, n_wg, R, I, t_max=50 * R * I, ext_max=120)
    hdr, per_region, rows = check(kp, oracle_mod, oracle_mod.stage_block(tab), n_wg, R, I)
    assert hdr["n_paths"] == n_wg or R * I < 8


def test_many_ties_and_zero_lengths(kp, oracle_mod):
    """Few distinct clock values: equal ends and stages of length zero everywhere; the order by index decides."""
    n_wg, R, I = 40, 6, 50
    tab = random_table(oracle_mod, 5, n_wg, R, I, p_empty=0.3, t_max=12, ext_max=4)
    check(kp, oracle_mod, oracle_mod.stage_block(tab), n_wg, R, I)


def test_empty_workgroups_and_large_clocks(kp, oracle_mod):
    n_wg, R, I = 9, 3, 10
    tab = random_table(oracle_mod, 6, n_wg, R, I)
    tab[2] = (0, 0xFFFFFFFF, 0, 0)
    tab[7] = (0, 0xFFFFFFFF, 0, 0)
    big = tab[4]["n_waves"] > 0
    tab[4]["min_start"][big] += np.uint32(0xFFF00000)
    tab[4]["max_end"][big] += np.uint32(0xFFF00000)
    hdr, per_region, rows = check(kp, oracle_mod, oracle_mod.stage_block(tab), n_wg, R, I)
    assert rows[2]["n_stages"] == 0 and rows[7]["last_stage"] == 0xFFFFFFFF and hdr["n_paths"] == n_wg - 2


def test_a_serial_chain_of_maximum_length(kp, oracle_mod):
    """4096 stages one after the other: the longest list the pointer doubling has to mark."""
    R, I = 4, 1024
    tab = np.zeros((2, R, I), dtype=oracle_mod.STAGE_DTYPE)
    t = np.arange(R * I, dtype=np.uint32).reshape(I, R).T * 10   # iteration-major in time
    tab["min_start"][:] = t
    tab["max_end"][:] = t + 7
    tab["max_dur"][:] = 7
    tab["n_waves"][:] = 1
    hdr, per_region, rows = check(kp, oracle_mod, oracle_mod.stage_block(tab), 2, R, I)
    assert rows["n_stages"].tolist() == [R * I] * 2 and rows["bubbles"].tolist() == [3 * (R * I - 1)] * 2


def test_generated_trace_end_to_end(kp, oracle_mod):
    """From a raw trace: oracle rows and stage table, then both critical paths."""
    spec = inputs.TraceSpec(n_wg=300, waves=8, n_regions=16, cap_wave=512, total_per_wave=512, total_var=100, seed=91,
                            p_orphan=0.02, p_swap=1e-3)
    raw, _ = inputs.gen_trace(spec)
    n_wg, W, R, cap = (int(x) for x in raw[2:6])
    max_iter = 24
    block = oracle_mod.stages_raw(oracle_mod.pairs_raw(raw, fill=0), n_wg, W, cap, R, max_iter)
    hdr, per_region, rows = check(kp, oracle_mod, block, n_wg, R, max_iter)
    assert hdr["n_paths"] == n_wg and (rows["n_stages"] > 0).all()
    # the path's stages and bubbles cannot take longer than the stretch they lie in
    assert (rows["bubbles"] <= rows["last_end"].astype(np.int64) - rows["first_start"]).all()


def test_gpu_pipeline_end_to_end(kp, oracle_mod):
    """Recorded GEMM -> rows -> stage table -> critical path, all on the GPU; against the oracle chain on
    the same raw trace.  Every K step's regions follow one another in all waves, so the path is long."""
    M = N = 1024
    K = 512
    a, b = inputs.gemm_inputs(M, N, K, seed=8)
    A, B = a.cuda(), b.cuda()
    C = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    n_wg, waves, R = kp.kp_gemm_launch_shape(M, N, K)
    cap, kt = 1024, K // 64
    trace = torch.zeros(kp.kp_trace_bytes(n_wg, waves, cap), dtype=torch.uint8, device="cuda")
    kp.kp_gemm_instrumented(A, B, C, M, N, K, (1 << R) - 1, trace, cap)
    rows_blk = torch.zeros(kp.kp_pairs_bytes(n_wg, waves, cap), dtype=torch.uint8, device="cuda")
    kp.kp_trace_pairs(trace, n_wg * cap, rows_blk)
    stages = torch.zeros(kp.kp_stages_bytes(n_wg, R, kt), dtype=torch.uint8, device="cuda")
    kp.kp_pairs_stages(rows_blk, n_wg, waves, cap, R, kt, stages)
    out = torch.full((kp.kp_critical_bytes(n_wg, R),), 0x11, dtype=torch.uint8, device="cuda")
    kp.kp_stages_critical(stages, n_wg, R, kt, out)
    torch.cuda.synchronize()
    raw = trace.cpu().numpy().view(np.uint32).copy()
    want = oracle_mod.critical_raw(oracle_mod.stages_raw(oracle_mod.pairs_raw(raw, fill=0), n_wg, waves, cap // waves, R, kt),
                                   n_wg, R, kt)
    assert np.array_equal(want, out.cpu().numpy())
    hdr, per_region, rows = kp.parse_critical(out, n_wg, R)
    assert hdr["n_paths"] == n_wg and (rows["last_stage"] >> 16 == 3).all()   # the epilogue ends last
    assert (rows["n_stages"] >= kt).all()


def test_argument_errors(kp):
    dev = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    out = torch.zeros(kp.kp_critical_bytes(1, 128), dtype=torch.uint8, device="cuda")
    with pytest.raises(kp.KperfError) as e:
        kp.kp_stages_critical(dev, 1, 128, 33, out)      # 4224 stages per workgroup
    assert e.value.status == kp.KP_ERR_UNSUPPORTED_SHAPE
    for args in [(1, 0, 4), (1, 129, 1), (1, 3, 0), (-1, 3, 4)]:
        with pytest.raises(kp.KperfError) as e:
            kp.kp_stages_critical(dev, *args, out)
        assert e.value.status == kp.KP_ERR_INVALID_ARG
    kp.kp_stages_critical(dev, 0, 3, 4, out)               # no workgroups: header only
    torch.cuda.synchronize()
    assert out.cpu().numpy()[:64].view("<u8").tolist() == [0, 3, 4, 0, 0, 0, 0, 0]

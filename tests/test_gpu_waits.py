"""GPU parity of kp_trace_waits (waits behind asynchronous operations, Sec. 4.3) against
oracle/ref_waits.c, through the C ABI.  Bit-exact on the whole output block."""
import numpy as np
import pytest

import inputs

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kp():
    import paper_2505_21661_amd as kp

    return kp


def run_waits(kp, raw, use_hdr=False):
    n_wg, W, R, cap = (int(x) for x in raw[2:6])
    n = n_wg * W * cap
    dev = torch.from_numpy(raw.view(np.int32)).cuda()
    out = torch.full((kp.kp_waits_bytes(n_wg, W, R),), 0x5A, dtype=torch.uint8, device="cuda")
    if use_hdr:
        kp.kp_trace_waits_hdr(dev, n, kp.make_hdr(n_wg, W, R, cap, int(raw[6]), int(raw[7])), out)
    else:
        kp.kp_trace_waits(dev, n, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def assert_waits_equal(oracle_mod, raw, got):
    ref = oracle_mod.waits_raw(raw)
    assert got.size == ref.size
    if not np.array_equal(ref, got):
        r, g = oracle_mod.view_waits(ref), oracle_mod.view_waits(got)
        for k in ("n_waits", "n_uncovered", "n_async", "n_wg", "waves", "n_regions", "cap_wave", "rec_cost"):
            assert r[k] == g[k], (k, r[k], g[k])
        for k in ("cnt", "sum", "min", "max", "uncovered", "async_cnt", "async_sum", "hist"):
            assert np.array_equal(r[k], g[k]), (k, np.argwhere(r[k] != g[k])[:5].tolist())
        bad = np.argwhere(r["per"] != g["per"])
        raise AssertionError(f"per-wave entries differ at {bad[:5].tolist()}: ref {r['per'][tuple(bad[0])]} got {g['per'][tuple(bad[0])]}")


@pytest.mark.parametrize("seed", range(14))
def test_messy_traces(kp, oracle_mod, seed):
    waves = [1, 2, 3, 4, 5, 8, 16][seed % 7]
    n_regions = [1, 3, 5, 16, 17, 32, 100][seed % 7]
    cap = [2, 8, 32, 64, 128, 256][seed % 6]
    raw = inputs.messy_trace(4000 + seed, n_wg=9, waves=waves, n_regions=n_regions, cap_wave=cap,
                             flush=bool(seed & 1))
    raw[6] = [0, 7, 60][seed % 3]  # record cost
    assert_waits_equal(oracle_mod, raw, run_waits(kp, raw, use_hdr=bool(seed & 2)))


@pytest.mark.parametrize("W,R,cap,total", [(4, 3, 128, 48), (8, 16, 2048, 2048), (8, 16, 2048, 6144),
                                           (4, 7, 4096, 4096), (1, 2, 16384, 16384), (16, 16, 1024, 1000),
                                           (4, 64, 1024, 1024), (2, 100, 512, 700)])
def test_generated_traces(kp, oracle_mod, W, R, cap, total):
    spec = inputs.TraceSpec(n_wg=37, waves=W, n_regions=R, cap_wave=cap, total_per_wave=total, total_var=total // 3,
                            seed=W * 1000 + R + 1, p_orphan=0.02, p_swap=1e-3)
    raw, _ = inputs.gen_trace(spec)
    raw[6] = 25
    assert_waits_equal(oracle_mod, raw, run_waits(kp, raw))


def test_many_workgroups_exercise_generation_reuse(kp, oracle_mod):
    # more recorded workgroups than resident decoder workgroups: staging area and totals are reused
    spec = inputs.TraceSpec(n_wg=3000, waves=4, n_regions=6, cap_wave=64, total_per_wave=64, total_var=40, seed=78,
                            p_orphan=0.05, p_swap=0.01)
    raw, _ = inputs.gen_trace(spec)
    raw[6] = 3
    assert_waits_equal(oracle_mod, raw, run_waits(kp, raw, use_hdr=True))


def test_holes_below_a_start(kp, oracle_mod):
    """Invalid slots leave empty ranks: a START then finds the record below it by walking back."""
    S, E = inputs.PHASE_START, inputs.PHASE_END
    ev = []
    for i in range(150):
        ev += [(S, i % 3, 20 * i), (E, i % 3, 20 * i + 9)]
    wg = inputs.events_to_wg([ev, ev[:77]], 512)
    raw = inputs.encode_trace([wg], 2, 3, 512)
    rec0 = (64 + 128) // 4
    rng = np.random.default_rng(3)
    for s in rng.choice(300, size=60, replace=False):  # wave 0: give some slots a foreign wave id
        raw[rec0 + 2 * int(s)] ^= np.uint32(5 << 20)
    assert_waits_equal(oracle_mod, raw, run_waits(kp, raw))


def test_empty_and_argument_errors(kp, oracle_mod):
    raw = inputs.encode_trace([], 2, 3, 8)
    assert_waits_equal(oracle_mod, raw, run_waits(kp, raw))
    dev = torch.from_numpy(raw.view(np.int32)).cuda()
    out = torch.zeros(kp.kp_waits_bytes(0, 2, 3), dtype=torch.uint8, device="cuda")
    with pytest.raises(kp.KperfError):
        kp.kp_trace_waits(dev, 5, out)  # slot count does not match the header
    with pytest.raises(kp.KperfError) as e:  # 128 regions of histogram do not fit beside 16384 staged records
        kp.kp_trace_waits_hdr(dev, 8 * 2048, kp.make_hdr(1, 8, 128, 2048), out)
    assert e.value.status == kp.KP_ERR_UNSUPPORTED_SHAPE


def test_wait_at_the_barrier_of_a_real_gemm(kp, oracle_mod):
    """The 256x256x64 GEMM with its wait region switched off records END(1) right before the barrier
    and START(0) right after it: the paper's placement around the asynchronous staging loads."""
    M = N = 1024
    K = 512
    a, b = inputs.gemm_inputs(M, N, K, seed=6)
    A, B = a.cuda(), b.cuda()
    C = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    n_wg, waves, R = kp.kp_gemm_launch_shape(M, N, K)
    cap = 1024
    trace = torch.zeros(kp.kp_trace_bytes(n_wg, waves, cap), dtype=torch.uint8, device="cuda")
    kp.kp_gemm_instrumented(A, B, C, M, N, K, 0b1011, trace, cap)
    out = torch.zeros(kp.kp_waits_bytes(n_wg, waves, R), dtype=torch.uint8, device="cuda")
    kp.kp_trace_waits(trace, n_wg * cap, out)
    torch.cuda.synchronize()
    raw = trace.cpu().numpy().view(np.uint32).copy()
    assert_waits_equal(oracle_mod, raw, out.cpu().numpy())
    v = kp.parse_waits(out)
    kt = K // 64
    # region 0 ends where region 1 starts (gap 0, one clock sample); the barrier follows region 1
    assert v["cnt"].tolist() == [n_wg * waves * kt, n_wg * waves * kt, 0, 0]
    assert v["sum"][0] == 0 and v["sum"][1] > 0 and v["async_cnt"][1] == v["cnt"][1]
    assert (v["per"]["n"][:, :, 1] == kt).all()

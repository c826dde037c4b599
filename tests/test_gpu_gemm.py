"""Instrumented bf16 GEMM through the C ABI: outputs against the fp64 oracle and against the
uninstrumented kernel (bitwise), traces against closed forms, the CPU decoder oracle and timer
invariants."""
import numpy as np
import pytest
import torch

import inputs
from oracle import bf16_round, ref_gemm

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kp():
    import paper_2505_21661_amd as kp

    return kp


def run_gemm(kp, a, b, mask, trace_cap=None):
    M, K = a.shape
    N = b.shape[1]
    A, B = a.cuda(), b.cuda()
    C = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    n_wg, waves, n_regions = kp.kp_gemm_launch_shape(M, N, K)
    trace = None
    if mask & 0x7FFFFFFF:
        trace = torch.full((kp.kp_trace_bytes(n_wg, waves, trace_cap),), 0x77, dtype=torch.uint8, device="cuda")
    kp.kp_gemm_instrumented(A, B, C, M, N, K, mask, trace, trace_cap or 0)
    torch.cuda.synchronize()
    return C, trace, (n_wg, waves, n_regions)


def assert_close_to_oracle(C, a, b, rows=None):
    """|gpu - ref| <= 1e-2*|ref| + 1e-2*rms(ref) per element and 1e-2 relative in Frobenius norm
    (bf16 inputs, fp32 accumulation, bf16 output against the fp64 definition)."""
    ref = ref_gemm(a, b, rows=rows)
    got = C.float().cpu().numpy().astype(np.float64)
    if rows is not None:
        got = got[np.asarray(rows)]
    rms = np.sqrt(np.mean(ref ** 2))
    err = np.abs(got - ref)
    assert np.all(err <= 1e-2 * np.abs(ref) + 1e-2 * rms), float(err.max())
    assert np.linalg.norm(got - ref) <= 1e-2 * np.linalg.norm(ref)
    # tighter sanity: the only rounding beyond fp32 accumulation is the final bf16 rounding
    assert np.linalg.norm(got - bf16_round(ref)) <= 2e-3 * np.linalg.norm(ref)


def test_small_gemm_matches_oracle_and_vanilla(kp):
    a, b = inputs.gemm_inputs(256, 256, 256, seed=0, dist="uniform")
    c_van, _, shape = run_gemm(kp, a, b, 0)
    assert shape == (16, 4, 3)
    assert_close_to_oracle(c_van, a, b)
    c_ins, trace, _ = run_gemm(kp, a, b, 0b111, trace_cap=512)
    assert torch.equal(c_ins.view(torch.int16), c_van.view(torch.int16))  # bit-identical
    for mask in (0b001, 0b100, 0b110):
        c2, _, _ = run_gemm(kp, a, b, mask, trace_cap=512)
        assert torch.equal(c2.view(torch.int16), c_van.view(torch.int16))


def test_exact_special_cases(kp):
    _, b = inputs.gemm_inputs(128, 192, 128, seed=5)
    eye = torch.eye(128, dtype=torch.bfloat16)
    c, _, _ = run_gemm(kp, eye, b, 0b111, trace_cap=512)
    assert torch.equal(c.cpu().view(torch.int16), b.view(torch.int16))       # A = I  =>  C = B exactly
    ones_a = torch.ones(64, 256, dtype=torch.bfloat16)
    ones_b = torch.ones(256, 64, dtype=torch.bfloat16)
    c, _, _ = run_gemm(kp, ones_a, ones_b, 0)
    assert (c.float() == 256.0).all()


@pytest.mark.parametrize("M,N,K", [(64, 64, 32), (128, 320, 96), (192, 64, 608), (320, 448, 160)])
def test_other_shapes(kp, M, N, K):
    a, b = inputs.gemm_inputs(M, N, K, seed=M + N + K)
    c, _, _ = run_gemm(kp, a, b, 0b111, trace_cap=1024)
    assert_close_to_oracle(c, a, b)
    c0, _, _ = run_gemm(kp, a, b, 0)
    assert torch.equal(c.view(torch.int16), c0.view(torch.int16))


def test_small_gemm_trace(kp, oracle_mod):
    from tests.gpu_util import assert_stats_equal

    a, b = inputs.gemm_inputs(256, 256, 256, seed=0, dist="uniform")
    _, trace, (n_wg, waves, R) = run_gemm(kp, a, b, 0b111, trace_cap=512)
    raw = trace.cpu().numpy().view(np.uint32).copy()
    assert tuple(raw[:8]) == (0x4652504B, 1, n_wg, waves, R, 128, 0, 0)
    out = torch.zeros(kp.kp_stats_bytes(n_wg, waves, R), dtype=torch.uint8, device="cuda")
    kp.kp_trace_reduce(trace, n_wg * waves * 128, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert_stats_equal(oracle_mod.decode_bytes(raw, 8), got, oracle_mod)
    st = kp.parse_stats(got)
    # closed form: 8 K-steps x 3 regions x 2 records per wave
    k_steps = 256 // 32
    assert st["n_slots_valid"] == n_wg * waves * 3 * 2 * k_steps
    assert st["n_pairs"] == n_wg * waves * 3 * k_steps and (st["per"]["n"] == k_steps).all()
    for k in ("n_orphan_start", "n_orphan_end", "n_invalid", "n_dropped", "n_disorder", "n_nonmonotonic",
              "n_span_overflow_wgs"):
        assert st[k] == 0, k
    hdr = raw[16:16 + 32 * n_wg].reshape(n_wg, 32)
    span = ((hdr[:, 4].astype(np.uint64) | (hdr[:, 5].astype(np.uint64) << np.uint64(32)))
            - (hdr[:, 2].astype(np.uint64) | (hdr[:, 3].astype(np.uint64) << np.uint64(32)))).astype(np.int64)
    # regions of one wave are disjoint: their total time fits in the workgroup span
    assert (st["per"]["sum"].sum(axis=2).astype(np.int64) <= span[:, None]).all()
    assert (st["U"].astype(np.int64) <= span.sum()).all()
    # masked-off regions leave no records
    _, trace2, _ = run_gemm(kp, a, b, 0b101, trace_cap=512)
    out2 = torch.zeros_like(out)
    kp.kp_trace_reduce(trace2, n_wg * waves * 128, out2)
    torch.cuda.synchronize()
    st2 = kp.parse_stats(out2)
    assert st2["cnt"].tolist() == [n_wg * waves * k_steps, 0, n_wg * waves * k_steps]


def test_gemm_ring_wrap_and_flush(kp, oracle_mod):
    from tests.gpu_util import assert_stats_equal

    a, b = inputs.gemm_inputs(128, 128, 512, seed=9)       # 16 K-steps -> 96 records per wave
    for mask, cap_wave, dropped in ((0b111, 64, 32), (0b111 | (1 << 31), 128, 0), (0b111 | (1 << 31), 64, 32)):
        c, trace, (n_wg, waves, R) = run_gemm(kp, a, b, mask, trace_cap=cap_wave * 4)
        raw = trace.cpu().numpy().view(np.uint32).copy()
        out = torch.zeros(kp.kp_stats_bytes(n_wg, waves, R), dtype=torch.uint8, device="cuda")
        kp.kp_trace_reduce(trace, n_wg * waves * cap_wave, out)
        torch.cuda.synchronize()
        assert_stats_equal(oracle_mod.decode_bytes(raw, 8), out.cpu().numpy(), oracle_mod)
        st = kp.parse_stats(out)
        assert st["n_dropped"] == dropped * n_wg * waves, (mask, cap_wave)
        assert st["n_invalid"] == 0 and st["n_nonmonotonic"] == 0
        assert_close_to_oracle(c, a, b)


def test_gemm_errors(kp):
    a = torch.zeros(64, 64, dtype=torch.bfloat16, device="cuda")
    c = torch.zeros(64, 64, dtype=torch.bfloat16, device="cuda")
    tr = torch.zeros(kp.kp_trace_bytes(1, 4, 512), dtype=torch.uint8, device="cuda")
    with pytest.raises(kp.KperfError) as e:
        kp.kp_gemm_instrumented(a, a, c, 60, 64, 64, 0, None, 0)
    assert e.value.status == kp.KP_ERR_UNSUPPORTED_SHAPE
    with pytest.raises(kp.KperfError) as e:
        kp.kp_gemm_instrumented(a, a, c, 64, 64, 64, 7, tr, 500)
    assert e.value.status == kp.KP_ERR_TRACE_TOO_SMALL
    with pytest.raises(kp.KperfError) as e:
        kp.kp_gemm_instrumented(a, a, c, 64, 64, 64, 7, None, 512)
    assert e.value.status == kp.KP_ERR_INVALID_ARG
    with pytest.raises(kp.KperfError) as e:
        kp.kp_gemm_instrumented(a, a, c, 64, 64, 64, 0b1000, tr, 512)
    assert e.value.status == kp.KP_ERR_INVALID_ARG


# ---- 256x256x64 tile kernel ------------------------------------------------------------------

def test_big_tile_gemm_matches_oracle_and_vanilla(kp):
    a, b = inputs.gemm_inputs(1024, 1024, 256, seed=11)
    c_van, _, shape = run_gemm(kp, a, b, 0)
    assert shape == (16, 8, 4)
    assert_close_to_oracle(c_van, a, b)
    c_ins, _, _ = run_gemm(kp, a, b, 0b1111, trace_cap=4096)
    assert torch.equal(c_ins.view(torch.int16), c_van.view(torch.int16))
    c_fl, _, _ = run_gemm(kp, a, b, 0b1111 | (1 << 31), trace_cap=4096)
    assert torch.equal(c_fl.view(torch.int16), c_van.view(torch.int16))
    # exact cases
    eye = torch.eye(1024, dtype=torch.bfloat16)
    ones_a = torch.ones(1024, 512, dtype=torch.bfloat16)
    ones_b = torch.ones(512, 1024, dtype=torch.bfloat16)
    c, _, _ = run_gemm(kp, ones_a, ones_b, 0b1111, trace_cap=4096)
    assert (c.float() == 512.0).all()
    b2 = inputs.gemm_inputs(1024, 1280, 1024, seed=4)[1]
    c, _, _ = run_gemm(kp, eye, b2, 0)
    assert torch.equal(c.cpu().view(torch.int16), b2.view(torch.int16))


@pytest.mark.parametrize("M,N,K", [(768, 1536, 192), (2048, 512, 64), (1280, 1024, 448), (512, 2304, 128)])
def test_big_tile_other_shapes(kp, M, N, K):
    """Tile grids that are not square, with and without the XCD-block mapping of workgroups to tiles, one to
    seven K steps: both schedules of the K loop against the fp64 oracle, instrumented bit-identical."""
    a, b = inputs.gemm_inputs(M, N, K, seed=M + N + K)
    c_van, _, shape = run_gemm(kp, a, b, 0)
    assert shape == ((M // 256) * (N // 256), 8, 4)
    assert_close_to_oracle(c_van, a, b)
    c_ins, _, _ = run_gemm(kp, a, b, 0b1111, trace_cap=1024)
    assert torch.equal(c_ins.view(torch.int16), c_van.view(torch.int16))
    c_ph, _, _ = run_gemm_phased(kp, a, b, 0)
    assert torch.equal(c_ph.view(torch.int16), c_van.view(torch.int16))
    c_ph5, _, _ = run_gemm_phased(kp, a, b, 0b11111, trace_cap=1024)
    assert torch.equal(c_ph5.view(torch.int16), c_van.view(torch.int16))


def test_big_tile_trace_small_k(kp, oracle_mod):
    from tests.gpu_util import assert_stats_equal

    a, b = inputs.gemm_inputs(1024, 1024, 512, seed=12)      # 8 K-steps: 50 records per wave
    _, trace, (n_wg, waves, R) = run_gemm(kp, a, b, 0b1111, trace_cap=1024)
    raw = trace.cpu().numpy().view(np.uint32).copy()
    out = torch.zeros(kp.kp_stats_bytes(n_wg, waves, R), dtype=torch.uint8, device="cuda")
    kp.kp_trace_reduce(trace, n_wg * waves * 128, out)
    torch.cuda.synchronize()
    assert_stats_equal(oracle_mod.decode_bytes(raw, 8), out.cpu().numpy(), oracle_mod)
    st = kp.parse_stats(out)
    assert st["n_slots_valid"] == n_wg * waves * (8 * 3 * 2 + 2) and st["n_pairs"] == n_wg * waves * 25
    # per K-step: first half, second half, barrier wait; one epilogue
    assert st["cnt"].tolist() == [n_wg * waves * 8] * 3 + [n_wg * waves]
    for k in ("n_orphan_start", "n_orphan_end", "n_invalid", "n_dropped", "n_disorder", "n_nonmonotonic"):
        assert st[k] == 0, k
    assert sorted(raw[16:16 + 32 * n_wg].reshape(n_wg, 32)[:, 0].tolist()) == list(range(n_wg))


@pytest.mark.parametrize("cap_wave", [2, 16, 64, 256])
def test_big_tile_lean_sites_with_short_rings(kp, oracle_mod, cap_wave):
    """The large kernel keeps only the clocks of its sites (in a ring of twice as many entries as the trace has
    slots per wave) and makes the records when it copies the trace out.  Rings of two slots, rings that wrap and
    a ring that holds everything must all decode like the oracle says, with the drop count of the closed form."""
    from tests.gpu_util import assert_stats_equal

    K = 2048                                                     # 32 K-steps: 3 sites each, 194 records per wave
    a, b = inputs.gemm_inputs(1024, 1024, K, seed=13)
    c, trace, (n_wg, waves, R) = run_gemm(kp, a, b, 0b1111, trace_cap=cap_wave * 8)
    assert (n_wg, waves, R) == (16, 8, 4)
    raw = trace.cpu().numpy().view(np.uint32).copy()
    out = torch.zeros(kp.kp_stats_bytes(n_wg, waves, R), dtype=torch.uint8, device="cuda")
    kp.kp_trace_reduce(trace, n_wg * waves * cap_wave, out)
    torch.cuda.synchronize()
    assert_stats_equal(oracle_mod.decode_bytes(raw, 8), out.cpu().numpy(), oracle_mod)
    st = kp.parse_stats(out)
    total = 2 * 3 * (K // 64) + 2
    assert (raw[16:16 + 32 * n_wg].reshape(n_wg, 32)[:, 8:16] == total).all()
    assert st["n_dropped"] == n_wg * waves * max(0, total - cap_wave)
    assert st["n_slots_valid"] == n_wg * waves * min(total, cap_wave)
    assert st["n_invalid"] == 0 and st["n_nonmonotonic"] == 0 and st["n_disorder"] == 0
    # the survivors are the newest records: sequence numbers total - cap_wave .. total - 1
    recs = raw[16 + 32 * n_wg:].reshape(n_wg, waves, cap_wave, 2)
    keep = min(total, cap_wave)
    seq = np.sort(recs[:, :, :keep, 0] & 0xFFFFF, axis=2)   # a ring that wrapped is full: every slot is valid
    assert (seq == np.arange(total - keep, total)).all()
    assert_close_to_oracle(c, a, b)


@pytest.mark.parametrize("phased,regions", [(False, 0b1111), (False, 0b1011), (False, 0b0100), (False, 0b1000),
                                            (True, 0b11111), (True, 0b01010), (True, 0b10001)])
@pytest.mark.parametrize("cap_wave", [2, 32, 512])
def test_big_tile_chained_sites_write_the_generic_sites_records(kp, phased, regions, cap_wave):
    """The large kernel keeps only the clocks of its record sites and makes the records when it copies the
    trace out.  Against the records the generic sites write (KP_MASK_COLLAB selects them): the same record
    count and the same tag in every slot, for both schedules of the K loop and for region masks, also where
    the ring wrapped; clocks that do not decrease along the sequence numbers of a wave and stay inside the
    workgroup's span; cleared slots behind the last record."""
    K = 1024                                                     # 16 K-steps
    a, b = inputs.gemm_inputs(1024, 1024, K, seed=17)
    A, B = a.cuda(), b.cuda()
    n_wg, waves, _ = kp.kp_gemm_launch_shape(1024, 1024, K)
    assert (n_wg, waves) == (16, 8)
    R = 5 if phased else 4
    base = regions | (kp.KP_MASK_PHASES if phased else 0)
    raws = []
    for extra in (0, kp.KP_MASK_COLLAB):
        C = torch.empty(1024, 1024, dtype=torch.bfloat16, device="cuda")
        trace = torch.full((kp.kp_trace_bytes(n_wg, waves, cap_wave * waves),), 0x77, dtype=torch.uint8, device="cuda")
        kp.kp_gemm_instrumented(A, B, C, 1024, 1024, K, base | extra, trace, cap_wave * waves)
        torch.cuda.synchronize()
        raws.append(trace.cpu().numpy().view(np.uint32).copy())
    x, y = raws
    assert tuple(x[2:6]) == tuple(y[2:6]) == (n_wg, waves, R, cap_wave)
    hx, hy = (r[16:16 + 32 * n_wg].reshape(n_wg, 32) for r in (x, y))
    per_step = [2 * bin(regions & 0b0111).count("1"), 2 * bin(regions & 0b01111).count("1")][phased]
    total = per_step * (K // 64) + 2 * ((regions >> (R - 1)) & 1)
    assert (hx[:, 8:8 + waves] == total).all() and (hy[:, 8:8 + waves] == total).all() and (hx[:, 8 + waves:24] == 0).all()
    rx, ry = (r[16 + 32 * n_wg:].reshape(n_wg, waves, cap_wave, 2) for r in (x, y))
    n = min(total, cap_wave)
    assert (rx[:, :, :n, 0] == ry[:, :, :n, 0]).all()
    assert (rx[:, :, n:] == 0).all()
    seq = rx[:, :, :n, 0] & 0xFFFFF
    order = np.argsort(seq, axis=2)
    assert (np.take_along_axis(seq, order, 2) == np.arange(total - n, total)).all()
    ts = np.take_along_axis(rx[:, :, :n, 1], order, 2).astype(np.int64)
    assert (np.diff(ts, axis=2) >= 0).all() and (ts > 0).all()
    span = (hx[:, 4:6].copy().view(np.uint64) - hx[:, 2:4].copy().view(np.uint64)).astype(np.int64)
    assert (ts.reshape(n_wg, -1).max(axis=1) < span[:, 0]).all()


def _streams_of(raw, n_wg, streams, cap):
    hdr = raw[16:16 + 32 * n_wg].reshape(n_wg, 32)
    return hdr, raw[16 + 32 * n_wg:].reshape(n_wg, streams, cap, 2)


@pytest.mark.parametrize("case", range(10))
def test_big_tile_chained_sites_with_every_option(kp, case):
    """Seeded combinations of schedule, region mask, wave-group records, constant-rate clock, ring capacity and
    K: the chained sites must leave the record counts and tags of the generic sites (KP_MASK_COLLAB on top of
    the same options), slot by slot, and clocks that do not decrease along a stream."""
    rng = np.random.default_rng(100 + case)
    phased = bool(rng.integers(2))
    R = 5 if phased else 4
    regions = int(rng.integers(1, 1 << R))
    group = bool(rng.integers(2))
    realtime = bool(rng.integers(2))
    K = int(rng.choice([64, 192, 1024, 4096]))
    cap_wave = int(rng.choice([2, 8, 64, 512]))
    a, b = inputs.gemm_inputs(1024, 1024, K, seed=40 + case)
    A, B = a.cuda(), b.cuda()
    n_wg, waves, _ = kp.kp_gemm_launch_shape(1024, 1024, K)
    assert (n_wg, waves) == (16, 8)
    streams = waves // 4 if group else waves
    opts = regions | (kp.KP_MASK_PHASES if phased else 0) | (kp.KP_MASK_WAVE_GROUP if group else 0) | (kp.KP_MASK_REALTIME if realtime else 0)
    raws = []
    for extra in (0, kp.KP_MASK_COLLAB):
        C = torch.empty(1024, 1024, dtype=torch.bfloat16, device="cuda")
        trace = torch.full((kp.kp_trace_bytes(n_wg, streams, cap_wave * streams),), 0x5C, dtype=torch.uint8, device="cuda")
        kp.kp_gemm_instrumented(A, B, C, 1024, 1024, K, opts | extra, trace, cap_wave * streams)
        torch.cuda.synchronize()
        raws.append(trace.cpu().numpy().view(np.uint32).copy())
    x, y = raws
    assert tuple(x[2:6]) == tuple(y[2:6]) == (n_wg, streams, R, cap_wave), (phased, regions, group, realtime, K, cap_wave)
    (hx, rx), (hy, ry) = (_streams_of(r, n_wg, streams, cap_wave) for r in (x, y))
    assert (hx[:, 8:24] == hy[:, 8:24]).all()
    total = int(hx[0, 8])
    steps = K // 64
    assert total == 2 * steps * bin(regions & ((1 << (R - 1)) - 1)).count("1") + 2 * ((regions >> (R - 1)) & 1)
    n = min(total, cap_wave)
    assert (rx[:, :, :n, 0] == ry[:, :, :n, 0]).all(), (phased, regions, group, realtime, K, cap_wave)
    assert (rx[:, :, n:] == 0).all()
    if n:
        order = np.argsort(rx[:, :, :n, 0] & 0xFFFFF, axis=2)
        ts = np.take_along_axis(rx[:, :, :n, 1], order, 2).astype(np.int64)
        assert (np.diff(ts, axis=2) >= 0).all() and (ts > 0).all()


@pytest.mark.parametrize("shape,flush", [((1024, 1024, 512), 0), ((1024, 1024, 512), 1), ((128, 128, 256), 0)])
def test_wave_group_records(kp, oracle_mod, shape, flush):
    """KP_MASK_WAVE_GROUP: one record stream per group of four waves (Sec. 3.1 Granularity, Sec. 4.2
    buffer per warp group).  The trace holds waves / 4 streams with the per-wave record count each,
    decodes like the oracle says, and C stays bit-identical to the uninstrumented kernel's."""
    from tests.gpu_util import assert_stats_equal

    M, N, K = shape
    a, b = inputs.gemm_inputs(M, N, K, seed=14)
    n_wg, waves, R = kp.kp_gemm_launch_shape(M, N, K)
    streams, cap_stream = waves // 4, 256
    A, B = a.cuda(), b.cuda()
    C = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    C0 = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    trace = torch.full((kp.kp_trace_bytes(n_wg, streams, streams * cap_stream),), 0x77, dtype=torch.uint8, device="cuda")
    mask = ((1 << R) - 1) | kp.KP_MASK_WAVE_GROUP | (kp.KP_MASK_FLUSH if flush else 0)
    kp.kp_gemm_instrumented(A, B, C, M, N, K, mask, trace, streams * cap_stream)
    kp.kp_gemm_instrumented(A, B, C0, M, N, K, 0, None, 0)
    torch.cuda.synchronize()
    assert torch.equal(C.view(torch.int16), C0.view(torch.int16))
    raw = trace.cpu().numpy().view(np.uint32).copy()
    assert tuple(raw[2:8]) == (n_wg, streams, R, cap_stream, 0, flush)
    out = torch.zeros(kp.kp_stats_bytes(n_wg, streams, R), dtype=torch.uint8, device="cuda")
    kp.kp_trace_reduce(trace, n_wg * streams * cap_stream, out)
    torch.cuda.synchronize()
    assert_stats_equal(oracle_mod.decode_bytes(raw, 8), out.cpu().numpy(), oracle_mod)
    st = kp.parse_stats(out)
    if waves == 8:   # large tile: three regions per K-step of 64 and one epilogue
        per_stream, cnt = 2 * 3 * (K // 64) + 2, [n_wg * streams * (K // 64)] * 3 + [n_wg * streams]
    else:            # small tile: three regions per K-step of 32
        per_stream, cnt = 2 * 3 * (K // 32), [n_wg * streams * (K // 32)] * 3
    hdr = raw[16:16 + 32 * n_wg].reshape(n_wg, 32)
    assert (hdr[:, 8:8 + streams] == per_stream).all() and (hdr[:, 8 + streams:24] == 0).all()
    assert st["n_slots_valid"] == n_wg * streams * per_stream and st["cnt"].tolist() == cnt
    for k in ("n_orphan_start", "n_orphan_end", "n_invalid", "n_dropped", "n_disorder", "n_nonmonotonic"):
        assert st[k] == 0, k


def test_full_size_gemm_4096(kp, oracle_mod):
    """The benchmark configuration: 4096^3, N(0,1) inputs, 4 regions, ring of 4096 records per
    workgroup.  Output is checked on sampled rows, the trace against closed forms and the oracle."""
    from tests.gpu_util import assert_stats_equal

    M = N = K = 4096
    a, b = inputs.gemm_inputs(M, N, K, seed=2)
    c_van, _, shape = run_gemm(kp, a, b, 0)
    assert shape == (256, 8, 4)
    rows = np.random.default_rng(0).choice(M, size=48, replace=False)
    assert_close_to_oracle(c_van, a, b, rows=np.sort(rows))
    c_ins, trace, (n_wg, waves, R) = run_gemm(kp, a, b, 0b1111, trace_cap=4096)
    assert torch.equal(c_ins.view(torch.int16), c_van.view(torch.int16))
    raw = trace.cpu().numpy().view(np.uint32).copy()
    out = torch.zeros(kp.kp_stats_bytes(n_wg, waves, R), dtype=torch.uint8, device="cuda")
    kp.kp_trace_reduce(trace, n_wg * waves * 512, out)
    torch.cuda.synchronize()
    assert_stats_equal(oracle_mod.decode_bytes(raw, 8), out.cpu().numpy(), oracle_mod)
    st = kp.parse_stats(out)
    # 64 K-steps x 3 regions x 2 + 2 epilogue records = 386 per wave into 512 slots
    assert st["n_dropped"] == 0 and st["n_slots_valid"] == 386 * n_wg * waves
    assert st["n_pairs"] == 193 * n_wg * waves and st["n_orphan_end"] == 0 and st["n_orphan_start"] == 0
    per = n_wg * waves
    assert st["cnt"].tolist() == [64 * per, 64 * per, 64 * per, per]
    assert st["n_invalid"] == 0 and st["n_nonmonotonic"] == 0 and st["n_span_overflow_wgs"] == 0


def test_real_trace_carries_the_record_cost(kp, oracle_mod):
    """Replay takes the constant cost of a record off every duration (Sec. 4.3).  The cost set with
    kp_set_rec_cost goes into the header of a trace recorded afterwards, and both decoders subtract it:
    the durations of a real GEMM trace drop by exactly that much per pair (none of them is shorter)."""
    from tests.gpu_util import assert_stats_equal

    a, b = inputs.gemm_inputs(256, 256, 256, seed=0, dist="uniform")
    stats = {}
    for cost in (0, 37):
        kp.kp_set_rec_cost(cost)
        try:
            _, trace, (n_wg, waves, R) = run_gemm(kp, a, b, 0b111, trace_cap=512)
        finally:
            kp.kp_set_rec_cost(0)
        raw = trace.cpu().numpy().view(np.uint32).copy()
        assert raw[6] == cost
        out = torch.zeros(kp.kp_stats_bytes(n_wg, waves, R), dtype=torch.uint8, device="cuda")
        kp.kp_trace_reduce(trace, n_wg * waves * 128, out)
        torch.cuda.synchronize()
        assert_stats_equal(oracle_mod.decode_bytes(raw, 8), out.cpu().numpy(), oracle_mod)
        stats[cost] = (kp.parse_stats(out), raw)
    st, raw = stats[37]
    # the same trace decoded without the compensation: every pair is 37 ticks longer
    raw0 = raw.copy()
    raw0[6] = 0
    st0 = oracle_mod.view_stats(oracle_mod.decode_bytes(raw0, 8))
    assert st0["min"].min() > 37
    assert np.array_equal(st0["sum"] - st["sum"], 37 * st["cnt"])
    assert np.array_equal(st0["U"], st["U"])  # overlap uses the uncompensated intervals


def run_gemm_phased(kp, a, b, regions, trace_cap=None, extra=0):
    """The 256x256x64 kernel with the stages of a K step one after the other (KP_MASK_PHASES, 5 regions)."""
    M, K = a.shape
    N = b.shape[1]
    A, B = a.cuda(), b.cuda()
    C = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    n_wg, waves, _ = kp.kp_gemm_launch_shape(M, N, K)
    trace = None
    if regions:
        trace = torch.full((kp.kp_trace_bytes(n_wg, waves, trace_cap),), 0x77, dtype=torch.uint8, device="cuda")
    kp.kp_gemm_instrumented(A, B, C, M, N, K, regions | kp.KP_MASK_PHASES | extra, trace, trace_cap or 0)
    torch.cuda.synchronize()
    return C, trace, (n_wg, waves, 5)


@pytest.mark.parametrize("shape", [(1024, 1024, 512), (4096, 4096, 4096)])
def test_stage_by_stage_regions(kp, oracle_mod, shape):
    """The configured region set of the large GEMM (Sec. 5.3: a software-pipelined GEMM timed stage by
    stage): load issue, wait, LDS write, MFMA once per K-step and one epilogue, (4 x K/64 + 1) x 2
    records per wave (514 at K = 4096) into a ring of 4096 records per workgroup.  C is bit-identical
    to the default kernel's, the trace decodes like the oracle says and holds the closed-form counts."""
    from tests.gpu_util import assert_stats_equal

    M, N, K = shape
    a, b = inputs.gemm_inputs(M, N, K, seed=2 if M == 4096 else 21)
    c_ref, _, _ = run_gemm(kp, a, b, 0)
    c_van, _, _ = run_gemm_phased(kp, a, b, 0)
    assert torch.equal(c_van.view(torch.int16), c_ref.view(torch.int16))
    c_loose, _, _ = run_gemm_phased(kp, a, b, 0, extra=kp.KP_MASK_UNFENCED)   # the same source without scheduling fences
    assert torch.equal(c_loose.view(torch.int16), c_ref.view(torch.int16))
    c_ins, trace, (n_wg, waves, R) = run_gemm_phased(kp, a, b, 0b11111, trace_cap=4096)
    assert torch.equal(c_ins.view(torch.int16), c_ref.view(torch.int16))
    raw = trace.cpu().numpy().view(np.uint32).copy()
    assert tuple(raw[2:8]) == (n_wg, waves, 5, 512, 0, 0)
    out = torch.zeros(kp.kp_stats_bytes(n_wg, waves, R), dtype=torch.uint8, device="cuda")
    kp.kp_trace_reduce(trace, n_wg * waves * 512, out)
    torch.cuda.synchronize()
    assert_stats_equal(oracle_mod.decode_bytes(raw, 8), out.cpu().numpy(), oracle_mod)
    st = kp.parse_stats(out)
    steps, per = K // 64, n_wg * waves
    total = (4 * steps + 1) * 2
    assert (raw[16:16 + 32 * n_wg].reshape(n_wg, 32)[:, 8:16] == total).all()
    # 514 records per wave at K = 4096 into 512 slots: the two oldest, START and END of the first LDS write, are lost
    lost = max(0, total - 512)
    assert lost in (0, 2) and st["n_dropped"] == per * lost
    assert st["n_slots_valid"] == per * (total - lost) and st["n_pairs"] == per * (total - lost) // 2
    assert st["cnt"].tolist() == [steps * per, steps * per, (steps - lost // 2) * per, steps * per, per]
    for k in ("n_orphan_start", "n_orphan_end", "n_invalid", "n_disorder", "n_nonmonotonic", "n_span_overflow_wgs"):
        assert st[k] == 0, k
    # regions of one wave follow one another: their total time fits in the workgroup span
    hdr = raw[16:16 + 32 * n_wg].reshape(n_wg, 32).astype(np.uint64)
    span = ((hdr[:, 4] | (hdr[:, 5] << np.uint64(32))) - (hdr[:, 2] | (hdr[:, 3] << np.uint64(32)))).astype(np.int64)
    assert (st["per"]["sum"].sum(axis=2).astype(np.int64) <= span[:, None]).all()
    # a subset of the regions (generic record sites) and the flush strategy leave C alone too
    c_m, trace_m, _ = run_gemm_phased(kp, a, b, 0b01010, trace_cap=4096)
    assert torch.equal(c_m.view(torch.int16), c_ref.view(torch.int16))
    raw_m = trace_m.cpu().numpy().view(np.uint32).copy()
    out_m = torch.zeros_like(out)
    kp.kp_trace_reduce(trace_m, n_wg * waves * 512, out_m)
    torch.cuda.synchronize()
    assert_stats_equal(oracle_mod.decode_bytes(raw_m, 8), out_m.cpu().numpy(), oracle_mod)
    assert kp.parse_stats(out_m)["cnt"].tolist() == [0, steps * per, 0, steps * per, 0]


def test_stage_by_stage_needs_the_large_tile(kp):
    a, b = inputs.gemm_inputs(256, 256, 256, seed=0)
    with pytest.raises(kp.KperfError) as e:
        run_gemm_phased(kp, a, b, 0)
    assert e.value.status == kp.KP_ERR_INVALID_ARG
    a, b = inputs.gemm_inputs(1024, 1024, 256, seed=0)
    n_wg, waves, _ = kp.kp_gemm_launch_shape(1024, 1024, 256)
    with pytest.raises(kp.KperfError) as e:
        run_gemm_phased(kp, a, b, 0b100000, trace_cap=4096)   # region 5 does not exist
    assert e.value.status == kp.KP_ERR_INVALID_ARG
    # the unfenced form exists without record sites only, and only of the staged schedule
    with pytest.raises(kp.KperfError) as e:
        run_gemm_phased(kp, a, b, 0b11111, trace_cap=4096, extra=kp.KP_MASK_UNFENCED)
    assert e.value.status == kp.KP_ERR_INVALID_ARG
    A, B = a.cuda(), b.cuda()
    with pytest.raises(kp.KperfError) as e:
        kp.kp_gemm_instrumented(A, B, torch.empty(1024, 1024, dtype=torch.bfloat16, device="cuda"), 1024, 1024, 256,
                                kp.KP_MASK_UNFENCED, None, 0)
    assert e.value.status == kp.KP_ERR_INVALID_ARG


def _wg_headers(raw, n_wg):
    return raw[16:16 + 32 * n_wg].reshape(n_wg, 32)


@pytest.mark.gpu
@pytest.mark.parametrize("shape", [(1024, 1024, 512), (128, 128, 256)])
def test_constant_rate_clock_records(kp, oracle_mod, shape):
    """KP_MASK_REALTIME: the records carry the constant-rate 100 MHz clock (the MetricType of the counter
    read, Sec. 3.1).  Same records, decoded like the oracle says, C bit-identical; the workgroup spans
    on the two clocks give a shader clock between 1 and 2.6 GHz."""
    from tests.gpu_util import assert_stats_equal

    M, N, K = shape
    a, b = inputs.gemm_inputs(M, N, K, seed=21)
    n_wg, waves, R = kp.kp_gemm_launch_shape(M, N, K)
    cap_wave = 256
    A, B = a.cuda(), b.cuda()
    C = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    C0 = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    trace = torch.full((kp.kp_trace_bytes(n_wg, waves, waves * cap_wave),), 0x55, dtype=torch.uint8, device="cuda")
    kp.kp_gemm_instrumented(A, B, C, M, N, K, ((1 << R) - 1) | kp.KP_MASK_REALTIME, trace, waves * cap_wave)
    kp.kp_gemm_instrumented(A, B, C0, M, N, K, 0, None, 0)
    torch.cuda.synchronize()
    assert torch.equal(C.view(torch.int16), C0.view(torch.int16))
    raw = trace.cpu().numpy().view(np.uint32).copy()
    assert tuple(raw[2:6]) == (n_wg, waves, R, cap_wave) and raw[7] == kp.KP_FLAG_REALTIME
    out = torch.zeros(kp.kp_stats_bytes(n_wg, waves, R), dtype=torch.uint8, device="cuda")
    kp.kp_trace_reduce(trace, n_wg * waves * cap_wave, out)
    torch.cuda.synchronize()
    assert_stats_equal(oracle_mod.decode_bytes(raw, 8), out.cpu().numpy(), oracle_mod)
    st = kp.parse_stats(out)
    steps = K // 64 if waves == 8 else K // 32
    assert st["cnt"].tolist() == [n_wg * waves * steps] * 3 + ([n_wg * waves] if waves == 8 else [])
    for k in ("n_orphan_start", "n_orphan_end", "n_invalid", "n_dropped", "n_disorder", "n_nonmonotonic"):
        assert st[k] == 0, k
    hdr64 = _wg_headers(raw, n_wg)[:, 2:8].copy().view(np.uint64)   # t_begin, t_end, reserved
    span_rt = (hdr64[:, 1] - hdr64[:, 0]).astype(np.float64)        # 100 MHz ticks
    span_clk = hdr64[:, 2].astype(np.float64)                        # the same stretch on the shader clock
    ghz = span_clk.sum() / span_rt.sum() * 0.1
    assert 1.0 < ghz < 2.6, ghz
    # a duration in 100 MHz ticks cannot exceed its workgroup's span
    assert int(st["max"].max()) <= int(span_rt.max())


@pytest.mark.gpu
@pytest.mark.parametrize("shape,extra", [((1024, 1024, 512), 0), ((1024, 1024, 512), "flush"), ((128, 128, 256), 0)])
def test_collaborative_store_gives_the_same_records(kp, oracle_mod, shape, extra):
    """KP_MASK_COLLAB (Sec. 4.2, the store for AMD): all 64 lanes write a record to one address, and the
    wave's hardware id goes to the workgroup header.  The tag words are those of the one-lane store, the
    decode matches the oracle, C is bit-identical, and the ids of a workgroup's waves name one compute
    unit and distinct (SIMD, wave slot) pairs."""
    from tests.gpu_util import assert_stats_equal

    M, N, K = shape
    a, b = inputs.gemm_inputs(M, N, K, seed=22)
    n_wg, waves, R = kp.kp_gemm_launch_shape(M, N, K)
    cap_wave = 128
    A, B = a.cuda(), b.cuda()
    flush = kp.KP_MASK_FLUSH if extra == "flush" else 0
    regions = (1 << R) - 1 - 2     # region 1 off: both runs go through the generic sites
    traces, outs = [], []
    for collab in (0, kp.KP_MASK_COLLAB):
        C = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
        trace = torch.full((kp.kp_trace_bytes(n_wg, waves, waves * cap_wave),), 0x33, dtype=torch.uint8, device="cuda")
        kp.kp_gemm_instrumented(A, B, C, M, N, K, regions | flush | collab, trace, waves * cap_wave)
        torch.cuda.synchronize()
        traces.append(trace.cpu().numpy().view(np.uint32).copy())
        outs.append(C.view(torch.int16).cpu())
        st_out = torch.zeros(kp.kp_stats_bytes(n_wg, waves, R), dtype=torch.uint8, device="cuda")
        kp.kp_trace_reduce(trace, n_wg * waves * cap_wave, st_out)
        torch.cuda.synchronize()
        assert_stats_equal(oracle_mod.decode_bytes(traces[-1], 8), st_out.cpu().numpy(), oracle_mod)
    C0 = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    kp.kp_gemm_instrumented(A, B, C0, M, N, K, 0, None, 0)
    torch.cuda.synchronize()
    assert torch.equal(outs[0], C0.view(torch.int16).cpu()) and torch.equal(outs[1], outs[0])
    plain, collab = traces
    assert plain[7] == (1 if flush else 0) and collab[7] == (1 if flush else 0) | kp.KP_FLAG_HW_IDS
    h0, h1 = _wg_headers(plain, n_wg), _wg_headers(collab, n_wg)
    assert (h0[:, 8:24] == h1[:, 8:24]).all()                       # records written per wave
    assert (h0[:, 24:32] == 0).all()
    first = 16 + 32 * n_wg
    rec0 = plain[first:].reshape(n_wg, waves, cap_wave, 2)
    rec1 = collab[first:].reshape(n_wg, waves, cap_wave, 2)
    held = np.minimum(h0[:, 8:8 + waves], cap_wave)                 # slots that hold a record
    valid = np.arange(cap_wave)[None, None, :] < held[:, :, None]
    assert (rec0[..., 0][valid] == rec1[..., 0][valid]).all()       # the tag words
    ids = h1[:, 24:32].copy().view(np.uint16).reshape(n_wg, 16)
    assert (ids[:, waves:] == 0).all() and (ids < 4096).all()
    cu = ids[:, :waves] >> 8
    assert (cu == cu[:, :1]).all()                                  # one compute unit per workgroup
    slot = ids[:, :waves] & 0x3F                                    # wave slot and SIMD
    assert all(len(set(row.tolist())) == waves for row in slot)

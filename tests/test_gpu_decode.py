"""GPU decoder (kp_trace_reduce, through the C ABI) against the CPU oracle, bit for bit."""
import numpy as np
import pytest
import torch

import inputs
from inputs import PHASE_END as E
from inputs import PHASE_START as S

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kp():
    import paper_2505_21661_amd as kp

    return kp


def check(raw, oracle_mod, use_hdr=False, threads=8):
    from tests.gpu_util import assert_stats_equal, gpu_decode_bytes

    want = oracle_mod.decode_bytes(raw, threads)
    got = gpu_decode_bytes(raw, use_hdr=use_hdr)
    assert_stats_equal(want, got, oracle_mod)


def test_hand_patterns(kp, oracle_mod):
    cases = [
        ([[(S, 0, 10), (E, 0, 30), (S, 1, 40), (E, 1, 100)]], 2, 16),
        ([[(S, 0, 10), (S, 1, 20), (E, 1, 50), (E, 0, 90)]], 2, 16),
        ([[(S, 0, 0), (E, 0, 5), (S, 0, 8), (E, 0, 16), (S, 0, 20), (E, 0, 21)]], 1, 16),
        ([[(S, 0, 0), (E, 0, 10)], [(S, 1, 5), (S, 0, 12), (E, 1, 15), (E, 0, 20)]], 2, 16),
        ([[(S, 0, 0), (E, 0, 10)], [(S, 0, 5), (E, 0, 15)]], 1, 16),
        ([[(S, 0, 0), (E, 0, 10), (S, 1, 20), (E, 1, 30), (S, 0, 40), (E, 0, 50), (S, 1, 60)]], 2, 4),
        ([[(S, 0, 0), (S, 0, 7), (E, 0, 10), (E, 0, 30)]], 1, 16),
        ([[], []], 2, 8),
        # equal timestamps across waves and inside a wave
        ([[(S, 0, 5), (E, 0, 5), (S, 1, 5), (E, 1, 9)], [(S, 1, 5), (E, 1, 9), (S, 0, 9), (E, 0, 9)],
          [(S, 0, 5), (S, 1, 5), (E, 0, 9), (E, 1, 9)]], 2, 8),
    ]
    for evs, R, cap in cases:
        for flush in (False, True):
            wg = inputs.events_to_wg(evs, cap, flush=flush)
            raw = inputs.encode_trace([wg], len(evs), R, cap, rec_cost=1, flush=flush)
            check(raw, oracle_mod)
            check(raw, oracle_mod, use_hdr=True)


def test_clock_wrap_and_span_overflow(kp, oracle_mod):
    wg = inputs.events_to_wg([[(S, 0, 0xFFFFFFF0), (E, 0, 0x10)]], 8, t_end=1000 + (1 << 32) + 100)
    check(inputs.encode_trace([wg], 1, 1, 8), oracle_mod)


@pytest.mark.parametrize("seed", range(24))
def test_messy_traces(kp, oracle_mod, seed):
    waves = [1, 2, 3, 4, 7, 8, 16][seed % 7]
    n_regions = [1, 3, 5, 16, 17, 32][seed % 6]
    cap = [2, 8, 16, 64, 256][seed % 5]
    raw = inputs.messy_trace(1000 + seed, n_wg=9, waves=waves, n_regions=n_regions, cap_wave=cap,
                             p_bad=0.03 if seed % 3 else 0.0, allow_nonmono=bool(seed % 2),
                             flush=(seed % 4 == 3))
    check(raw, oracle_mod, use_hdr=bool(seed & 1))


def test_small_gemm_shape_trace(kp, oracle_mod):
    raw, _ = inputs.gen_trace(inputs.spec_small_gemm_shape())
    check(raw, oracle_mod)


@pytest.mark.parametrize("log2n,wrap", [(17, False), (20, False), (20, True), (22, False)])
def test_decode_workload_scaled(kp, oracle_mod, log2n, wrap):
    raw, _ = inputs.gen_trace(inputs.spec_decode_standalone(log2n, wrap=wrap))
    check(raw, oracle_mod, use_hdr=True)


@pytest.mark.parametrize("W,R,cap,total", [(4, 5, 1024, 1500), (8, 20, 1024, 1024), (16, 16, 1024, 700),
                                             (2, 32, 4096, 4096), (5, 3, 512, 512), (1, 2, 16384, 20000)])
def test_other_geometries(kp, oracle_mod, W, R, cap, total):
    spec = inputs.TraceSpec(n_wg=37, waves=W, n_regions=R, cap_wave=cap, total_per_wave=total, total_var=total // 3,
                            seed=W * 100 + R, dist="lognormal", p0=5.0, p1=1.2, p_orphan=0.03, p_swap=0.002)
    raw, _ = inputs.gen_trace(spec)
    check(raw, oracle_mod)


@pytest.mark.parametrize("p0", [0.0, 1.0, 2.0, 3.0, 4.0, 5.0, 6.5, 8.0, 10.0, 12.0, 14.0])
def test_spans_from_a_few_ticks_to_many_million(kp, oracle_mod, p0):
    """The overlap sweep bins a workgroup's records into time cells whose width follows the workgroup's
    span; spans from fewer ticks than cells to 2^27 ticks take every form of that width (and, at the
    long end, the wide merge keys), and the phase offsets give every workgroup a different span."""
    for W, cap, seed in ((8, 128, 1), (3, 1024, 2)):
        spec = inputs.TraceSpec(n_wg=24, waves=W, n_regions=6, cap_wave=cap, total_per_wave=cap, seed=seed + int(10 * p0),
                                dist="lognormal", p0=p0, p1=0.7, gap_max=1 if p0 < 3 else 32, phase_min=0,
                                phase_max=int(2 ** min(p0 + 2, 12)) - 1, p_orphan=0.01)
        raw, _ = inputs.gen_trace(spec)
        n_wg = int(raw[2])
        hdr = raw[16:16 + 32 * n_wg].reshape(n_wg, 32).astype(np.uint64)
        span = (hdr[:, 4] | (hdr[:, 5] << np.uint64(32))) - (hdr[:, 2] | (hdr[:, 3] << np.uint64(32)))
        assert span.max() < 2 ** 32
        check(raw, oracle_mod)


def test_empty_trace(kp, oracle_mod):
    check(inputs.encode_trace([], 4, 3, 8), oracle_mod)


def test_errors(kp):
    raw, _ = inputs.gen_trace(inputs.spec_small_gemm_shape())
    n_wg, W, R, cap = (int(x) for x in raw[2:6])
    dev = torch.from_numpy(raw.view(np.int32)).cuda()
    out = torch.zeros(kp.kp_stats_bytes(n_wg, W, R), dtype=torch.uint8, device="cuda")
    with pytest.raises(kp.KperfError) as e:
        kp.kp_trace_reduce(dev, n_wg * W * cap + 1, out)
    assert e.value.status == kp.KP_ERR_BAD_TRACE
    bad = raw.copy(); bad[0] ^= 4
    with pytest.raises(kp.KperfError) as e:
        kp.kp_trace_reduce(torch.from_numpy(bad.view(np.int32)).cuda(), n_wg * W * cap, out)
    assert e.value.status == kp.KP_ERR_BAD_TRACE
    # more record slots per workgroup than any kernel takes; more regions than the tag names
    with pytest.raises(kp.KperfError) as e:
        kp.kp_trace_reduce_hdr(dev, 16 * (1 << 16), kp.make_hdr(1, 16, 4, 1 << 16), out)
    assert e.value.status == kp.KP_ERR_UNSUPPORTED_SHAPE
    with pytest.raises(kp.KperfError) as e:
        kp.kp_trace_reduce_hdr(dev, n_wg * W * cap, kp.make_hdr(n_wg, W, 129, cap), out)
    assert e.value.status == kp.KP_ERR_BAD_TRACE
    # host header that disagrees with the device header: flagged in the stats block, no statistics
    kp.kp_trace_reduce_hdr(dev, n_wg * W * cap, kp.make_hdr(n_wg, W, R + 1, cap),
                           torch.zeros(kp.kp_stats_bytes(n_wg, W, R + 1), dtype=torch.uint8, device="cuda"))
    st_buf = torch.zeros(kp.kp_stats_bytes(n_wg, W, R + 1), dtype=torch.uint8, device="cuda")
    kp.kp_trace_reduce_hdr(dev, n_wg * W * cap, kp.make_hdr(n_wg, W, R + 1, cap), st_buf)
    torch.cuda.synchronize()
    st = kp.parse_stats(st_buf)
    assert st["status"] == 1 and st["n_pairs"] == 0


def test_repeated_calls_are_deterministic(kp, oracle_mod):
    from tests.gpu_util import gpu_decode_bytes

    raw, _ = inputs.gen_trace(inputs.spec_decode_standalone(19))
    dev = torch.from_numpy(raw.view(np.int32)).cuda()
    first = gpu_decode_bytes(raw, dev_raw=dev)
    for _ in range(3):
        assert np.array_equal(first, gpu_decode_bytes(raw, use_hdr=True, dev_raw=dev))


def test_decode_workload_full_size(kp, oracle_mod):
    """The benchmark's decode workload at its full size (2^28 records, 16384 workgroups x 8 waves x
    2048 records, 16 regions) in the launch configuration bench.py times (kp_trace_reduce_hdr,
    kp_trace_pairs_hdr, kp_trace_waits_hdr and kp_pairs_stages): the whole statistics block, every
    timeline row, the whole waits block and the whole stage table, bit for bit."""
    import os

    spec = inputs.spec_decode_standalone(28)
    raw, _ = inputs.gen_trace(spec)
    n = spec.n_slots
    dev_raw = torch.from_numpy(raw.view(np.int32)).cuda()
    hdr = kp.make_hdr(spec.n_wg, spec.waves, spec.n_regions, spec.cap_wave)
    out = torch.full((kp.kp_stats_bytes(spec.n_wg, spec.waves, spec.n_regions),), 0xAB, dtype=torch.uint8, device="cuda")
    kp.kp_trace_reduce_hdr(dev_raw, n, hdr, out)
    rows = torch.full((kp.kp_pairs_bytes(spec.n_wg, spec.waves, spec.waves * spec.cap_wave),), 0xA5, dtype=torch.uint8,
                      device="cuda")
    kp.kp_trace_pairs_hdr(dev_raw, n, hdr, rows)
    waits = torch.full((kp.kp_waits_bytes(spec.n_wg, spec.waves, spec.n_regions),), 0x5A, dtype=torch.uint8, device="cuda")
    kp.kp_trace_waits_hdr(dev_raw, n, hdr, waits)
    max_iter = 64
    stages = torch.full((kp.kp_stages_bytes(spec.n_wg, spec.n_regions, max_iter),), 0x3C, dtype=torch.uint8, device="cuda")
    kp.kp_pairs_stages(rows, spec.n_wg, spec.waves, spec.waves * spec.cap_wave, spec.n_regions, max_iter, stages)
    torch.cuda.synchronize()
    from tests.gpu_util import assert_stats_equal

    want = oracle_mod.decode_bytes(raw, min(16, os.cpu_count() or 1))
    assert_stats_equal(want, out.cpu().numpy(), oracle_mod)
    st = kp.parse_stats(out)
    assert st["n_slots_valid"] == n and st["n_overlap_wgs"] == spec.n_wg and st["n_invalid"] == 0
    del out, want
    want_rows = oracle_mod.pairs_raw(raw, fill=0xA5)
    got_rows = rows.cpu().numpy()
    assert np.array_equal(want_rows, got_rows)
    want_stages = oracle_mod.stages_raw(want_rows, spec.n_wg, spec.waves, spec.cap_wave, spec.n_regions, max_iter)
    assert np.array_equal(want_stages, stages.cpu().numpy())
    del want_rows, got_rows, want_stages
    assert np.array_equal(oracle_mod.waits_raw(raw), waits.cpu().numpy())


def test_events_around_the_main_kernel(kp, oracle_mod):
    """kp_trace_reduce_hdr_events: the same statistics, and two events of the caller's recorded around the
    replay kernel (their distance is below that of events around the whole call)."""
    from tests.gpu_util import assert_stats_equal

    raw, _ = inputs.gen_trace(inputs.spec_decode_standalone(20))
    n_wg, W, R, cap = (int(x) for x in raw[2:6])
    dev = torch.from_numpy(raw.view(np.int32)).cuda()
    out = torch.full((kp.kp_stats_bytes(n_wg, W, R),), 0x5A, dtype=torch.uint8, device="cuda")
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    for e in ev:
        e.record()
    torch.cuda.synchronize()
    hdr = kp.make_hdr(n_wg, W, R, cap)
    ev[0].record()
    kp.kp_trace_reduce_hdr_events(dev, n_wg * W * cap, hdr, out, ev[1], ev[2])
    ev[3].record()
    torch.cuda.synchronize()
    assert_stats_equal(oracle_mod.decode_bytes(raw, 8), out.cpu().numpy(), oracle_mod)
    assert 0.0 < ev[1].elapsed_time(ev[2]) <= ev[0].elapsed_time(ev[3])
    kp.kp_trace_reduce_hdr_events(dev, n_wg * W * cap, hdr, out, None, None)   # events are optional
    torch.cuda.synchronize()
    with pytest.raises(ValueError):
        kp.kp_trace_reduce_hdr_events(dev, n_wg * W * cap, hdr, out, torch.cuda.Event(enable_timing=True), None)


def test_sequence_numbers_that_wrap(kp, oracle_mod):
    """Waves that wrote more than 2^20 records: the 20-bit sequence numbers wrap around inside the surviving
    tail of the ring (a generated trace with a multiple of the ring size added to every sequence number and
    to the waves' record counts)."""
    W, cap, n_wg = 8, 2048, 5
    spec = inputs.TraceSpec(n_wg=n_wg, waves=W, n_regions=16, cap_wave=cap, total_per_wave=2600, total_var=400,
                            seed=32, dist="exp", p0=30.0, gap_max=4, phase_max=10, p_orphan=0.01, p_swap=0.002)
    raw, _ = inputs.gen_trace(spec)
    shift = (1 << 20) - cap
    raw = raw.copy()
    hdrs = raw[16:16 + 32 * n_wg].reshape(n_wg, 32)
    assert (hdrs[:, 8:8 + W] > cap).all()
    hdrs[:, 8:8 + W] += shift
    recs = raw[16 + 32 * n_wg:].reshape(-1, 2)
    recs[:, 0] = (recs[:, 0] & 0xFFF00000) | ((recs[:, 0] + shift) & 0xFFFFF)
    check(raw, oracle_mod)
    check(raw, oracle_mod, use_hdr=True)

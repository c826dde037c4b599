"""GPU decoder on geometries outside the LDS-resident kernel's (more than 32 regions, more than 16384
record slots per workgroup) against the CPU oracle, bit for bit, through the C ABI."""
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
    return oracle_mod.view_stats(want)


def test_hand_patterns_with_many_regions(kp, oracle_mod):
    """The paper's record patterns (common, nested, multi-iteration; Sec. 4.3) with region numbers from the
    upper end of the tag's field, so that the multi-pass kernel decodes them."""
    a, b = 97, 127
    cases = [
        [[(S, a, 10), (E, a, 30), (S, b, 40), (E, b, 100)]],
        [[(S, a, 10), (S, b, 20), (E, b, 50), (E, a, 90)]],
        [[(S, a, 0), (E, a, 5), (S, a, 8), (E, a, 16), (S, a, 20), (E, a, 21)]],
        [[(S, a, 0), (E, a, 10)], [(S, b, 5), (S, a, 12), (E, b, 15), (E, a, 20)]],
        [[(S, 0, 0), (E, 0, 10)], [(S, 0, 5), (E, 0, 15)], [(S, 64, 7), (E, 64, 30)]],
        [[(S, a, 0), (S, a, 7), (E, a, 10), (E, a, 30)]],
        [[], []],
        [[(S, a, 5), (E, a, 5), (S, b, 5), (E, b, 9)], [(S, b, 5), (E, b, 9), (S, a, 9), (E, a, 9)],
         [(S, a, 5), (S, b, 5), (E, a, 9), (E, b, 9)]],
    ]
    for evs in cases:
        for flush in (False, True):
            for cap in (4, 16):
                wg = inputs.events_to_wg(evs, cap, flush=flush)
                raw = inputs.encode_trace([wg], len(evs), 128, cap, rec_cost=1, flush=flush)
                check(raw, oracle_mod)
                check(raw, oracle_mod, use_hdr=True)


@pytest.mark.parametrize("seed", range(18))
def test_messy_traces_with_many_regions(kp, oracle_mod, seed):
    waves = [1, 2, 3, 5, 8, 16][seed % 6]
    n_regions = [33, 64, 65, 100, 128][seed % 5]
    cap = [2, 8, 64, 256][seed % 4]
    raw = inputs.messy_trace(3000 + seed, n_wg=7, waves=waves, n_regions=n_regions, cap_wave=cap,
                             p_bad=0.03 if seed % 3 else 0.0, allow_nonmono=bool(seed % 2),
                             flush=(seed % 4 == 3))
    check(raw, oracle_mod, use_hdr=bool(seed & 1))


@pytest.mark.parametrize("seed", range(8))
def test_messy_traces_with_long_rings(kp, oracle_mod, seed):
    """Rings beyond what the LDS-resident kernel stages: several ranges of ranks per wave, several
    windows of the sweep, wrapped rings, corrupt records, duplicated seq, swapped slots."""
    waves = [16, 3, 8, 1][seed % 4]
    cap = [2048, 8192, 4096, 32768][seed % 4]
    raw = inputs.messy_trace(4000 + seed, n_wg=3, waves=waves, n_regions=[5, 40][seed % 2], cap_wave=cap,
                             p_bad=0.0005 if seed % 3 == 1 else 0.0, allow_nonmono=False, flush=(seed == 5))
    st = check(raw, oracle_mod, use_hdr=bool(seed & 1))
    if seed % 3 != 1:
        assert st["n_overlap_wgs"] > 0


@pytest.mark.parametrize("W,R,cap,total", [(16, 8, 2048, 2048), (16, 5, 4096, 6000), (4, 12, 16384, 16384),
                                             (1, 3, 65536, 70000), (16, 128, 1024, 1024), (2, 64, 1024, 3000),
                                             (16, 128, 8192, 8192), (16, 16, 32768, 20000)])
def test_generated_traces(kp, oracle_mod, W, R, cap, total):
    """Traces in the shape of the decode workload (regions follow one another in every wave, lognormal
    durations, a few orphans and swapped slots) at wide geometries, up to the largest ones the kernel takes."""
    n_wg = 5 if W * cap >= (1 << 17) else 12
    spec = inputs.TraceSpec(n_wg=n_wg, waves=W, n_regions=R, cap_wave=cap, total_per_wave=total, total_var=total // 5,
                            seed=W * 1000 + R, dist="lognormal", p0=5.0, p1=1.0, p_orphan=0.02, p_swap=0.0005)
    raw, _ = inputs.gen_trace(spec)
    st = check(raw, oracle_mod, use_hdr=True)
    assert st["n_pairs"] > 0 and st["n_overlap_wgs"] > 0


@pytest.mark.parametrize("W,R,cap,p_swap", [(16, 8, 4096, 0.2), (16, 128, 1024, 0.15), (3, 40, 16384, 0.3), (8, 16, 8192, 0.004)])
def test_heavily_shuffled_rings(kp, oracle_mod, W, R, cap, p_swap):
    """So many records outside the slot of their sequence number that the kernel's list of them overflows
    (it then scans all slots for every range of ranks), and, in the last case, a list that is nearly full."""
    spec = inputs.TraceSpec(n_wg=4, waves=W, n_regions=R, cap_wave=cap, total_per_wave=cap + cap // 2, total_var=cap // 4,
                            seed=W + R, dist="lognormal", p0=4.0, p1=1.0, p_orphan=0.02, p_swap=p_swap, swap_max=40)
    raw, _ = inputs.gen_trace(spec)
    st = check(raw, oracle_mod)
    assert st["n_disorder"] > 0.5 * p_swap * st["n_slots_valid"] and st["n_overlap_wgs"] > 0


def test_sequence_numbers_that_wrap(kp, oracle_mod):
    """Waves that wrote more than 2^20 records: the 20-bit sequence numbers wrap around inside the
    surviving tail of the ring; the rank is still seq - first modulo 2^20.  Built from a generated trace by
    adding a multiple of the ring size to every sequence number and to the waves' record counts."""
    W, cap = 8, 4096
    spec = inputs.TraceSpec(n_wg=3, waves=W, n_regions=40, cap_wave=cap, total_per_wave=5000, total_var=600,
                            seed=31, dist="exp", p0=30.0, gap_max=4, phase_max=10, p_orphan=0.01, p_swap=0.002)
    raw, _ = inputs.gen_trace(spec)
    shift = (1 << 20) - cap
    raw = raw.copy()
    hdrs = raw[16:16 + 32 * 3].reshape(3, 32)
    assert (hdrs[:, 8:8 + W] > cap).all()            # every ring has wrapped, so every slot holds a record
    hdrs[:, 8:8 + W] += shift
    recs = raw[16 + 32 * 3:].reshape(-1, 2)
    recs[:, 0] = (recs[:, 0] & 0xFFF00000) | ((recs[:, 0] + shift) & 0xFFFFF)
    first = hdrs[:, 8:8 + W].astype(np.int64) - cap
    assert (first < (1 << 20)).all() and (first + cap > (1 << 20)).all()   # the wrap lies inside the tail
    st = check(raw, oracle_mod)
    assert st["n_invalid"] == 0 and st["n_pairs"] > 3 * W * cap // 3 and st["n_overlap_wgs"] == 3
    assert st["n_dropped"] == int((hdrs[:, 8:8 + W].astype(np.int64) - cap).sum())


def test_clean_generated_trace_all_workgroups_in_the_overlap(kp, oracle_mod):
    spec = inputs.TraceSpec(n_wg=300, waves=16, n_regions=48, cap_wave=512, total_per_wave=512, total_var=60, seed=77,
                            dist="lognormal", p0=4.5, p1=0.8)
    raw, _ = inputs.gen_trace(spec)
    st = check(raw, oracle_mod)
    assert st["n_overlap_wgs"] == 300 and st["n_invalid"] == 0


def test_span_overflow_and_nonmonotonic_workgroups_stay_out_of_the_overlap(kp, oracle_mod):
    evs = [[(S, 40, 10), (E, 40, 30)], [(S, 41, 12), (E, 41, 50)]]
    ok = inputs.events_to_wg(evs, 8)
    long_one = inputs.events_to_wg(evs, 8, t_end=1000 + (1 << 32) + 3)
    back = inputs.events_to_wg([[(S, 40, 10), (E, 40, 30), (S, 40, 20), (E, 40, 25)], [(S, 41, 12), (E, 41, 50)]], 8)
    raw = inputs.encode_trace([ok, long_one, back, ok], 2, 42, 8)
    st = check(raw, oracle_mod)
    assert st["n_overlap_wgs"] == 2 and st["n_span_overflow_wgs"] == 1 and st["n_nonmonotonic"] == 1


def test_empty_trace_and_limits(kp, oracle_mod):
    check(inputs.encode_trace([], 4, 100, 8), oracle_mod)
    dev = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    out = torch.zeros(kp.kp_stats_bytes(1, 16, 128), dtype=torch.uint8, device="cuda")
    # more record slots per workgroup than the kernel has bits for
    for R, cap in ((128, 16384), (8, 65536)):
        with pytest.raises(kp.KperfError) as e:
            kp.kp_trace_reduce_hdr(dev, 16 * cap, kp.make_hdr(1, 16, R, cap), out)
        assert e.value.status == kp.KP_ERR_UNSUPPORTED_SHAPE
    with pytest.raises(kp.KperfError) as e:
        kp.kp_trace_reduce_hdr(dev, 16 * 64, kp.make_hdr(1, 16, 129, 64), out)
    assert e.value.status == kp.KP_ERR_BAD_TRACE
    with pytest.raises(kp.KperfError) as e:   # single steps exist for the LDS-resident kernel only
        kp.kp_trace_reduce_steps(dev, 16 * 64, kp.make_hdr(1, 16, 40, 64), out, 3)
    assert e.value.status == kp.KP_ERR_UNSUPPORTED_SHAPE

"""Pins for the CPU trace-decode oracle (no GPU).

Each test checks oracle/ref_decode.c against something other than itself:
hand-worked traces for the record patterns the paper names (Sec. 4.2, "SM-level
Data Layout": common, nested, multi-iteration), the circular-buffer tail rule
(Sec. 4.2 "Shared Memory Circular Buffer"), the 2^32 clock rule (Sec. 4.2,
32-bit clock paragraph), an independent tick-by-tick brute force, construction
truth from the generator, and invariants / metamorphic relations.
"""
import numpy as np
import pytest

import inputs
from inputs import PHASE_END as E
from inputs import PHASE_START as S
from tests.brute import assert_same, brute_decode

U64MAX = np.iinfo(np.uint64).max


def one_wg(oracle_mod, wave_events, n_regions, cap_wave=16, rec_cost=0, flush=False, **kw):
    wg = inputs.events_to_wg(wave_events, cap_wave, flush=flush, **kw)
    raw = inputs.encode_trace([wg], len(wave_events), n_regions, cap_wave, rec_cost=rec_cost, flush=flush)
    return raw, oracle_mod.decode(raw)


# ---- layout pins --------------------------------------------------------------------------

def test_record_is_8_bytes_and_64_slots_are_half_a_kb():
    # Sec. 4.2: 8-byte records; 64 slots = 0.5 KB; two groups share them as 32 slots each.
    payload = inputs.trace_bytes(1, 2, 32) - inputs.HDR_BYTES - inputs.WGHDR_BYTES
    assert payload == 512
    assert inputs.trace_bytes(1, 1, 64) - inputs.trace_bytes(1, 1, 0) == 64 * 8


def test_flag_bit_is_one_bit_of_the_tag():
    assert inputs.make_tag(E, 0, 0, 0) ^ inputs.make_tag(S, 0, 0, 0) == 1 << 31


# ---- hand-worked patterns ---------------------------------------------------------------------

def test_common_pattern(oracle_mod):
    _, st = one_wg(oracle_mod, [[(S, 0, 10), (E, 0, 30), (S, 1, 40), (E, 1, 100)]], 2)
    assert st["n_pairs"] == 2 and st["n_orphan_start"] == 0 and st["n_orphan_end"] == 0
    assert st["cnt"].tolist() == [1, 1] and st["sum"].tolist() == [20, 60]
    assert st["hist"][0, 4] == 1 and st["hist"][1, 5] == 1 and st["hist"].sum() == 2
    assert st["U"].tolist() == [20, 60]
    assert st["O"].tolist() == [[20, 0], [0, 60]]
    assert st["F"].tolist() == [[1.0, 0.0], [0.0, 1.0]]
    assert st["per"]["sum"][0, 0].tolist() == [20, 60]


def test_nested_pattern(oracle_mod):
    _, st = one_wg(oracle_mod, [[(S, 0, 10), (S, 1, 20), (E, 1, 50), (E, 0, 90)]], 2)
    assert st["n_pairs"] == 2
    assert st["sum"].tolist() == [80, 30]
    assert st["hist"][0, 6] == 1 and st["hist"][1, 4] == 1
    assert st["U"].tolist() == [80, 30]
    assert st["O"].tolist() == [[80, 30], [30, 30]]
    assert st["F"][1, 0] == 1.0 and st["F"][0, 1] == 0.375


def test_multi_iteration_pattern(oracle_mod):
    ev = [(S, 0, 0), (E, 0, 5), (S, 0, 8), (E, 0, 16), (S, 0, 20), (E, 0, 21)]
    _, st = one_wg(oracle_mod, [ev], 1)
    assert st["n_pairs"] == 3
    assert (st["cnt"][0], st["sum"][0], st["min"][0], st["max"][0]) == (3, 14, 1, 8)
    assert st["hist"][0, 2] == 1 and st["hist"][0, 3] == 1 and st["hist"][0, 0] == 1
    assert st["U"][0] == 14
    p = st["per"][0, 0, 0]
    assert (p["sum"], p["n"], p["max"]) == (14, 3, 8)


def test_overlap_is_union_over_waves(oracle_mod):
    # wave0: r0 [0,10)   wave1: r1 [5,15), r0 [12,20)
    _, st = one_wg(oracle_mod, [[(S, 0, 0), (E, 0, 10)], [(S, 1, 5), (S, 0, 12), (E, 1, 15), (E, 0, 20)]], 2)
    assert st["U"].tolist() == [18, 10]
    assert st["O"][0, 1] == 8 and st["O"][1, 0] == 8
    # same region active in two waves at once counts once
    _, st = one_wg(oracle_mod, [[(S, 0, 0), (E, 0, 10)], [(S, 0, 5), (E, 0, 15)]], 1)
    assert st["U"][0] == 15 and st["sum"][0] == 20


def test_circular_buffer_keeps_tail(oracle_mod):
    # 7 records into a 4-slot sub-ring: the first 3 are overwritten.
    ev = [(S, 0, 0), (E, 0, 10), (S, 1, 20), (E, 1, 30), (S, 0, 40), (E, 0, 50), (S, 1, 60)]
    raw, st = one_wg(oracle_mod, [ev], 2, cap_wave=4)
    assert st["n_dropped"] == 3 and st["n_slots_valid"] == 4
    assert st["n_orphan_end"] == 1      # E1@30 lost its START
    assert st["n_orphan_start"] == 1    # S1@60 never ended
    assert st["n_pairs"] == 1 and st["sum"].tolist() == [10, 0]
    assert st["n_disorder"] == 0 and st["n_invalid"] == 0
    # nested variant: 6 written, 4 kept, survivors E1 E0 S2 E2
    ev = [(S, 0, 0), (S, 1, 5), (E, 1, 9), (E, 0, 12), (S, 2, 20), (E, 2, 27)]
    _, st = one_wg(oracle_mod, [ev], 3, cap_wave=4)
    assert (st["n_dropped"], st["n_orphan_end"], st["n_pairs"]) == (2, 2, 1)
    assert st["sum"].tolist() == [0, 0, 7]


def test_flush_strategy_keeps_head(oracle_mod):
    ev = [(S, 0, 0), (E, 0, 10), (S, 1, 20), (E, 1, 30), (S, 0, 40), (E, 0, 50), (S, 1, 60)]
    _, st = one_wg(oracle_mod, [ev], 2, cap_wave=4, flush=True)
    assert st["n_dropped"] == 3 and st["n_pairs"] == 2 and st["sum"].tolist() == [10, 10]
    assert st["n_orphan_end"] == 0 and st["n_orphan_start"] == 0


def test_start_start_end_pairs_the_inner_start(oracle_mod):
    _, st = one_wg(oracle_mod, [[(S, 0, 0), (S, 0, 7), (E, 0, 10), (E, 0, 30)]], 1)
    assert (st["n_pairs"], st["n_orphan_start"], st["n_orphan_end"]) == (1, 1, 1)
    assert st["sum"][0] == 3 and st["U"][0] == 3


def test_clock_wrap_inside_interval(oracle_mod):
    # Sec. 4.2: a 32-bit clock stays usable while an interval is shorter than 2^32 ticks.
    ev = [(S, 0, 0xFFFFFFF0), (E, 0, 0x00000010)]
    _, st = one_wg(oracle_mod, [ev], 1, t_end=1000 + (1 << 32) + 100)
    assert st["n_pairs"] == 1 and st["sum"][0] == 0x20
    # ... and the overflow is detected: the workgroup is flagged and left out of the overlap sums
    assert st["n_span_overflow_wgs"] == 1 and st["n_nonmonotonic"] == 1 and st["n_overlap_wgs"] == 0
    assert st["U"][0] == 0


def test_record_cost_is_subtracted_saturating(oracle_mod):
    # Sec. 4.3: synchronous regions are rebuilt by subtracting the constant record overhead.
    ev = [(S, 0, 0), (E, 0, 100), (S, 0, 200), (E, 0, 210)]
    _, st = one_wg(oracle_mod, [ev], 1, rec_cost=25)
    assert st["sum"][0] == 75 + 0 and st["min"][0] == 0 and st["max"][0] == 75
    assert st["U"][0] == 110  # overlap uses the raw clock interval


def test_empty_and_degenerate(oracle_mod):
    _, st = one_wg(oracle_mod, [[], []], 2)
    assert st["n_slots_valid"] == 0 and st["n_pairs"] == 0 and st["n_overlap_wgs"] == 1
    assert all(int(m) == int(U64MAX) for m in st["min"])
    raw = inputs.encode_trace([], 4, 3, 8)
    st = oracle_mod.decode(raw)
    assert st["n_wg"] == 0 and st["per"].size == 0


def test_bad_header_is_rejected(oracle_mod):
    raw, _ = one_wg(oracle_mod, [[(S, 0, 0), (E, 0, 1)]], 1)
    bad = raw.copy(); bad[0] ^= 1
    with pytest.raises(ValueError):
        oracle_mod.decode(bad)
    bad = raw.copy(); bad[5] = 12  # cap_wave not a power of two
    with pytest.raises(ValueError):
        oracle_mod.decode(bad)


def test_out_of_order_slots_are_reordered_by_seq(oracle_mod):
    ev = [(S, 0, 0), (E, 0, 10), (S, 1, 20), (E, 1, 35)]
    wg = inputs.events_to_wg([ev], 8)
    ref = oracle_mod.decode(inputs.encode_trace([wg], 1, 2, 8))
    seg = wg["slots"][0]
    seg[1], seg[3] = seg[3], seg[1]
    st = oracle_mod.decode(inputs.encode_trace([wg], 1, 2, 8))
    assert st["n_disorder"] == 2
    for k in ("hist", "cnt", "sum", "U", "O"):
        assert np.array_equal(st[k], ref[k])


# ---- brute force --------------------------------------------------------------------------

@pytest.mark.parametrize("seed", range(12))
def test_against_tick_by_tick_brute_force(oracle_mod, seed):
    raw = inputs.messy_trace(seed, n_wg=5, waves=1 + seed % 4, n_regions=1 + seed % 5, cap_wave=16,
                             p_bad=0.04 if seed % 3 else 0.0, allow_nonmono=bool(seed % 2),
                             flush=(seed % 4 == 3))
    assert_same(brute_decode(raw), oracle_mod.decode(raw))


@pytest.mark.parametrize("seed", range(4))
def test_generator_traces_against_brute_force(oracle_mod, seed):
    spec = inputs.TraceSpec(n_wg=3, waves=3, n_regions=4, cap_wave=32, total_per_wave=[20, 32, 70, 45][seed],
                            total_var=5, seed=seed, dist="exp", p0=40.0, gap_max=8, phase_max=50,
                            p_orphan=0.1, p_swap=0.05, swap_max=5, rec_cost=seed, flush=(seed == 3))
    raw, _ = inputs.gen_trace(spec)
    assert_same(brute_decode(raw), oracle_mod.decode(raw))


# ---- construction truth -------------------------------------------------------------------

def expected_from_truth(spec, truth):
    """Statistics computed from the generator's interval list, never from encoded bytes.
    Valid when nothing is dropped (total <= cap) so every instance survives."""
    R = spec.n_regions
    t = truth[truth["has_end"] == 1]
    d = np.maximum(t["dur"].astype(np.int64) - spec.rec_cost, 0)
    hist = np.zeros((R, 64), dtype=np.uint64)
    bins = np.where(d < 2, 0, np.floor(np.log2(np.maximum(d, 1))).astype(np.int64))
    np.add.at(hist, (t["region"], bins), 1)
    per_sum = np.zeros((spec.n_wg, spec.waves, R), dtype=np.uint64)
    per_n = np.zeros((spec.n_wg, spec.waves, R), dtype=np.uint64)
    np.add.at(per_sum, (t["wg"], t["wave"], t["region"]), d.astype(np.uint64))
    np.add.at(per_n, (t["wg"], t["wave"], t["region"]), 1)
    return dict(n_pairs=len(t), n_orphan_start=int((truth["has_end"] == 0).sum()), hist=hist,
                per_sum=per_sum, per_n=per_n)


@pytest.mark.parametrize("which", ["small_gemm_shape", "decode_scaled"])
def test_construction_truth(oracle_mod, which):
    if which == "small_gemm_shape":
        spec = inputs.spec_small_gemm_shape()
    else:
        spec = inputs.spec_decode_standalone(17)
    raw, truth = inputs.gen_trace(spec, want_truth=True)
    st = oracle_mod.decode(raw, n_threads=4)
    ex = expected_from_truth(spec, truth)
    assert st["n_pairs"] == ex["n_pairs"]
    assert st["n_orphan_start"] == ex["n_orphan_start"] and st["n_orphan_end"] == 0
    assert st["n_dropped"] == 0 and st["n_invalid"] == 0
    assert np.array_equal(st["hist"], ex["hist"])
    assert np.array_equal(st["per"]["sum"], ex["per_sum"])
    assert np.array_equal(st["per"]["n"].astype(np.uint64), ex["per_n"])
    if which == "small_gemm_shape":
        assert st["n_pairs"] == 64 * 4 * 3 * 8 and st["n_slots_valid"] == 12288 and st["n_disorder"] == 0
    else:
        assert st["n_disorder"] > 0  # ~0.1 % displaced slots, all put back by seq
        frac = ex["n_orphan_start"] / st["n_slots_valid"]
        assert 0.005 < frac < 0.02


def test_wrap_copy_drop_counts(oracle_mod):
    spec = inputs.spec_decode_standalone(16, wrap=True)
    raw, truth = inputs.gen_trace(spec, want_truth=True)
    st = oracle_mod.decode(raw, n_threads=4)
    assert st["n_dropped"] == spec.n_wg * spec.waves * 2 * spec.cap_wave
    # survivors are the records with seq >= 2*cap; an instance survives whole iff its START does
    first = 2 * spec.cap_wave
    ended = truth[truth["has_end"] == 1]
    assert st["n_pairs"] == int((ended["seq_start"] >= first).sum())
    assert st["n_orphan_end"] == int((ended["seq_start"] == first - 1).sum())


# ---- invariants and metamorphic relations -------------------------------------------------

def check_invariants(st):
    assert np.array_equal(st["hist"].sum(axis=1), st["cnt"])
    assert int(st["cnt"].sum()) == st["n_pairs"]
    assert st["n_slots_valid"] == 2 * st["n_pairs"] + st["n_orphan_start"] + st["n_orphan_end"] + st["n_invalid"]
    O, U = st["O"].astype(object), st["U"].astype(object)
    assert np.array_equal(st["O"], st["O"].T)
    assert np.array_equal(np.diag(st["O"]), st["U"])
    R = len(U)
    for a in range(R):
        for b in range(R):
            assert O[a, b] <= min(U[a], U[b])
    assert np.array_equal(st["per"]["sum"].sum(axis=(0, 1)), st["sum"])
    assert np.array_equal(st["per"]["n"].astype(np.uint64).sum(axis=(0, 1)), st["cnt"])
    if st["per"].size:
        assert np.array_equal(st["per"]["max"].max(axis=(0, 1)).astype(np.uint64), st["max"])


@pytest.mark.parametrize("seed", range(6))
def test_invariants(oracle_mod, seed):
    if seed < 3:
        raw = inputs.messy_trace(100 + seed, n_wg=8, waves=4, n_regions=6, cap_wave=64)
    else:
        raw, _ = inputs.gen_trace(inputs.spec_decode_standalone(15, seed=seed, wrap=(seed == 5)))
    check_invariants(oracle_mod.decode(raw, n_threads=2))


def _records_view(raw):
    n_wg = int(raw[2])
    return raw[(64 + 128 * n_wg) // 4:].reshape(-1, 2)


def test_doubling_time_shifts_bins_and_doubles_overlap(oracle_mod):
    spec = inputs.TraceSpec(n_wg=4, waves=4, n_regions=5, cap_wave=64, total_per_wave=64, seed=9,
                            dist="lognormal", p0=4.0, p1=1.0, p_orphan=0.05)
    raw, _ = inputs.gen_trace(spec)
    a = oracle_mod.decode(raw)
    raw2 = raw.copy()
    _records_view(raw2)[:, 1] *= 2
    for wg in range(spec.n_wg):  # keep span >= last timestamp
        h = (64 + 128 * wg) // 4
        raw2[h + 4] = raw2[h + 2] + 2 * (raw[h + 4] - raw[h + 2])
    b = oracle_mod.decode(raw2)
    assert np.array_equal(b["hist"][:, 1:], a["hist"][:, :-1]) and not b["hist"][:, 0].any()
    assert np.array_equal(b["U"], 2 * a["U"]) and np.array_equal(b["O"], 2 * a["O"])
    assert np.array_equal(b["F"], a["F"])


def test_constant_clock_offset_changes_nothing(oracle_mod):
    spec = inputs.TraceSpec(n_wg=3, waves=2, n_regions=3, cap_wave=32, total_per_wave=40, seed=3,
                            dist="exp", p0=30.0, p_orphan=0.1)
    raw, _ = inputs.gen_trace(spec)
    a = oracle_mod.decode_bytes(raw)
    raw2 = raw.copy()
    _records_view(raw2)[:, 1] += 12345
    for wg in range(spec.n_wg):
        raw2[(64 + 128 * wg) // 4 + 4] += 12345
    b = oracle_mod.decode_bytes(raw2)
    assert np.array_equal(a, b)


def test_slot_permutation_only_changes_disorder(oracle_mod):
    spec = inputs.TraceSpec(n_wg=2, waves=2, n_regions=3, cap_wave=32, total_per_wave=32, seed=5,
                            dist="exp", p0=30.0)
    raw, _ = inputs.gen_trace(spec)
    a = oracle_mod.decode(raw)
    raw2 = raw.copy()
    recs = _records_view(raw2).reshape(spec.n_wg * spec.waves, spec.cap_wave, 2)
    rng = np.random.default_rng(0)
    for i in range(recs.shape[0]):
        recs[i] = recs[i][rng.permutation(spec.cap_wave)]
    b = oracle_mod.decode(raw2)
    assert b["n_disorder"] > 0 and a["n_disorder"] == 0
    for k in ("hist", "cnt", "sum", "min", "max", "U", "O", "F", "per"):
        assert np.array_equal(a[k], b[k]), k


def test_thread_count_does_not_change_the_result(oracle_mod):
    raw, _ = inputs.gen_trace(inputs.spec_decode_standalone(16))
    assert np.array_equal(oracle_mod.decode_bytes(raw, 1), oracle_mod.decode_bytes(raw, 5))


# ---- the format's own limits: up to 128 regions, long rings ------------------------------------

@pytest.mark.parametrize("R,cap,waves", [(33, 16, 2), (64, 8, 3), (128, 16, 2), (100, 64, 1), (127, 4, 16)])
def test_many_regions_against_brute_force(oracle_mod, R, cap, waves):
    """The tag names up to 128 regions (7 bits): the same brute force, with region numbers that use the
    whole field."""
    for k in range(2):
        raw = inputs.messy_trace(7 * R + cap + k, n_wg=3, waves=waves, n_regions=R, cap_wave=cap,
                                 p_bad=0.03 * k, allow_nonmono=False, flush=bool(k))
        assert_same(brute_decode(raw), oracle_mod.decode(raw))


@pytest.mark.parametrize("seed", range(3))
def test_long_rings_against_brute_force(oracle_mod, seed):
    """Rings of 1024 and 4096 records per wave, wrapped, with swapped slots and orphans."""
    spec = inputs.TraceSpec(n_wg=2, waves=2 + seed, n_regions=[3, 40, 6][seed], cap_wave=[1024, 1024, 4096][seed],
                            total_per_wave=[1500, 1024, 5000][seed], total_var=100, seed=50 + seed, dist="exp", p0=6.0,
                            gap_max=4, phase_max=30, p_orphan=0.05, p_swap=0.01, swap_max=7, rec_cost=1)
    raw, _ = inputs.gen_trace(spec)
    assert_same(brute_decode(raw), oracle_mod.decode(raw))

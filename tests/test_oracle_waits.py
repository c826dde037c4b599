"""Pins for the CPU wait-replay oracle oracle/ref_waits.c (no GPU).

It is checked against something other than itself: the START / END / START placement of the paper's
asynchronous-instruction replay worked by hand (Sec. 4.3: T_wait = CLK2 - CLK1, the record cost
cancels; the condition that the wait must outlast one record), the circular-buffer tail rule
(Sec. 4.2), an independently written Python routine, traces built from known gaps, and a telescoping
identity against the statistics decoder (an independent routine of the oracle package): in a wave
whose regions follow one another without nesting, the raw durations and the waits add up to the
distance between the first START and the last END.
"""
import numpy as np
import pytest

import inputs
from inputs import PHASE_END as E
from inputs import PHASE_START as S
from tests.brute import assert_waits_same, brute_waits, waits_summary


def one_wg(oracle_mod, wave_events, n_regions, cap_wave=16, rec_cost=0, flush=False, **kw):
    wg = inputs.events_to_wg(wave_events, cap_wave, flush=flush, **kw)
    raw = inputs.encode_trace([wg], len(wave_events), n_regions, cap_wave, rec_cost=rec_cost, flush=flush)
    return raw, oracle_mod.waits(raw)


def per_tuple(v, wg, w, a):
    p = v["per"][wg, w, a]
    return int(p["sum"]), int(p["n"]), int(p["max"])


# ---- the paper's placement, by hand ---------------------------------------------------------------

def test_start_end_start_placement(oracle_mod):
    # CLK0 = 100 (START before the launch), CLK1 = 400 (END before the barrier), CLK2 = 1000
    _, v = one_wg(oracle_mod, [[(S, 0, 100), (E, 0, 400), (S, 1, 1000), (E, 1, 1100)]], 2)
    assert (v["n_waits"], v["n_uncovered"], v["n_async"]) == (1, 0, 1)
    assert list(v["cnt"]) == [1, 0] and list(v["sum"]) == [600, 0]
    assert list(v["min"]) == [600, 2 ** 64 - 1] and list(v["max"]) == [600, 0]
    assert list(v["async_cnt"]) == [1, 0] and list(v["async_sum"]) == [900, 0]
    assert per_tuple(v, 0, 0, 0) == (600, 1, 600) and per_tuple(v, 0, 0, 1) == (0, 0, 0)
    assert v["hist"][0, 9] == 1 and v["hist"].sum() == 1   # 512 <= 600 < 1024


def test_record_cost_cancels_in_the_wait_but_not_in_the_whole(oracle_mod):
    # T_wait = (CLK2 - T_a) - (CLK1 - T_a): no cost is taken off; the whole interval holds one record
    _, v = one_wg(oracle_mod, [[(S, 0, 100), (E, 0, 400), (S, 1, 1000)]], 2, rec_cost=25)
    assert list(v["sum"]) == [600, 0] and list(v["async_sum"]) == [875, 0] and v["n_uncovered"] == 0


def test_wait_must_outlast_one_record(oracle_mod):
    ev = [(S, 0, 0), (E, 0, 100), (S, 0, 124), (E, 0, 200), (S, 0, 225), (E, 0, 300), (S, 0, 326), (E, 0, 400)]
    _, v = one_wg(oracle_mod, [ev], 1, rec_cost=25)
    # gaps 24, 25, 26 against a cost of 25: the first two are not covered
    assert v["n_waits"] == 3 and v["n_uncovered"] == 2 and list(v["uncovered"]) == [2]
    assert list(v["sum"]) == [75] and list(v["min"]) == [24] and list(v["max"]) == [26]
    # whole intervals 124 - 0, 225 - 124, 326 - 225, each minus 25
    assert list(v["async_sum"]) == [99 + 76 + 76]


def test_only_end_then_start_is_a_wait(oracle_mod):
    # START START, END END and a trailing END give nothing; an END whose START is missing still waits
    ev = [(S, 0, 10), (S, 1, 20), (E, 1, 30), (E, 0, 40), (E, 2, 50), (S, 1, 65), (E, 1, 70)]
    _, v = one_wg(oracle_mod, [ev], 3)
    assert v["n_waits"] == 1 and v["n_async"] == 0
    assert list(v["cnt"]) == [0, 0, 1] and list(v["sum"]) == [0, 0, 15]


def test_wait_belongs_to_the_region_of_the_end(oracle_mod):
    ev = [(S, 3, 0), (E, 3, 10), (S, 1, 17), (E, 1, 20), (S, 3, 28)]
    _, v = one_wg(oracle_mod, [ev], 4)
    assert list(v["cnt"]) == [0, 1, 0, 1] and list(v["sum"]) == [0, 8, 0, 7]
    assert list(v["async_sum"]) == [0, 11, 0, 17]


def test_nested_end_pairs_with_its_own_start(oracle_mod):
    # the inner region ends, then the outer one: only the outer END is followed by a START
    ev = [(S, 0, 0), (S, 1, 5), (E, 1, 50), (E, 0, 60), (S, 2, 100)]
    _, v = one_wg(oracle_mod, [ev], 3)
    assert list(v["cnt"]) == [1, 0, 0] and list(v["sum"]) == [40, 0, 0] and list(v["async_sum"]) == [100, 0, 0]


def test_waves_are_independent(oracle_mod):
    _, v = one_wg(oracle_mod, [[(S, 0, 0), (E, 0, 10), (S, 0, 13)], [(S, 0, 1), (E, 0, 20), (S, 0, 50)]], 1)
    assert per_tuple(v, 0, 0, 0) == (3, 1, 3) and per_tuple(v, 0, 1, 0) == (30, 1, 30)
    assert list(v["min"]) == [3] and list(v["max"]) == [30] and list(v["sum"]) == [33]


def test_histogram_bins(oracle_mod):
    gaps = [0, 1, 2, 3, 4, 1023, 1024]
    ev, t = [], 0
    for g in gaps:
        ev += [(S, 0, t), (E, 0, t + 5)]
        t += 5 + g
    ev.append((S, 0, t))
    _, v = one_wg(oracle_mod, [ev], 1, cap_wave=32)
    want = np.zeros(64, dtype=np.uint64)
    for b in (0, 0, 1, 1, 2, 9, 10):
        want[b] += 1
    assert np.array_equal(v["hist"][0], want)


def test_clock_wrap_inside_the_wait(oracle_mod):
    _, v = one_wg(oracle_mod, [[(S, 0, 0xFFFFFF00), (E, 0, 0xFFFFFFF0), (S, 0, 0x10)]], 1, t_end=1000 + (1 << 33))
    assert list(v["sum"]) == [0x20] and list(v["async_sum"]) == [0x110]


def test_circular_buffer_keeps_tail(oracle_mod):
    ev = [(S, 0, 0), (E, 0, 5), (S, 0, 8), (E, 0, 16), (S, 0, 20), (E, 0, 21)]
    # 6 records into 4 slots: S8 E16 S20 E21 survive -> one wait of 4, END paired with S8
    _, v = one_wg(oracle_mod, [ev], 1, cap_wave=4)
    assert list(v["sum"]) == [4] and list(v["cnt"]) == [1] and list(v["async_sum"]) == [12]
    # 5 records into 4 slots: E5 S8 E16 S20 -> waits 3 and 4; the first END has lost its START
    _, v = one_wg(oracle_mod, [ev[:5]], 1, cap_wave=4)
    assert list(v["sum"]) == [7] and list(v["cnt"]) == [2] and list(v["async_cnt"]) == [1]
    # the flush strategy keeps the head instead: S0 E5 S8 E16
    _, v = one_wg(oracle_mod, [ev], 1, cap_wave=4, flush=True)
    assert list(v["sum"]) == [3] and list(v["cnt"]) == [1] and list(v["async_sum"]) == [8]


def test_empty_trace(oracle_mod):
    raw = inputs.encode_trace([], 2, 3, 8)
    v = oracle_mod.waits(raw)
    assert v["n_waits"] == 0 and v["per"].size == 0 and list(v["min"]) == [2 ** 64 - 1] * 3
    _, v = one_wg(oracle_mod, [[], []], 3)
    assert v["n_waits"] == 0 and v["hist"].sum() == 0


def test_header_echo(oracle_mod):
    _, v = one_wg(oracle_mod, [[(S, 0, 1)], [], []], 5, cap_wave=8, rec_cost=17)
    assert (v["n_wg"], v["waves"], v["n_regions"], v["cap_wave"], v["rec_cost"]) == (1, 3, 5, 8, 17)


# ---- independent routine, construction truth, statistics decoder ---------------------------------------

@pytest.mark.parametrize("seed", range(8))
def test_against_independent_python_routine(oracle_mod, seed):
    raw = inputs.messy_trace(700 + seed, n_wg=4, waves=1 + seed % 4, n_regions=1 + seed % 5, cap_wave=16,
                             flush=bool(seed & 1))
    raw[6] = [0, 3, 40][seed % 3]  # record cost
    assert_waits_same(waits_summary(raw, brute_waits(raw)), oracle_mod.waits(raw))


def test_generated_trace_against_independent_python_routine(oracle_mod):
    spec = inputs.TraceSpec(n_wg=5, waves=3, n_regions=4, cap_wave=64, total_per_wave=90, total_var=20, seed=5,
                            p_orphan=0.05, p_swap=0.01)
    raw, _ = inputs.gen_trace(spec)
    raw[6] = 11
    assert_waits_same(waits_summary(raw, brute_waits(raw)), oracle_mod.waits(raw))


@pytest.mark.parametrize("seed", range(4))
def test_traces_built_from_known_gaps(oracle_mod, seed):
    """Every wave runs region after region with drawn execution times and gaps; the sums are known."""
    rng = np.random.default_rng(seed)
    R, W, n_it, cost = 3, 2, 20, 9
    waves, want_sum, want_cnt, want_unc, want_async = [], np.zeros(R, int), np.zeros(R, int), np.zeros(R, int), np.zeros(R, int)
    for _w in range(W):
        t, ev = int(rng.integers(0, 50)), []
        for i in range(n_it):
            a = int(rng.integers(0, R))
            exe, gap = int(rng.integers(1, 400)), int(rng.integers(0, 30))
            ev += [(S, a, t), (E, a, t + exe)]
            if i + 1 < n_it:  # the last END has no successor
                want_sum[a] += gap
                want_cnt[a] += 1
                want_unc[a] += gap <= cost
                want_async[a] += max(exe + gap - cost, 0)
            t += exe + gap
        waves.append(ev)
    _, v = one_wg(oracle_mod, waves, R, cap_wave=64, rec_cost=cost, t_end=1000 + 40000)
    assert list(v["sum"]) == list(want_sum) and list(v["cnt"]) == list(want_cnt)
    assert list(v["uncovered"]) == list(want_unc) and list(v["async_sum"]) == list(want_async)
    assert list(v["async_cnt"]) == list(want_cnt)


@pytest.mark.parametrize("seed", range(3))
def test_durations_and_waits_telescope(oracle_mod, seed):
    """Regions in sequence, no nesting, no cost: sum of durations + sum of waits = last END - first START."""
    rng = np.random.default_rng(100 + seed)
    R, W = 4, 3
    waves, span = [], 0
    for _w in range(W):
        t0 = t = int(rng.integers(0, 100))
        ev = []
        for _ in range(25):
            a = int(rng.integers(0, R))
            exe, gap = int(rng.integers(1, 1000)), int(rng.integers(0, 200))
            ev += [(S, a, t), (E, a, t + exe)]
            last_end = t + exe
            t += exe + gap
        span += last_end - t0
        waves.append(ev)
    wg = inputs.events_to_wg(waves, 64, t_end=1000 + 100000)
    raw = inputs.encode_trace([wg], W, R, 64)
    stats, v = oracle_mod.decode(raw), oracle_mod.waits(raw)
    assert int(stats["sum"].sum()) + int(v["sum"].sum()) == span
    assert stats["n_pairs"] == v["n_waits"] + W == v["n_async"] + W

"""Pins for the CPU timeline oracle oracle/ref_pairs.c (no GPU).

It is checked against something other than itself: hand-worked traces for the three record
patterns the paper names (Sec. 4.2 "SM-level Data Layout": common, nested, multi-iteration), the
circular-buffer tail rule (Sec. 4.2), the constant record cost of the replay (Sec. 4.3), an
independently written Python routine, the generator's construction truth, and the statistics
decoder (an independent routine of the oracle package): the rows of every (workgroup, wave, region)
must add up to that decoder's sum / count / maximum and reproduce its histogram.
"""
import numpy as np
import pytest

import inputs
from inputs import PHASE_END as E
from inputs import PHASE_START as S
from tests.brute import brute_pairs


def rows_of(oracle_mod, raw):
    count, rows = oracle_mod.pairs(raw)
    return {(wg, w): [tuple(int(x) for x in r) for r in rows[wg, w, : count[wg, w]]]
            for wg in range(count.shape[0]) for w in range(count.shape[1])}


def one_wg(oracle_mod, wave_events, n_regions, cap_wave=16, rec_cost=0, flush=False, **kw):
    wg = inputs.events_to_wg(wave_events, cap_wave, flush=flush, **kw)
    raw = inputs.encode_trace([wg], len(wave_events), n_regions, cap_wave, rec_cost=rec_cost, flush=flush)
    return raw, rows_of(oracle_mod, raw)


# ---- hand-worked patterns: rows are (start, dur, iter, region) ---------------------------------

def test_common_pattern(oracle_mod):
    _, rows = one_wg(oracle_mod, [[(S, 0, 10), (E, 0, 30), (S, 1, 40), (E, 1, 100)]], 2)
    assert rows[(0, 0)] == [(10, 20, 0, 0), (40, 60, 0, 1)]


def test_nested_pattern_lists_rows_in_end_order(oracle_mod):
    _, rows = one_wg(oracle_mod, [[(S, 0, 10), (S, 1, 20), (E, 1, 50), (E, 0, 90)]], 2)
    assert rows[(0, 0)] == [(20, 30, 0, 1), (10, 80, 0, 0)]


def test_multi_iteration_pattern_numbers_the_iterations(oracle_mod):
    ev = [(S, 0, 0), (E, 0, 5), (S, 1, 6), (E, 1, 7), (S, 0, 8), (E, 0, 16), (S, 0, 20), (E, 0, 21)]
    _, rows = one_wg(oracle_mod, [ev], 2)
    assert rows[(0, 0)] == [(0, 5, 0, 0), (6, 1, 0, 1), (8, 8, 1, 0), (20, 1, 2, 0)]


def test_waves_are_independent(oracle_mod):
    _, rows = one_wg(oracle_mod, [[(S, 0, 0), (E, 0, 10)], [(S, 1, 5), (S, 0, 12), (E, 1, 15), (E, 0, 20)]], 2)
    assert rows[(0, 0)] == [(0, 10, 0, 0)]
    assert rows[(0, 1)] == [(5, 10, 0, 1), (12, 8, 0, 0)]


def test_orphans_give_no_row_and_do_not_count_as_iterations(oracle_mod):
    # START START END: the inner START pairs; END END: the second END is an orphan
    ev = [(S, 0, 1), (S, 0, 4), (E, 0, 9), (E, 0, 12), (S, 0, 20), (E, 0, 26)]
    _, rows = one_wg(oracle_mod, [ev], 1)
    assert rows[(0, 0)] == [(4, 5, 0, 0), (20, 6, 1, 0)]


def test_circular_buffer_keeps_tail(oracle_mod):
    ev = [(S, 0, 0), (E, 0, 5), (S, 0, 8), (E, 0, 16), (S, 0, 20), (E, 0, 21)]
    # 6 records into 4 slots: the survivors are S8 E16 S20 E21; the first surviving pair is iteration 0
    _, rows = one_wg(oracle_mod, [ev], 1, cap_wave=4)
    assert rows[(0, 0)] == [(8, 8, 0, 0), (20, 1, 1, 0)]
    # 5 records into 4 slots: E5 S8 E16 S20 survive; the END whose START was overwritten gives no row,
    # and neither does the START that is still open at the end
    _, rows = one_wg(oracle_mod, [ev[:5]], 1, cap_wave=4)
    assert rows[(0, 0)] == [(8, 8, 0, 0)]


def test_flush_strategy_keeps_head(oracle_mod):
    ev = [(S, 0, 0), (E, 0, 5), (S, 0, 8), (E, 0, 16), (S, 0, 20), (E, 0, 21)]
    _, rows = one_wg(oracle_mod, [ev], 1, cap_wave=4, flush=True)
    assert rows[(0, 0)] == [(0, 5, 0, 0), (8, 8, 1, 0)]


def test_record_cost_is_subtracted_saturating(oracle_mod):
    _, rows = one_wg(oracle_mod, [[(S, 0, 10), (E, 0, 30), (S, 0, 40), (E, 0, 43)]], 1, rec_cost=5)
    assert rows[(0, 0)] == [(10, 15, 0, 0), (40, 0, 1, 0)]


def test_clock_wrap_inside_interval(oracle_mod):
    _, rows = one_wg(oracle_mod, [[(S, 0, 0xFFFFFFF0), (E, 0, 0x10)]], 1, t_end=1000 + (1 << 33))
    assert rows[(0, 0)] == [(0xFFFFFFF0, 0x20, 0, 0)]


def test_empty_trace(oracle_mod):
    raw = inputs.encode_trace([], 2, 3, 8)
    count, rows = oracle_mod.pairs(raw)
    assert count.size == 0 and rows.size == 0
    _, rows = one_wg(oracle_mod, [[], []], 3)
    assert rows == {(0, 0): [], (0, 1): []}


def test_rows_past_the_count_are_untouched(oracle_mod):
    raw, _ = one_wg(oracle_mod, [[(S, 0, 10), (E, 0, 30)]], 1, cap_wave=8)
    buf = oracle_mod.pairs_raw(raw, fill=0xA5)
    count, rows = oracle_mod.view_pairs(buf, 1, 1, 8)
    assert count[0, 0] == 1
    assert rows[0, 0, 1:].tobytes() == b"\xA5" * (3 * 16)


# ---- independent routine, construction truth, statistics decoder ---------------------------------

@pytest.mark.parametrize("seed", range(6))
def test_against_independent_python_routine(oracle_mod, seed):
    raw = inputs.messy_trace(300 + seed, n_wg=4, waves=1 + seed % 4, n_regions=1 + seed % 5, cap_wave=16,
                             flush=bool(seed & 1))
    assert rows_of(oracle_mod, raw) == brute_pairs(raw)


@pytest.mark.parametrize("which", ["small", "wrap", "orphans"])
def test_construction_truth(oracle_mod, which):
    if which == "small":
        spec = inputs.spec_small_gemm_shape()
    elif which == "wrap":
        spec = inputs.TraceSpec(n_wg=5, waves=3, n_regions=4, cap_wave=32, total_per_wave=70, seed=21,
                                dist="exp", p0=50.0, p_swap=0.02)
    else:
        spec = inputs.TraceSpec(n_wg=4, waves=4, n_regions=5, cap_wave=64, total_per_wave=64, seed=22,
                                p_orphan=0.2, p_swap=0.01)
    raw, truth = inputs.gen_trace(spec, want_truth=True)
    got = rows_of(oracle_mod, raw)
    T, cap = spec.total_per_wave, spec.cap_wave
    first = max(0, T - cap)
    for wg in range(spec.n_wg):
        for w in range(spec.waves):
            inst = truth[(truth["wg"] == wg) & (truth["wave"] == w)]
            # an instance survives as a pair when its START and its END (the next record) both survive
            exp, it = [], {}
            for t in inst[np.argsort(inst["seq_start"])]:
                if not t["has_end"] or int(t["seq_start"]) < first:
                    continue
                r = int(t["region"])
                exp.append((int(t["ts_start"]), int(t["dur"]), it.get(r, 0), r))
                it[r] = it.get(r, 0) + 1
            assert got[(wg, w)] == exp, (wg, w)


@pytest.mark.parametrize("seed", range(4))
def test_rows_add_up_to_the_statistics_decoder(oracle_mod, seed):
    raw = inputs.messy_trace(400 + seed, n_wg=6, waves=4, n_regions=6, cap_wave=64)
    st = oracle_mod.decode(raw)
    count, rows = oracle_mod.pairs(raw)
    n_wg, W, R = 6, 4, 6
    assert int(count.sum()) == st["n_pairs"]
    hist = np.zeros((R, 64), dtype=np.uint64)
    for wg in range(n_wg):
        for w in range(W):
            rr = rows[wg, w, : count[wg, w]]
            for r in range(R):
                d = rr["dur"][rr["region"] == r].astype(np.uint64)
                p = st["per"][wg, w, r]
                assert (int(d.sum()), d.size, int(d.max()) if d.size else 0) == (int(p["sum"]), int(p["n"]), int(p["max"]))
                assert rr["iter"][rr["region"] == r].tolist() == list(range(d.size))
                for x in d:
                    hist[r, 0 if x < 2 else int(x).bit_length() - 1] += np.uint64(1)
    assert np.array_equal(hist, st["hist"])


def test_bad_header_is_rejected(oracle_mod):
    raw = inputs.encode_trace([inputs.events_to_wg([[(S, 0, 1), (E, 0, 2)]], 8)], 1, 1, 8)
    bad = raw.copy(); bad[0] ^= 1
    with pytest.raises(ValueError):
        oracle_mod.pairs(bad)

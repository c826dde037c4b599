"""Pins for the CPU stage-table oracle oracle/ref_stages.c and the overlap models (no GPU).

The table is checked against something other than itself: hand-worked traces, an independently
written Python routine that starts from the raw trace, a numpy group-by over the timeline rows, and
its defining properties (every row lands in exactly one entry or is counted as clipped).  The
models of Table 4 are checked on numbers worked by hand on both sides of the discriminant.
"""
import numpy as np
import pytest

import inputs
from inputs import PHASE_END as E
from inputs import PHASE_START as S
from tests.brute import brute_stages


def table_of(oracle_mod, wave_events, n_regions, max_iter, cap_wave=32, rec_cost=0, **kw):
    wg = inputs.events_to_wg(wave_events, cap_wave, **kw)
    raw = inputs.encode_trace([wg], len(wave_events), n_regions, cap_wave, rec_cost=rec_cost)
    hdr, tab = oracle_mod.stages(raw, max_iter)
    return raw, hdr, tab


def entry(tab, wg, r, it):
    e = tab[wg, r, it]
    return int(e["max_dur"]), int(e["min_start"]), int(e["max_end"]), int(e["n_waves"])


EMPTY = (0, 0xFFFFFFFF, 0, 0)


def test_slowest_wave_sets_the_stage_latency(oracle_mod):
    # two waves run load (region 0) then compute (region 1), two iterations each
    w0 = [(S, 0, 0), (E, 0, 10), (S, 1, 10), (E, 1, 50), (S, 0, 50), (E, 0, 58), (S, 1, 60), (E, 1, 95)]
    w1 = [(S, 0, 2), (E, 0, 20), (S, 1, 21), (E, 1, 40), (S, 0, 41), (E, 0, 45), (S, 1, 47), (E, 1, 99)]
    _, hdr, tab = table_of(oracle_mod, [w0, w1], 2, 4)
    assert hdr == {"n_rows": 8, "n_clipped": 0, "n_bad_region": 0}
    assert entry(tab, 0, 0, 0) == (18, 0, 20, 2)    # load, iteration 0: 10 vs 18 ticks
    assert entry(tab, 0, 1, 0) == (40, 10, 50, 2)   # compute, iteration 0: 40 vs 19
    assert entry(tab, 0, 0, 1) == (8, 41, 58, 2)
    assert entry(tab, 0, 1, 1) == (52, 47, 99, 2)
    assert entry(tab, 0, 0, 2) == EMPTY and entry(tab, 0, 1, 3) == EMPTY


def test_waves_with_different_trip_counts(oracle_mod):
    w0 = [(S, 0, 0), (E, 0, 5), (S, 0, 10), (E, 0, 17), (S, 0, 20), (E, 0, 29)]
    w1 = [(S, 0, 1), (E, 0, 4)]
    _, hdr, tab = table_of(oracle_mod, [w0, w1, []], 1, 3)
    assert [entry(tab, 0, 0, i) for i in range(3)] == [(5, 0, 5, 2), (7, 10, 17, 1), (9, 20, 29, 1)]
    assert hdr["n_rows"] == 4


def test_iterations_past_the_limit_are_counted_not_stored(oracle_mod):
    ev = []
    for i in range(6):
        ev += [(S, 0, 10 * i), (E, 0, 10 * i + 3 + i)]
    _, hdr, tab = table_of(oracle_mod, [ev], 1, 4)
    assert hdr == {"n_rows": 4, "n_clipped": 2, "n_bad_region": 0}
    assert [entry(tab, 0, 0, i)[0] for i in range(4)] == [3, 4, 5, 6]


def test_record_cost_shortens_latency_and_end(oracle_mod):
    _, _, tab = table_of(oracle_mod, [[(S, 0, 100), (E, 0, 160)], [(S, 0, 90), (E, 0, 95)]], 1, 1, rec_cost=10)
    # durations 50 and 0 (5 - 10 saturates); ends 150 and 90
    assert entry(tab, 0, 0, 0) == (50, 90, 150, 2)


def test_end_wraps_modulo_2_32(oracle_mod):
    _, _, tab = table_of(oracle_mod, [[(S, 0, 0xFFFFFFF0), (E, 0, 0x10)]], 1, 1, t_end=1000 + (1 << 33))
    assert entry(tab, 0, 0, 0) == (0x20, 0xFFFFFFF0, 0x10, 1)


def test_bad_region_rows_are_dropped(oracle_mod):
    # a timeline block written by hand: one good row, one with a region the table does not have
    blk = np.zeros(16 + 2 * 16, dtype=np.uint8)
    blk[:4].view("<u4")[0] = 2
    blk[16:].view("<u4")[:] = [5, 7, 0, 1, 9, 9, 0, 3]
    hdr, tab = oracle_mod.view_stages(oracle_mod.stages_raw(blk, 1, 1, 4, 2, 2), 1, 2, 2)
    assert hdr == {"n_rows": 1, "n_clipped": 0, "n_bad_region": 1}
    assert entry(tab, 0, 1, 0) == (7, 5, 12, 1) and entry(tab, 0, 0, 0) == EMPTY


def test_empty(oracle_mod):
    raw = inputs.encode_trace([], 2, 3, 8)
    hdr, tab = oracle_mod.stages(raw, 5)
    assert hdr["n_rows"] == 0 and tab.size == 0


@pytest.mark.parametrize("seed", range(6))
def test_against_independent_python_routine(oracle_mod, seed):
    raw = inputs.messy_trace(900 + seed, n_wg=4, waves=1 + seed % 4, n_regions=1 + seed % 5, cap_wave=32,
                             flush=bool(seed & 1))
    raw[6] = [0, 4][seed % 2]
    max_iter = [1, 3, 16][seed % 3]
    n_wg, _W, R = (int(x) for x in raw[2:5])
    hdr, tab = oracle_mod.stages(raw, max_iter)
    n_rows, n_clipped, want = brute_stages(raw, max_iter)
    assert (hdr["n_rows"], hdr["n_clipped"], hdr["n_bad_region"]) == (n_rows, n_clipped, 0)
    for wg in range(n_wg):
        for r in range(R):
            for it in range(max_iter):
                assert entry(tab, wg, r, it) == want.get((wg, r, it), EMPTY), (wg, r, it)


def test_numpy_group_by_over_the_timeline_rows(oracle_mod):
    spec = inputs.TraceSpec(n_wg=6, waves=4, n_regions=5, cap_wave=128, total_per_wave=120, total_var=30, seed=9,
                            p_orphan=0.03, p_swap=0.005)
    raw, _ = inputs.gen_trace(spec)
    max_iter = 8
    hdr, tab = oracle_mod.stages(raw, max_iter)
    count, rows = oracle_mod.pairs(raw)
    used = 0
    for wg in range(6):
        allr = np.concatenate([rows[wg, w, : count[wg, w]] for w in range(4)])
        for r in range(5):
            for it in range(max_iter):
                sel = allr[(allr["region"] == r) & (allr["iter"] == it)]
                used += sel.size
                if sel.size == 0:
                    assert entry(tab, wg, r, it) == EMPTY
                else:
                    end = (sel["start"].astype(np.uint64) + sel["dur"]) % (1 << 32)
                    assert entry(tab, wg, r, it) == (int(sel["dur"].max()), int(sel["start"].min()), int(end.max()), sel.size)
    assert hdr["n_rows"] == used and hdr["n_rows"] + hdr["n_clipped"] == int(count.sum())
    assert int(tab["n_waves"].sum()) == used


# ---- overlap models (Table 4) ------------------------------------------------------------------------

def test_swp_model_both_sides_of_the_discriminant():
    from paper_2505_21661_amd import model

    t_load, t_comp = [300.0, 500.0], [100.0, 150.0]
    # one warp group, two pipeline stages: 1*2*250 - max(400, 650) = -150 < 0 -> loading dominates
    assert model.swp_discriminant(t_load, t_comp, n_wg=1, n_pipe=2) == -150.0
    assert model.swp_latency(t_load, t_comp, n_loop=64, n_pipe=2, n_wg=1) == 650.0 * 64 / 2
    # two warp groups: 2*2*250 - 650 = 350 >= 0 -> loads hidden, the computation adds up
    assert model.swp_discriminant(t_load, t_comp, n_wg=2, n_pipe=2) == 350.0
    assert model.swp_latency(t_load, t_comp, n_loop=64, n_pipe=2, n_wg=2) == 250.0 * 64
    # the boundary belongs to the compute-bound side
    assert model.swp_latency([100.0], [100.0], n_loop=10, n_pipe=2, n_wg=1) == 1000.0


def test_ws_compute_and_memory_models():
    from paper_2505_21661_amd import model

    lat = {3: 120.0, 6: 80.0, 12: 400.0, 22: 410.0, 15: 390.0, 25: 395.0, 13: 200.0}
    # Sec. 5.2: the vanilla kernel's critical path holds four GEMM stages and two loads
    assert model.ws_latency(lat, [22, 12, 25, 15, 6, 3]) == 410 + 400 + 395 + 390 + 80 + 120
    assert model.compute_time(2.0 * 4096 ** 3, 1e15) == pytest.approx(1.37438953472e-4)
    assert model.memory_time(1e-6, 64e6, 8e12) == pytest.approx(9e-6)


def test_models_read_the_stage_table(oracle_mod):
    from paper_2505_21661_amd import model

    w0 = [(S, 0, 0), (E, 0, 10), (S, 1, 10), (E, 1, 50), (S, 0, 50), (E, 0, 58), (S, 1, 60), (E, 1, 95)]
    w1 = [(S, 0, 2), (E, 0, 20), (S, 1, 21), (E, 1, 40), (S, 0, 41), (E, 0, 45), (S, 1, 47), (E, 1, 99)]
    _, _, tab = table_of(oracle_mod, [w0, w1], 2, 4)
    assert model.stage_latencies(tab, 0) == [(18 + 8) / 2, (40 + 52) / 2]
    assert model.stage_latencies(tab, 0, n_iter=1) == [18.0, 40.0]
    assert model.critical_stage_per_iteration(tab, 0).tolist() == [1, 1, -1, -1]

"""Pins for the CPU critical-path oracle oracle/ref_critical.c (no GPU).

The chain is checked against something other than itself: schedules worked by hand (a serial loop, a
producer and two consumers in the shape of the paper's attention case study with each of its stages
made the long one in turn), an independently written Python routine (sort and bisect instead of the
oracle's quadratic search), the identity that the stages on a path and the bubbles between them tile
the stretch from the first start to the last end, and an end-to-end run from a raw trace.
"""
import bisect

import numpy as np
import pytest

import inputs
from inputs import PHASE_END as E
from inputs import PHASE_START as S

EMPTY_ENTRY = (0, 0xFFFFFFFF, 0, 0)


def make_table(oracle_mod, n_wg, n_regions, max_iter):
    tab = np.zeros((n_wg, n_regions, max_iter), dtype=oracle_mod.STAGE_DTYPE)
    tab["min_start"] = 0xFFFFFFFF
    return tab


def put(tab, wg, region, it, start, end, lat=None, n_waves=1):
    tab[wg, region, it] = (end - start if lat is None else lat, start, end, n_waves)


def run(oracle_mod, tab):
    n_wg, R, I = tab.shape
    return oracle_mod.view_critical(oracle_mod.critical_raw(oracle_mod.stage_block(tab), n_wg, R, I), n_wg, R)


def path_by_bisect(tab_wg, max_iter):
    """The same reading written differently: stages sorted by (end, index); the stage before X is the
    last one of that order that lies before X and ends by X's start."""
    flat = tab_wg.reshape(-1)
    nodes = sorted((int(e["max_end"]), i) for i, e in enumerate(flat) if e["n_waves"] > 0)
    ends = [n[0] for n in nodes]
    path = []
    k = len(nodes) - 1
    while k >= 0:
        i = nodes[k][1]
        path.append(i)
        c = bisect.bisect_right(ends, int(flat[i]["min_start"]))  # stages that end by this start
        k = min(k, c) - 1
    return path  # last stage first


def check_against_bisect(oracle_mod, tab):
    n_wg, R, I = tab.shape
    hdr, per_region, rows = run(oracle_mod, tab)
    cnt = np.zeros(R, dtype=np.int64)
    lat = np.zeros(R, dtype=np.int64)
    for wg in range(n_wg):
        flat = tab[wg].reshape(-1)
        path = path_by_bisect(tab[wg], I)
        row = rows[wg]
        assert row["n_stages"] == len(path)
        if not path:
            assert (row["last_stage"], row["first_start"], row["last_end"], row["sum_latency"], row["bubbles"]) == (0xFFFFFFFF, 0, 0, 0, 0)
            continue
        assert row["last_stage"] == ((path[0] // I) << 16 | (path[0] % I))
        assert row["last_end"] == flat[path[0]]["max_end"] and row["first_start"] == flat[path[-1]]["min_start"]
        assert row["sum_latency"] == sum(int(flat[i]["max_dur"]) for i in path)
        bubbles = sum(int(flat[a]["min_start"]) - int(flat[b]["max_end"]) for a, b in zip(path[:-1], path[1:]))
        assert row["bubbles"] == bubbles
        # the stages of the path and the bubbles tile [first start, last end)
        extent = sum(int(flat[i]["max_end"]) - int(flat[i]["min_start"]) for i in path)
        assert extent + bubbles == int(row["last_end"]) - int(row["first_start"])
        for i in path:
            cnt[i // I] += 1
            lat[i // I] += int(flat[i]["max_dur"])
    assert per_region[:, 0].tolist() == cnt.tolist() and per_region[:, 1].tolist() == lat.tolist()
    assert hdr["n_path_stages"] == int(cnt.sum()) and hdr["sum_latency"] == int(lat.sum())
    assert hdr["sum_bubbles"] == int(rows["bubbles"].sum()) and hdr["n_paths"] == int((rows["n_stages"] > 0).sum())
    return hdr, per_region, rows


def test_a_serial_loop_is_its_own_critical_path(oracle_mod):
    # one wave: load (region 0) then compute (region 1), three iterations, gaps of 2 and 5 ticks
    tab = make_table(oracle_mod, 1, 2, 4)
    t = 100
    spans = []
    for it in range(3):
        put(tab, 0, 0, it, t, t + 10); t += 10 + 2
        put(tab, 0, 1, it, t, t + 30); t += 30 + 5
    hdr, per_region, rows = run(oracle_mod, tab)
    assert hdr == {"n_wg": 1, "n_regions": 2, "max_iter": 4, "n_paths": 1, "n_path_stages": 6,
                   "sum_latency": 3 * 40, "sum_bubbles": 3 * 2 + 2 * 5}
    assert per_region.tolist() == [[3, 30], [3, 90]]
    r = rows[0]
    assert (r["n_stages"], r["last_stage"], r["first_start"], r["last_end"]) == (6, (1 << 16) | 2, 100, 100 + 3 * 47 - 5)
    assert (r["sum_latency"], r["bubbles"]) == (120, 16)


def fa_like(oracle_mod, t_load, t_gemm0, t_softmax, t_gemm1, iters=4):
    """A producer that loads K and V tiles back to back and a consumer that runs GEMM0, softmax and GEMM1
    on a tile as soon as both the tile and its own previous step are done (Sec. 5.2, Table 3 stages):
    regions 0 load, 1 GEMM0, 2 softmax, 3 GEMM1."""
    tab = make_table(oracle_mod, 1, 4, iters)
    load_done, cons_free = [], 0
    t = 0
    for it in range(iters):
        put(tab, 0, 0, it, t, t + t_load)
        t += t_load
        load_done.append(t)
    for it in range(iters):
        s = max(load_done[it], cons_free)
        put(tab, 0, 1, it, s, s + t_gemm0); s += t_gemm0
        put(tab, 0, 2, it, s, s + t_softmax); s += t_softmax
        put(tab, 0, 3, it, s, s + t_gemm1); s += t_gemm1
        cons_free = s
    return tab


def test_the_long_stage_dominates_the_path(oracle_mod):
    """The paper names three common critical paths of the attention kernel, each dominated by a
    different operation (Sec. 3.3).  With slow loads the path is every load and the last tile's
    compute; with slow compute it is the first load and every compute stage."""
    iters = 4
    # loads dominate: the consumer waits for every tile
    hdr, per_region, rows = check_against_bisect(oracle_mod, fa_like(oracle_mod, 100, 10, 10, 10, iters))
    assert per_region[:, 0].tolist() == [iters, 1, 1, 1] and hdr["sum_bubbles"] == 0
    assert rows[0]["sum_latency"] == iters * 100 + 30 == rows[0]["last_end"] - rows[0]["first_start"]
    # GEMM0 dominates: after the first tile the consumer never waits
    hdr, per_region, rows = check_against_bisect(oracle_mod, fa_like(oracle_mod, 10, 100, 10, 10, iters))
    assert per_region[:, 0].tolist() == [1, iters, iters, iters]
    assert per_region[1, 1] == iters * 100 and per_region[1, 1] > per_region[[0, 2, 3], 1].max()
    # softmax dominates
    hdr, per_region, rows = check_against_bisect(oracle_mod, fa_like(oracle_mod, 10, 10, 100, 10, iters))
    assert per_region[:, 0].tolist() == [1, iters, iters, iters] and per_region[2, 1] == iters * 100
    assert rows[0]["last_end"] == 10 + iters * 120 and rows[0]["bubbles"] == 0


def test_a_stage_waits_for_the_latest_finisher_not_for_its_own_wave(oracle_mod):
    # region 1 starts at 50: region 0 (ends 20) and region 2 (ends 48) both finished before it; it waited for 2
    tab = make_table(oracle_mod, 1, 3, 1)
    put(tab, 0, 0, 0, 0, 20)
    put(tab, 0, 2, 0, 5, 48)
    put(tab, 0, 1, 0, 50, 90)
    hdr, per_region, rows = run(oracle_mod, tab)
    assert per_region[:, 0].tolist() == [0, 1, 1] and rows[0]["bubbles"] == 2 + 0
    assert rows[0]["first_start"] == 5 and rows[0]["last_end"] == 90 and rows[0]["sum_latency"] == 40 + 43


def test_ties_zero_lengths_and_empty_workgroups(oracle_mod):
    tab = make_table(oracle_mod, 3, 2, 3)
    # workgroup 0: nothing.  workgroup 1: stages of length 0 and equal ends
    put(tab, 1, 0, 0, 10, 10)
    put(tab, 1, 0, 1, 10, 10)
    put(tab, 1, 1, 0, 10, 10)
    put(tab, 1, 1, 2, 10, 30)
    put(tab, 1, 0, 2, 12, 30)   # same end as (1, 2): the later index, region 1, is the last stage
    # workgroup 2: a stage whose slowest wave (latency 9) is shorter than its extent over the waves (20)
    put(tab, 2, 0, 0, 0, 20, lat=9, n_waves=4)
    put(tab, 2, 1, 0, 25, 40, lat=15, n_waves=4)
    hdr, per_region, rows = check_against_bisect(oracle_mod, tab)
    assert rows[0]["n_stages"] == 0 and rows[0]["last_stage"] == 0xFFFFFFFF
    # path of workgroup 1: (1,2) <- (1,0) <- (0,1) <- (0,0): the zero-length stages chain up by index
    assert rows[1]["n_stages"] == 4 and rows[1]["last_stage"] == (1 << 16 | 2) and rows[1]["bubbles"] == 0
    assert rows[2]["n_stages"] == 2 and rows[2]["sum_latency"] == 24 and rows[2]["bubbles"] == 5
    assert hdr["n_paths"] == 2


@pytest.mark.parametrize("seed", range(6))
def test_random_tables_against_sort_and_bisect(oracle_mod, seed):
    rng = np.random.default_rng(seed)
    n_wg, R, I = 5, int(rng.integers(1, 7)), int(rng.integers(1, 20))
    tab = make_table(oracle_mod, n_wg, R, I)
    for wg in range(n_wg):
        for r in range(R):
            for it in range(I):
                if rng.random() < 0.2:
                    continue
                start = int(rng.integers(0, 400))
                ext = int(rng.integers(0, 60)) if rng.random() < 0.9 else 0
                put(tab, wg, r, it, start, start + ext, lat=int(rng.integers(0, ext + 1)), n_waves=int(rng.integers(1, 9)))
    check_against_bisect(oracle_mod, tab)


def test_large_clock_values_compare_unsigned(oracle_mod):
    tab = make_table(oracle_mod, 1, 2, 2)
    put(tab, 0, 0, 0, 0x7FFFFFF0, 0x80000010)
    put(tab, 0, 1, 0, 0x80000020, 0xFFFFFFF0)
    hdr, per_region, rows = check_against_bisect(oracle_mod, tab)
    assert rows[0]["n_stages"] == 2 and rows[0]["bubbles"] == 0x10


def test_from_a_raw_trace(oracle_mod):
    """Two waves: wave 0 loads (region 0), wave 1 computes (region 1) on what wave 0 loaded."""
    w0 = [(S, 0, 0), (E, 0, 40), (S, 0, 40), (E, 0, 80), (S, 0, 80), (E, 0, 120)]
    w1 = [(S, 1, 41), (E, 1, 60), (S, 1, 82), (E, 1, 100), (S, 1, 121), (E, 1, 150)]
    wg = inputs.events_to_wg([w0, w1], 16)
    raw = inputs.encode_trace([wg], 2, 2, 16)
    _, tab = oracle_mod.stages(raw, 4)
    hdr, per_region, rows = check_against_bisect(oracle_mod, tab)
    # the three loads and the last compute: the computes of iterations 0 and 1 finish under the next load
    assert per_region.tolist() == [[3, 120], [1, 29]] and rows[0]["bubbles"] == 1
    assert rows[0]["last_stage"] == (1 << 16 | 2) and rows[0]["last_end"] - rows[0]["first_start"] == 150

"""Host-side logic without a GPU: the binding's views of the output blocks (statistics, timeline rows,
waits, stage table).  The CPU oracle writes the same byte layouts (include/kperf.h), so its blocks are
parsed here and checked against values worked out by hand for a small trace."""
import numpy as np

import inputs
import oracle
from paper_2505_21661_amd import binding


def hand_raw():
    # one workgroup of two waves, three regions:
    #   wave 0: region 0 [100, 300), region 1 [300, 900), region 0 [1000, 1100)
    #   wave 1: region 2 [50, 2050)
    S, E = 0, 1
    wg = inputs.events_to_wg([
        [(S, 0, 100), (E, 0, 300), (S, 1, 300), (E, 1, 900), (S, 0, 1000), (E, 0, 1100)],
        [(S, 2, 50), (E, 2, 2050)],
    ], 8)
    return inputs.encode_trace([wg], waves=2, n_regions=3, cap_wave=8)


def test_parse_stats_of_a_hand_built_trace():
    raw = hand_raw()
    st = binding.parse_stats(oracle.decode_bytes(raw, 1))
    assert (st["n_wg"], st["waves_per_wg"], st["n_regions"], st["cap_wave"]) == (1, 2, 3, 8)
    assert st["n_slots_valid"] == 8 and st["n_pairs"] == 4 and st["n_orphan_start"] == 0 and st["n_invalid"] == 0
    assert st["cnt"].tolist() == [2, 1, 1] and st["sum"].tolist() == [300, 600, 2000]
    assert st["min"].tolist() == [100, 600, 2000] and st["max"].tolist() == [200, 600, 2000]
    assert st["per"]["n"].tolist() == [[[2, 1, 0], [0, 0, 1]]]
    assert st["per"]["sum"].tolist() == [[[300, 600, 0], [0, 0, 2000]]]
    assert st["per"]["max"].tolist() == [[[200, 600, 0], [0, 0, 2000]]]
    # region 2 is open over all of regions 0 and 1; those two never overlap
    assert st["U"].tolist() == [300, 600, 2000]
    assert st["O"].tolist() == [[300, 0, 300], [0, 600, 600], [300, 600, 2000]]
    assert st["F"][0, 2] == 1.0 and st["F"][2, 0] == 300 / 2000 and st["F"][0, 1] == 0.0
    # durations 100, 200 -> bins 6, 7; 600 -> bin 9; 2000 -> bin 10
    assert np.flatnonzero(st["hist"][0]).tolist() == [6, 7] and np.flatnonzero(st["hist"][1]).tolist() == [9]
    assert np.flatnonzero(st["hist"][2]).tolist() == [10]


def test_parse_pairs_waits_and_stages_of_a_hand_built_trace():
    raw = hand_raw()
    blk = oracle.pairs_raw(raw)
    count, rows = binding.parse_pairs(blk, 1, 2, 16)
    assert count.tolist() == [[3, 1]]
    assert [tuple(int(x) for x in r) for r in rows[0, 0, :3]] == [(100, 200, 0, 0), (300, 600, 0, 1), (1000, 100, 1, 0)]
    assert tuple(int(x) for x in rows[0, 1, 0]) == (50, 2000, 0, 2)

    w = binding.parse_waits(oracle.waits_raw(raw))
    assert (w["n_wg"], w["waves_per_wg"], w["n_regions"]) == (1, 2, 3)
    # wave 0: after region 0's END comes a START at the same clock (wait 0), after region 1's END one 100 later
    assert w["n_waits"] == 2 and w["cnt"].tolist() == [1, 1, 0] and w["sum"].tolist() == [0, 100, 0]
    assert w["per"]["sum"][0, 0].tolist() == [0, 100, 0]

    hdr, tab = binding.parse_stages(oracle.stages_raw(blk, 1, 2, 8, 3, 4), 1, 3, 4)
    assert hdr == {"n_rows": 4, "n_clipped": 0, "n_bad_region": 0}
    assert tab["max_dur"][0].tolist() == [[200, 100, 0, 0], [600, 0, 0, 0], [2000, 0, 0, 0]]
    assert tab["n_waves"][0].tolist() == [[1, 1, 0, 0], [1, 0, 0, 0], [1, 0, 0, 0]]
    assert tab["min_start"][0, 0, :2].tolist() == [100, 1000] and tab["max_end"][0, 2, 0] == 2050


def test_parsers_agree_with_the_oracle_views_on_a_synthetic_trace():
    spec = inputs.TraceSpec(n_wg=6, waves=4, n_regions=5, cap_wave=64, total_per_wave=90, seed=21, p_orphan=0.04,
                            p_swap=0.01)
    raw, _ = inputs.gen_trace(spec)
    a, b = binding.parse_stats(oracle.decode_bytes(raw, 1)), oracle.decode(raw, 1)
    for k in ("hist", "cnt", "sum", "min", "max", "U", "O", "F", "per"):
        assert np.array_equal(a[k], b[k]), k
    for k in ("n_slots_valid", "n_pairs", "n_orphan_start", "n_orphan_end", "n_dropped", "n_disorder"):
        assert a[k] == b[k], k
    wa, wb = binding.parse_waits(oracle.waits_raw(raw)), oracle.waits(raw)
    for k in ("hist", "cnt", "sum", "min", "max", "uncovered", "async_cnt", "async_sum", "per"):
        assert np.array_equal(wa[k], wb[k]), k
    ca, ra = binding.parse_pairs(oracle.pairs_raw(raw), 6, 4, 256)
    cb, rb = oracle.pairs(raw)
    assert np.array_equal(ca, cb)
    for wg in range(6):
        for wv in range(4):
            assert np.array_equal(ra[wg, wv, : ca[wg, wv]], rb[wg, wv, : cb[wg, wv]])
    (ha, ta), (hb, tb) = binding.parse_stages(oracle.stages_raw(oracle.pairs_raw(raw), 6, 4, 64, 5, 16), 6, 5, 16), oracle.stages(raw, 16)
    assert ha == hb and np.array_equal(ta, tb)


def test_make_hdr_matches_the_generated_trace_header():
    spec = inputs.TraceSpec(n_wg=3, waves=2, n_regions=4, cap_wave=32, total_per_wave=20, seed=1)
    raw, _ = inputs.gen_trace(spec)
    h = binding.make_hdr(3, 2, 4, 32)
    words = np.frombuffer(bytes(h), dtype="<u4")
    assert words[:8].tolist() == raw[:8].tolist()

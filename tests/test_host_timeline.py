"""Host-side logic without a GPU: the Chrome Trace export of timeline rows (Sec. 3.2: decoded region
instances go to a timeline front end).  Rows come from the CPU oracle on a hand-built trace, so the
expected events can be written down."""
import json

import numpy as np

import inputs
import oracle
from paper_2505_21661_amd import timeline


def hand_trace():
    # one workgroup, two waves, two regions; wave 0: region 0 twice, region 1 once; wave 1: region 1 once
    S, E = 0, 1
    wg = inputs.events_to_wg([
        [(S, 0, 100), (E, 0, 300), (S, 1, 300), (E, 1, 900), (S, 0, 1000), (E, 0, 1100)],
        [(S, 1, 50), (E, 1, 2050)],
    ], 8)
    wg["wg_id"] = 7
    return inputs.encode_trace([wg], waves=2, n_regions=2, cap_wave=8)


def test_chrome_trace_events_of_a_hand_built_trace(tmp_path):
    raw = hand_trace()
    count, rows = oracle.pairs(raw)
    assert count.tolist() == [[3, 1]]
    ev = list(timeline.chrome_trace_events(count, rows, ["load", "mma"], ticks_per_us=100.0, wg_ids=[7]))
    got = [(e["pid"], e["tid"], e["name"], e["ts"], e["dur"], e["args"]["iter"]) for e in ev]
    assert got == [
        (7, 0, "load", 1.0, 2.0, 0),
        (7, 0, "mma", 3.0, 6.0, 0),
        (7, 0, "load", 10.0, 1.0, 1),
        (7, 1, "mma", 0.5, 20.0, 0),
    ]
    assert all(e["ph"] == "X" and e["cat"] == "kperf" for e in ev)
    assert [e["args"]["dur_ticks"] for e in ev] == [200, 600, 100, 2000]
    # regions without a name fall back to their number; max_wgs cuts the output
    ev2 = list(timeline.chrome_trace_events(count, rows, ["load"]))
    assert [e["name"] for e in ev2] == ["load", "region 1", "load", "region 1"] and ev2[0]["pid"] == 0
    assert list(timeline.chrome_trace_events(count, rows, max_wgs=0)) == []
    path = tmp_path / "t.json"
    n = timeline.write_chrome_trace(str(path), count, rows, ["load", "mma"])
    doc = json.loads(path.read_text())
    assert n == 4 and len(doc["traceEvents"]) == 4 and doc["displayTimeUnit"] == "ns"


def test_event_count_and_time_order_on_a_synthetic_trace():
    spec = inputs.TraceSpec(n_wg=5, waves=3, n_regions=4, cap_wave=64, total_per_wave=64, seed=11, p_orphan=0.05)
    raw, _ = inputs.gen_trace(spec)
    count, rows = oracle.pairs(raw)
    ev = list(timeline.chrome_trace_events(count, rows))
    assert len(ev) == int(count.sum())
    # rows of a wave are ordered by their END records: end times never decrease within a (pid, tid)
    last = {}
    for e in ev:
        key = (e["pid"], e["tid"])
        end = e["args"]["start_ticks"] + e["args"]["dur_ticks"]
        assert end >= last.get(key, 0)
        last[key] = end

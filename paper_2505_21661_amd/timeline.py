"""Chrome Trace export of the timeline rows produced by kp_trace_pairs.

The paper hands the decoded region instances to timeline front ends such as Chrome Trace
(Sec. 3.2) and shows per-iteration timelines of the instrumented kernels (Sec. 3.3, Fig. 5).
This module only formats rows that the GPU decoder has already produced: one complete event
("ph": "X") per row, process = recorded workgroup, thread = wave, name = region name, and the
iteration index in the event arguments.  Load the file in chrome://tracing or Perfetto.
"""
from __future__ import annotations

import json


def chrome_trace_events(count, rows, region_names=None, ticks_per_us: float = 100.0, wg_ids=None, max_wgs=None):
    """Yield Chrome Trace events for parsed pairs (see binding.parse_pairs).

    ticks_per_us converts clock ticks to the microseconds the format expects (s_memtime runs at
    the shader clock; kp_calibrate measures it).  max_wgs limits the output to the first workgroups.
    """
    n_wg, waves = count.shape
    if max_wgs is not None:
        n_wg = min(n_wg, max_wgs)
    for wg in range(n_wg):
        pid = int(wg_ids[wg]) if wg_ids is not None else wg
        for w in range(waves):
            for r in rows[wg, w, : int(count[wg, w])]:
                region = int(r["region"])
                name = region_names[region] if region_names and region < len(region_names) else f"region {region}"
                yield {
                    "name": name, "cat": "kperf", "ph": "X", "pid": pid, "tid": w,
                    "ts": int(r["start"]) / ticks_per_us, "dur": int(r["dur"]) / ticks_per_us,
                    "args": {"iter": int(r["iter"]), "region": region, "start_ticks": int(r["start"]),
                             "dur_ticks": int(r["dur"])},
                }


def write_chrome_trace(path: str, count, rows, region_names=None, ticks_per_us: float = 100.0, wg_ids=None,
                       max_wgs=None) -> int:
    """Write a Chrome Trace JSON file; returns the number of events written."""
    events = list(chrome_trace_events(count, rows, region_names, ticks_per_us, wg_ids, max_wgs))
    with open(path, "w") as f:
        json.dump({"traceEvents": events, "displayTimeUnit": "ns"}, f)
    return len(events)

"""Independent brute-force decoder used to pin the oracle on tiny traces.

Pure Python, written differently from oracle/ref_decode.c on purpose:
  * ordering uses a dict keyed by rank instead of a slot_of_rank array,
  * pairing uses one "open START" cell per region (a depth-1 stack) instead of
    walking each region's subsequence for adjacent START/END,
  * overlap is a tick-by-tick simulation of which regions are active in at
    least one wave, instead of an event sweep.
It reads the raw words directly and knows the trace layout only from the
format description (Sec. 4.2 of the paper for record size and flag bit).
"""
import numpy as np


def brute_decode(raw: np.ndarray) -> dict:
    raw = [int(x) for x in raw]
    assert raw[0] == 0x4652504B and raw[1] == 1
    n_wg, W, R, cap, rec_cost, flags = raw[2:8]
    flush = flags & 1
    rec0 = (64 + 128 * n_wg) // 4
    st = dict(n_slots_valid=0, n_pairs=0, n_orphan_start=0, n_orphan_end=0, n_invalid=0, n_dropped=0,
              n_disorder=0, n_span_overflow_wgs=0, n_nonmonotonic=0, n_overlap_wgs=0)
    hist = np.zeros((R, 64), dtype=np.uint64)
    cnt = np.zeros(R, dtype=np.uint64)
    ssum = np.zeros(R, dtype=np.uint64)
    smin = np.full(R, np.iinfo(np.uint64).max, dtype=np.uint64)
    smax = np.zeros(R, dtype=np.uint64)
    U = np.zeros(R, dtype=np.uint64)
    O = np.zeros((R, R), dtype=np.uint64)
    per = np.zeros((n_wg, W, R, 3), dtype=np.uint64)
    for wg in range(n_wg):
        h = (64 + 128 * wg) // 4
        t_begin = raw[h + 2] | (raw[h + 3] << 32)
        t_end = raw[h + 4] | (raw[h + 5] << 32)
        span = (t_end - t_begin) % (1 << 64)
        intervals = []  # (region, start, end)
        bad = 0
        nonmono = 0
        for w in range(W):
            T = raw[h + 8 + w]
            V = min(T, cap)
            st["n_dropped"] += T - V
            st["n_slots_valid"] += V
            first = 0 if flush else T - V
            by_rank = {}
            for s in range(V):
                tag = raw[rec0 + 2 * ((wg * W + w) * cap + s)]
                ts = raw[rec0 + 2 * ((wg * W + w) * cap + s) + 1]
                seq, wave, region, phase = tag & 0xFFFFF, (tag >> 20) & 15, (tag >> 24) & 127, tag >> 31
                k = (seq - first) % (1 << 20)
                if k >= V or wave != w or region >= R:
                    bad += 1
                    continue
                if k in by_rank:
                    bad += 1
                by_rank[k] = (s, seq, region, phase, ts)
            seqn = [by_rank[k] for k in sorted(by_rank)]
            st["n_disorder"] += sum(1 for (s, seq, *_r) in seqn if s != seq % cap)
            nonmono += sum(1 for a, b in zip(seqn, seqn[1:]) if b[4] < a[4])
            open_ts = [None] * R
            for (_s, _seq, region, phase, ts) in seqn:
                if phase == 0:
                    if open_ts[region] is not None:
                        st["n_orphan_start"] += 1
                    open_ts[region] = ts
                else:
                    if open_ts[region] is None:
                        st["n_orphan_end"] += 1
                    else:
                        d_raw = (ts - open_ts[region]) % (1 << 32)
                        d = max(0, d_raw - rec_cost)
                        st["n_pairs"] += 1
                        b = 0 if d < 2 else int(d).bit_length() - 1
                        hist[region, b] += np.uint64(1)
                        cnt[region] += np.uint64(1)
                        ssum[region] += np.uint64(d)
                        smin[region] = min(int(smin[region]), d)
                        smax[region] = max(int(smax[region]), d)
                        per[wg, w, region, 0] += np.uint64(d)
                        per[wg, w, region, 1] += np.uint64(1)
                        per[wg, w, region, 2] = max(int(per[wg, w, region, 2]), d)
                        intervals.append((region, open_ts[region], open_ts[region] + d_raw))
                        open_ts[region] = None
            st["n_orphan_start"] += sum(1 for x in open_ts if x is not None)
        st["n_invalid"] += bad
        st["n_nonmonotonic"] += nonmono
        if span >= (1 << 32):
            st["n_span_overflow_wgs"] += 1
            continue
        if bad or nonmono:
            continue
        st["n_overlap_wgs"] += 1
        if intervals:
            horizon = max(e for _r, _s, e in intervals)
            assert horizon < 200000, "brute force is for tiny traces"
            act = np.zeros((R, horizon), dtype=bool)
            for r, s, e in intervals:
                act[r, s:e] = True
            for a in range(R):
                U[a] += np.uint64(int(act[a].sum()))
                for b in range(R):
                    O[a, b] += np.uint64(int((act[a] & act[b]).sum()))
    F = np.zeros((R, R))
    for a in range(R):
        for b in range(R):
            F[a, b] = float(O[a, b]) / float(U[a]) if U[a] else 0.0
    st.update(hist=hist, cnt=cnt, sum=ssum, min=smin, max=smax, U=U, O=O, F=F, per=per)
    return st


def assert_same(ref: dict, got: dict):
    for k in ("n_slots_valid", "n_pairs", "n_orphan_start", "n_orphan_end", "n_invalid", "n_dropped",
              "n_disorder", "n_span_overflow_wgs", "n_nonmonotonic", "n_overlap_wgs"):
        assert ref[k] == got[k], (k, ref[k], got[k])
    for k in ("hist", "cnt", "sum", "min", "max", "U", "O"):
        assert np.array_equal(np.asarray(ref[k]), np.asarray(got[k])), k
    assert np.array_equal(np.asarray(ref["F"]), np.asarray(got["F"])), "F"
    p = got["per"]
    assert np.array_equal(ref["per"][..., 0], p["sum"])
    assert np.array_equal(ref["per"][..., 1], p["n"].astype(np.uint64))
    assert np.array_equal(ref["per"][..., 2], p["max"].astype(np.uint64))


def brute_pairs(raw: np.ndarray):
    """Independent timeline rows: per (wg, wave) a list of (start, dur, iter, region).

    Written differently from oracle/ref_pairs.c on purpose: the records of a wave are sorted by
    rank with a dict, each region's subsequence is extracted as a list and scanned for adjacent
    START/END neighbours, and the rows are then ordered by the rank of their END record.
    """
    raw = [int(x) for x in raw]
    assert raw[0] == 0x4652504B and raw[1] == 1
    n_wg, W, R, cap, rec_cost, flags = raw[2:8]
    flush = flags & 1
    rec0 = (64 + 128 * n_wg) // 4
    out = {}
    for wg in range(n_wg):
        h = (64 + 128 * wg) // 4
        for w in range(W):
            T = raw[h + 8 + w]
            V = min(T, cap)
            first = 0 if flush else T - V
            by_rank = {}
            for s in range(V):
                tag = raw[rec0 + 2 * ((wg * W + w) * cap + s)]
                ts = raw[rec0 + 2 * ((wg * W + w) * cap + s) + 1]
                seq, wave, region, phase = tag & 0xFFFFF, (tag >> 20) & 15, (tag >> 24) & 127, tag >> 31
                k = (seq - first) % (1 << 20)
                if k >= V or wave != w or region >= R:
                    continue
                by_rank[k] = (region, phase, ts)
            rows = []  # (rank of END, start, dur, iter, region)
            for r in range(R):
                sub = [(k, ph, ts) for k, (rg, ph, ts) in sorted(by_rank.items()) if rg == r]
                it = 0
                for (k0, p0, t0), (k1, p1, t1) in zip(sub, sub[1:]):
                    if p0 == 0 and p1 == 1:
                        rows.append((k1, t0, max(0, (t1 - t0) % (1 << 32) - rec_cost), it, r))
                        it += 1
            out[(wg, w)] = [row[1:] for row in sorted(rows)]
    return out


def brute_waits(raw: np.ndarray) -> dict:
    """Independent wait replay: for every (wg, wave) the list of (region, gap, whole) in rank order,
    `whole` = CLK2 - CLK0 (mod 2^32) when the END is paired, else None.

    Written differently from oracle/ref_waits.c on purpose: the records of a wave are put into one
    list in rank order, every adjacent (END, START) couple is a wait, and whether the END is paired
    is found by searching that list backwards for the nearest record of the END's region.
    """
    raw = [int(x) for x in raw]
    assert raw[0] == 0x4652504B and raw[1] == 1
    n_wg, W, R, cap, _rec_cost, flags = raw[2:8]
    flush = flags & 1
    rec0 = (64 + 128 * n_wg) // 4
    out = {}
    for wg in range(n_wg):
        h = (64 + 128 * wg) // 4
        for w in range(W):
            T = raw[h + 8 + w]
            V = min(T, cap)
            first = 0 if flush else T - V
            by_rank = {}
            for s in range(V):
                tag = raw[rec0 + 2 * ((wg * W + w) * cap + s)]
                ts = raw[rec0 + 2 * ((wg * W + w) * cap + s) + 1]
                seq, wave, region, phase = tag & 0xFFFFF, (tag >> 20) & 15, (tag >> 24) & 127, tag >> 31
                k = (seq - first) % (1 << 20)
                if k >= V or wave != w or region >= R:
                    continue
                by_rank[k] = (region, phase, ts)
            order = [by_rank[k] for k in sorted(by_rank)]
            waits = []
            for i in range(len(order) - 1):
                (ra, pa, ta), (_rb, pb, tb) = order[i], order[i + 1]
                if not (pa == 1 and pb == 0):
                    continue
                whole = None
                for rq, pq, tq in reversed(order[:i]):
                    if rq == ra:
                        if pq == 0:
                            whole = (tb - tq) % (1 << 32)
                        break
                waits.append((ra, (tb - ta) % (1 << 32), whole))
            out[(wg, w)] = waits
    return out


def waits_summary(raw: np.ndarray, per_wave: dict) -> dict:
    """Fold brute_waits' lists into the totals of the waits block (plain Python integers)."""
    n_wg, W, R, _cap, rec_cost = (int(x) for x in raw[2:7])
    z = lambda: [0] * R
    s = {"n_waits": 0, "n_uncovered": 0, "n_async": 0, "cnt": z(), "sum": z(), "min": [2 ** 64 - 1] * R, "max": z(),
         "uncovered": z(), "async_cnt": z(), "async_sum": z(), "hist": [[0] * 64 for _ in range(R)],
         "per": {}}
    for (wg, w), lst in per_wave.items():
        for a, gap, whole in lst:
            s["n_waits"] += 1
            s["cnt"][a] += 1
            s["sum"][a] += gap
            s["min"][a] = min(s["min"][a], gap)
            s["max"][a] = max(s["max"][a], gap)
            s["hist"][a][max(gap, 1).bit_length() - 1] += 1
            if gap <= rec_cost:
                s["n_uncovered"] += 1
                s["uncovered"][a] += 1
            if whole is not None:
                s["n_async"] += 1
                s["async_cnt"][a] += 1
                s["async_sum"][a] += max(whole - rec_cost, 0)
            sm, n, mx = s["per"].get((wg, w, a), (0, 0, 0))
            s["per"][(wg, w, a)] = (sm + gap, n + 1, max(mx, gap))
    return s


def assert_waits_same(ref: dict, got: dict):
    """ref: waits_summary(); got: oracle.view_waits() / the GPU block viewed the same way."""
    for k in ("n_waits", "n_uncovered", "n_async"):
        assert ref[k] == got[k], (k, ref[k], got[k])
    for k in ("cnt", "sum", "min", "max", "uncovered", "async_cnt", "async_sum"):
        assert [int(x) for x in got[k]] == ref[k], (k, ref[k], got[k])
    assert [[int(x) for x in row] for row in got["hist"]] == ref["hist"]
    per = got["per"]
    for wg in range(per.shape[0]):
        for w in range(per.shape[1]):
            for a in range(per.shape[2]):
                want = ref["per"].get((wg, w, a), (0, 0, 0))
                have = (int(per[wg, w, a]["sum"]), int(per[wg, w, a]["n"]), int(per[wg, w, a]["max"]))
                assert want == have, ((wg, w, a), want, have)


def brute_stages(raw: np.ndarray, max_iter: int):
    """Independent stage table straight from the raw trace: brute_pairs' rows of every wave are
    grouped by (wg, region, iter) in a dict.  Returns (n_rows, n_clipped, {key: (max_dur, min_start, max_end, n)})."""
    rows = brute_pairs(raw)
    tab, n_rows, n_clipped = {}, 0, 0
    for (wg, _w), lst in rows.items():
        for start, dur, it, region in lst:
            if it >= max_iter:
                n_clipped += 1
                continue
            n_rows += 1
            d, s, e, n = tab.get((wg, region, it), (0, 2 ** 32 - 1, 0, 0))
            tab[(wg, region, it)] = (max(d, dur), min(s, start), max(e, (start + dur) % (1 << 32)), n + 1)
    return n_rows, n_clipped, tab

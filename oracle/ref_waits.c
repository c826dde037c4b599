/*
 * CPU oracle for the asynchronous-wait part of the trace replay  --  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow reference for kp_trace_waits; shares no code, headers, tables or helpers with
 * the HIP library.  Only tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * Sec. 4.3 ("Trace Replay", asynchronous instructions): around an asynchronous operation the
 * records are placed as START before the launch (clock CLK0), END right before the barrier that
 * waits for it (CLK1) and a second START right after that barrier (CLK2).  Then
 *     T_wait = CLK2 - CLK1      (the two records' own costs cancel, nothing is subtracted),
 *     T_exe  = CLK1 - CLK0      (the synchronous stretch, an ordinary START/END pair),
 * and the measurement only holds while the functional unit outlasts the inserted record,
 * T_MMA - T_exe > T_a + T_b, with T_a + T_b the cost of one record.
 *
 * The paper gives no data format for this step.  This project's reading:
 *   - the records of one (workgroup, wave) are ordered by sequence number exactly as in the
 *     statistics decoder (valid slots, rank = seq - first surviving seq, a later slot displaces
 *     an earlier one of the same rank, foreign wave / unknown region / rank out of range dropped);
 *   - a "wait" is an END record of region a whose successor in that order is a START record (of
 *     any region); it belongs to region a and lasts gap = (u32)(CLK2 - CLK1);
 *   - it is "uncovered" when gap <= rec_cost (the trace header's cost of one record): what is left
 *     of the asynchronous operation at the barrier is then too short to hide the record, the
 *     paper's condition fails and the value is not to be trusted;
 *   - when that END is paired (the nearest earlier record of region a in the wave is a START, at
 *     CLK0) the asynchronous operation itself took T_async = (u32)(CLK2 - CLK0) minus rec_cost,
 *     not below 0 (one record, the END, sits inside the interval).
 *
 * Raw trace (little endian): 64-byte header {u32 magic 'KPRF', version, n_wg, waves, n_regions,
 * cap_wave, rec_cost, flags (bit0: flush)}; n_wg headers of 128 B {u32 wg_id, hw_id, u64 t_begin,
 * t_end, reserved, u32 total_written[16]}; records {u32 tag, u32 payload}, segment of (wg, w) at
 * slot (wg*waves + w)*cap_wave; tag[31] END, [30:24] region, [23:20] wave, [19:0] seq.
 *
 * Output, u64 words: 16 header words {n_waits, n_uncovered, n_async, 0 x5, n_wg, waves, n_regions,
 * cap_wave, rec_cost, 0 x3}; hist[R][64] (bin 0 for gap 0 and 1, else floor(log2 gap));
 * cnt[R], sum[R], min[R] (all ones when cnt is 0), max[R], uncovered[R], async_cnt[R],
 * async_sum[R]; then per (wg, wave, region) 16 bytes {u64 sum, u32 n, u32 max} of the gaps.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

size_t kpo_waits_bytes(uint32_t n_wg, uint32_t waves, uint32_t n_regions) {
  return 128 + 8 * ((size_t)64 * n_regions + 7 * (size_t)n_regions) + 16 * (size_t)n_wg * waves * n_regions;
}

/* Returns 0, or <0 when the header is not a valid trace of n_slots records. */
int kpo_waits(const void* raw, size_t n_slots, void* out, size_t out_bytes) {
  const uint32_t* h = (const uint32_t*)raw;
  if (h[0] != 0x4652504Bu || h[1] != 1u) return -1;
  const uint32_t n_wg = h[2], W = h[3], R = h[4], cap = h[5], rec_cost = h[6];
  const int flush = (int)(h[7] & 1u);
  if (W < 1 || W > 16 || R < 1 || R > 128 || cap < 2 || (cap & (cap - 1))) return -2;
  if ((size_t)n_wg * W * cap != n_slots) return -3;
  if (out_bytes < kpo_waits_bytes(n_wg, W, R)) return -4;
  const uint32_t* wg_hdrs = h + 16;
  const uint32_t* recs = wg_hdrs + (size_t)32 * n_wg;

  uint64_t* o = (uint64_t*)out;
  memset(o, 0, kpo_waits_bytes(n_wg, W, R));
  uint64_t* hist = o + 16;
  uint64_t* cnt = hist + (size_t)64 * R;
  uint64_t *sum = cnt + R, *mn = sum + R, *mx = mn + R, *unc = mx + R, *acnt = unc + R, *asum = acnt + R;
  uint64_t* per = asum + R; /* 2 words per (wg, w, region) */
  for (uint32_t r = 0; r < R; ++r) mn[r] = ~(uint64_t)0;
  o[8] = n_wg; o[9] = W; o[10] = R; o[11] = cap; o[12] = rec_cost;

  int64_t* slot_of_rank = (int64_t*)malloc(sizeof(int64_t) * cap);
  uint32_t* open_ts = (uint32_t*)malloc(sizeof(uint32_t) * R);
  uint8_t* is_open = (uint8_t*)malloc(R);
  if (!slot_of_rank || !open_ts || !is_open) return -5;

  for (uint32_t wg = 0; wg < n_wg; ++wg) {
    const uint32_t* wh = wg_hdrs + (size_t)32 * wg;
    for (uint32_t w = 0; w < W; ++w) {
      const size_t seg_i = (size_t)wg * W + w;
      const uint32_t* seg = recs + 2 * seg_i * cap;
      const uint32_t T = wh[8 + w];
      const uint32_t V = T < cap ? T : cap;
      const uint32_t first_seq = flush ? 0u : T - V; /* circular keeps the last V records */
      for (uint32_t k = 0; k < V; ++k) slot_of_rank[k] = -1;
      for (uint32_t s = 0; s < V; ++s) {
        const uint32_t tag = seg[2 * s];
        const uint32_t k = ((tag & 0xFFFFFu) - first_seq) & 0xFFFFFu;
        if (k >= V || ((tag >> 20) & 0xFu) != w || ((tag >> 24) & 0x7Fu) >= R) continue;
        slot_of_rank[k] = (int64_t)s; /* a later slot displaces an earlier one */
      }
      memset(is_open, 0, R);
      /* the previous record of the wave: whether it is an END, its region and clock, and the
         clock of the START it is paired with (if any) */
      int prev_is_end = 0, prev_paired = 0;
      uint32_t prev_region = 0, prev_ts = 0, prev_start = 0;
      for (uint32_t k = 0; k < V; ++k) {
        if (slot_of_rank[k] < 0) continue;
        const uint32_t tag = seg[2 * slot_of_rank[k]], ts = seg[2 * slot_of_rank[k] + 1];
        const uint32_t r = (tag >> 24) & 0x7Fu;
        if ((tag >> 31) == 0) { /* START */
          if (prev_is_end) { /* CLK1 = prev_ts, CLK2 = ts */
            const uint32_t a = prev_region;
            const uint32_t gap = ts - prev_ts;
            uint32_t bin = 0;
            while (bin < 31 && (gap >> (bin + 1))) ++bin;
            ++hist[(size_t)a * 64 + bin];
            ++cnt[a]; sum[a] += gap;
            if (gap < mn[a]) mn[a] = gap;
            if (gap > mx[a]) mx[a] = gap;
            ++o[0];
            if (gap <= rec_cost) { ++unc[a]; ++o[1]; }
            if (prev_paired) {
              const uint32_t whole = ts - prev_start;
              ++acnt[a]; ++o[2];
              asum[a] += whole > rec_cost ? whole - rec_cost : 0u;
            }
            uint64_t* p = per + 2 * (seg_i * R + a);
            p[0] += gap;
            uint32_t n = (uint32_t)p[1], m = (uint32_t)(p[1] >> 32);
            ++n; if (gap > m) m = gap;
            p[1] = (uint64_t)n | ((uint64_t)m << 32);
          }
          is_open[r] = 1; open_ts[r] = ts;
          prev_is_end = 0;
        } else { /* END */
          prev_is_end = 1; prev_region = r; prev_ts = ts;
          prev_paired = is_open[r]; prev_start = is_open[r] ? open_ts[r] : 0u;
          is_open[r] = 0;
        }
      }
    }
  }
  free(slot_of_rank); free(open_ts); free(is_open);
  return 0;
}

/*
 * CPU oracle for the timeline rows of the trace replay  --  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow reference for kp_trace_pairs; shares no code, headers, tables or helpers with
 * the HIP library.  Only tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * The paper decodes the raw profile buffer into one C struct per timed region instance, which
 * front ends turn into a timeline (Sec. 3.2: activity structs in the manner of the vendor's activity
 * API, Chrome Trace), and associates loop iterations with the records for its iteration-based
 * timing use case (Sec. 3.3 "Iteration-based Timing").  It stores START/END records unpaired and
 * aligns them at replay (Sec. 4.2); a constant record overhead is subtracted (Sec. 4.3).
 * The row layout, the order of the rows and the iteration index are this project's reading:
 *
 *   - the records of one (workgroup, wave) are ordered by sequence number exactly as in the
 *     statistics decoder (valid slots, rank = seq - first surviving seq, a later slot displaces
 *     an earlier one of the same rank, foreign wave / unknown region / rank out of range dropped);
 *   - inside each region's subsequence a START immediately followed by an END is a pair;
 *   - one row per pair: start = payload of the START (ticks since the workgroup began),
 *     dur = (u32)(end - start) minus the trace header's rec_cost, not below 0,
 *     iter = how many pairs of the same (workgroup, wave, region) precede it, region;
 *   - the rows of a wave are listed in the order of their END records (for one region that is
 *     also the order of the STARTs, because its pairs cannot nest).
 *
 * Raw trace (little endian): 64-byte header {u32 magic 'KPRF', version, n_wg, waves, n_regions,
 * cap_wave, rec_cost, flags (bit0: flush)}; n_wg headers of 128 B {u32 wg_id, hw_id, u64 t_begin,
 * t_end, reserved, u32 total_written[16]}; records {u32 tag, u32 payload}, segment of (wg, w) at
 * slot (wg*waves + w)*cap_wave; tag[31] END, [30:24] region, [23:20] wave, [19:0] seq.
 *
 * Output: u32 count[n_wg*waves] (padded with zeros to a multiple of 4 entries), then rows of
 * {u32 start, u32 dur, u32 iter, u32 region}; the rows of (wg, w) start at row index
 * (wg*waves + w) * (cap_wave/2); rows past count are left untouched.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

size_t kpo_pairs_bytes(uint32_t n_wg, uint32_t waves, uint32_t cap_wave) {
  const size_t n_seg = (size_t)n_wg * waves;
  return ((n_seg + 3) / 4) * 16 + n_seg * (cap_wave / 2) * 16;
}

/* Returns 0, or <0 when the header is not a valid trace of n_slots records. */
int kpo_pairs(const void* raw, size_t n_slots, void* out, size_t out_bytes) {
  const uint32_t* h = (const uint32_t*)raw;
  if (h[0] != 0x4652504Bu || h[1] != 1u) return -1;
  const uint32_t n_wg = h[2], W = h[3], R = h[4], cap = h[5], rec_cost = h[6];
  const int flush = (int)(h[7] & 1u);
  if (W < 1 || W > 16 || R < 1 || R > 128 || cap < 2 || (cap & (cap - 1))) return -2;
  if ((size_t)n_wg * W * cap != n_slots) return -3;
  if (out_bytes < kpo_pairs_bytes(n_wg, W, cap)) return -4;
  const uint32_t* wg_hdrs = h + 16;
  const uint32_t* recs = wg_hdrs + (size_t)32 * n_wg;
  const size_t n_seg = (size_t)n_wg * W;
  uint32_t* count = (uint32_t*)out;
  uint32_t* rows = count + ((n_seg + 3) / 4) * 4;
  for (size_t i = n_seg; i < ((n_seg + 3) / 4) * 4; ++i) count[i] = 0;

  int64_t* slot_of_rank = (int64_t*)malloc(sizeof(int64_t) * cap);
  uint32_t* open_ts = (uint32_t*)malloc(sizeof(uint32_t) * R);
  uint8_t* is_open = (uint8_t*)malloc(R);
  uint32_t* done = (uint32_t*)malloc(sizeof(uint32_t) * R);
  if (!slot_of_rank || !open_ts || !is_open || !done) return -5;

  for (uint32_t wg = 0; wg < n_wg; ++wg) {
    const uint32_t* wh = wg_hdrs + (size_t)32 * wg;
    for (uint32_t w = 0; w < W; ++w) {
      const size_t seg_i = (size_t)wg * W + w;
      const uint32_t* seg = recs + 2 * seg_i * cap;
      uint32_t* my_rows = rows + 4 * seg_i * (cap / 2);
      const uint32_t T = wh[8 + w];
      const uint32_t V = T < cap ? T : cap;
      /* circular keeps the last V records, flush the first V */
      const uint32_t first_seq = flush ? 0u : T - V;
      for (uint32_t k = 0; k < V; ++k) slot_of_rank[k] = -1;
      for (uint32_t s = 0; s < V; ++s) {
        const uint32_t tag = seg[2 * s];
        const uint32_t k = ((tag & 0xFFFFFu) - first_seq) & 0xFFFFFu;
        if (k >= V || ((tag >> 20) & 0xFu) != w || ((tag >> 24) & 0x7Fu) >= R) continue;
        slot_of_rank[k] = (int64_t)s; /* a later slot displaces an earlier one */
      }
      /* one pass in rank order with one "open START" cell per region */
      memset(is_open, 0, R);
      memset(done, 0, sizeof(uint32_t) * R);
      uint32_t n = 0;
      for (uint32_t k = 0; k < V; ++k) {
        if (slot_of_rank[k] < 0) continue;
        const uint32_t tag = seg[2 * slot_of_rank[k]], ts = seg[2 * slot_of_rank[k] + 1];
        const uint32_t r = (tag >> 24) & 0x7Fu;
        if ((tag >> 31) == 0) { /* START: opens, or replaces an orphan START */
          is_open[r] = 1; open_ts[r] = ts;
        } else if (is_open[r]) { /* END right after the START of its region */
          const uint32_t d_raw = ts - open_ts[r];
          uint32_t* row = my_rows + 4 * (size_t)n;
          row[0] = open_ts[r];
          row[1] = d_raw > rec_cost ? d_raw - rec_cost : 0u;
          row[2] = done[r];
          row[3] = r;
          ++done[r]; ++n; is_open[r] = 0;
        } /* else: orphan END, no row */
      }
      count[seg_i] = n;
    }
  }
  free(slot_of_rank); free(open_ts); free(is_open); free(done);
  return 0;
}

/*
 * CPU oracle for the per-iteration stage table  --  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow reference for kp_pairs_stages; shares no code, headers, tables or helpers with
 * the HIP library.  Only tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * The paper's critical-path analysis and its overlap models (Sec. 3.3 "Critical-path Analysis",
 * Sec. 5.2 "Performance Modeling for GPU Overlapping", Table 4) work on the latency of every stage
 * (region) in every loop iteration: T_load^i, T_comp^i, the stages on the critical path.  A stage
 * that several warps of a thread block execute together lasts as long as its slowest warp.  The
 * paper gives no data format; this project's reading is a table with one entry per (workgroup,
 * region, iteration), folded from the timeline rows {start, dur, iter, region} of the workgroup's
 * waves (one row per paired START/END, iter = ordinal of the pair within its wave and region):
 *     max_dur   = max over the waves' rows of dur          (the stage's latency)
 *     min_start = min over the rows of start               (when the first wave entered it)
 *     max_end   = max over the rows of (u32)(start + dur)  (when the last wave left it)
 *     n_waves   = number of rows folded in
 * Rows with iter >= max_iter are left out and counted (n_clipped); so are rows whose region is
 * not below n_regions (n_bad_region).  An entry without rows reads {0, 0xFFFFFFFF, 0, 0}.
 *
 * Input: the timeline block of kp_trace_pairs: u32 count[n_wg*waves] padded with zeros to a
 * multiple of 4 entries, then rows of {u32 start, dur, iter, region}, those of (wg, w) starting at
 * row (wg*waves + w) * (cap_wave/2); only the first count rows of a wave are read.
 * Output: 4 u64 {n_rows, n_clipped, n_bad_region, 0}, then entries [n_wg][n_regions][max_iter] of
 * 16 bytes {u32 max_dur, min_start, max_end, n_waves}.
 */
#include <stdint.h>
#include <stdlib.h>

size_t kpo_stages_bytes(uint32_t n_wg, uint32_t n_regions, uint32_t max_iter) {
  return 32 + 16 * (size_t)n_wg * n_regions * max_iter;
}

int kpo_stages(const void* pairs, uint32_t n_wg, uint32_t waves, uint32_t cap_wave, uint32_t n_regions,
               uint32_t max_iter, void* out, size_t out_bytes) {
  if (waves < 1 || waves > 16 || n_regions < 1 || n_regions > 128 || cap_wave < 2 || max_iter < 1) return -2;
  if (out_bytes < kpo_stages_bytes(n_wg, n_regions, max_iter)) return -4;
  const size_t n_seg = (size_t)n_wg * waves;
  const uint32_t* count = (const uint32_t*)pairs;
  const uint32_t* rows = count + ((n_seg + 3) / 4) * 4;
  uint64_t* hdr = (uint64_t*)out;
  uint32_t* tab = (uint32_t*)(hdr + 4);
  hdr[0] = hdr[1] = hdr[2] = hdr[3] = 0;
  for (size_t e = 0; e < (size_t)n_wg * n_regions * max_iter; ++e) {
    tab[4 * e + 0] = 0; tab[4 * e + 1] = 0xFFFFFFFFu; tab[4 * e + 2] = 0; tab[4 * e + 3] = 0;
  }
  for (uint32_t wg = 0; wg < n_wg; ++wg) {
    for (uint32_t w = 0; w < waves; ++w) {
      const size_t seg = (size_t)wg * waves + w;
      const uint32_t* r = rows + 4 * seg * (cap_wave / 2);
      for (uint32_t j = 0; j < count[seg]; ++j, r += 4) {
        const uint32_t start = r[0], dur = r[1], it = r[2], region = r[3];
        if (region >= n_regions) { ++hdr[2]; continue; }
        if (it >= max_iter) { ++hdr[1]; continue; }
        uint32_t* e = tab + 4 * (((size_t)wg * n_regions + region) * max_iter + it);
        const uint32_t end = start + dur;
        if (dur > e[0]) e[0] = dur;
        if (start < e[1]) e[1] = start;
        if (end > e[2]) e[2] = end;
        ++e[3];
        ++hdr[0];
      }
    }
  }
  return 0;
}

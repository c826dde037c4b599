/*
 * CPU oracle for the critical path over the stage table  --  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow reference for kp_stages_critical; shares no code, headers, tables or helpers with
 * the HIP library.  Only tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * The paper reads the critical path of a warp-specialised kernel off its timeline: a chain of stages
 * in different warp groups, each of which could only start once the one before it had finished
 * (Sec. 3.3, critical-path analysis; in the case study of Sec. 5.2 the path is made of GEMM and loading
 * stages, one blocking the next), and models the kernel's latency as the sum of the latencies of the
 * stages on it (Table 4, WS model).  It gives no algorithm.  This project's reading,
 * on the stage table (one entry {max_dur, min_start, max_end, n_waves} per workgroup, region and
 * iteration; an entry with n_waves = 0 is no stage):
 *   - the stages of a workgroup are ordered by (max_end, region * max_iter + iteration);
 *   - the path ends in the last stage of that order, the one that finishes last;
 *   - the stage before a stage X on the path is the one X waited for: the latest stage in that order,
 *     earlier than X, with max_end <= X.min_start; X is the first stage of the path if there is none;
 *   - every stage on the path adds 1 and its latency max_dur to its region's totals; the ticks
 *     between the end of a stage on the path and the start of the next are the path's bubbles.
 * Clocks are the table's 32-bit values, compared as plain unsigned numbers (a workgroup's span is
 * below 2^32 ticks in every trace that takes part in the statistics).
 *
 * Input: the stage block: 4 u64, then entries [n_wg][n_regions][max_iter] of 16 bytes
 * {u32 max_dur, min_start, max_end, n_waves}.
 * Output, u64 words: 8 header words {n_wg, n_regions, max_iter, workgroups with a path, stages on all
 * paths, sum of their latencies, sum of all bubbles, 0}; per region {stages on paths, their
 * latencies}; per workgroup 32 bytes {u32 stages on the path, u32 last stage (region << 16 |
 * iteration; all ones: no stage), u32 min_start of the first stage, u32 max_end of the last, u64 sum
 * of latencies, u64 bubbles}.
 */
#include <stdint.h>
#include <stdlib.h>

size_t kpo_critical_bytes(uint32_t n_wg, uint32_t n_regions) {
  return 64 + 16 * (size_t)n_regions + 32 * (size_t)n_wg;
}

int kpo_critical(const void* stages, uint32_t n_wg, uint32_t n_regions, uint32_t max_iter, void* out,
                 size_t out_bytes) {
  if (n_regions < 1 || n_regions > 128 || max_iter < 1 || max_iter > 65535) return -2;
  if (out_bytes < kpo_critical_bytes(n_wg, n_regions)) return -4;
  const uint32_t* tab = (const uint32_t*)((const uint64_t*)stages + 4);
  uint64_t* hdr = (uint64_t*)out;
  uint64_t* per_region = hdr + 8;
  uint32_t* rows = (uint32_t*)(per_region + 2 * (size_t)n_regions);
  const uint32_t n_ent = n_regions * max_iter;
  hdr[0] = n_wg; hdr[1] = n_regions; hdr[2] = max_iter;
  hdr[3] = hdr[4] = hdr[5] = hdr[6] = hdr[7] = 0;
  for (uint32_t r = 0; r < 2 * n_regions; ++r) per_region[r] = 0;
  for (uint32_t wg = 0; wg < n_wg; ++wg) {
    const uint32_t* e = tab + 4 * (size_t)wg * n_ent;
    uint32_t* row = rows + 8 * (size_t)wg;
    /* the stage that finishes last: greatest (max_end, index) */
    int64_t cur = -1;
    for (uint32_t i = 0; i < n_ent; ++i) {
      if (e[4 * i + 3] == 0) continue;
      if (cur < 0 || e[4 * i + 2] >= e[4 * cur + 2]) cur = i;  /* later index wins a tie */
    }
    uint32_t n = 0;
    uint64_t lat = 0, bubbles = 0;
    row[1] = 0xFFFFFFFFu; row[2] = 0; row[3] = 0;
    if (cur >= 0) {
      row[1] = ((uint32_t)(cur / max_iter) << 16) | (uint32_t)(cur % max_iter);
      row[3] = e[4 * cur + 2];
      ++hdr[3];
    }
    while (cur >= 0) {
      const uint32_t region = (uint32_t)(cur / max_iter);
      ++n;
      lat += e[4 * cur + 0];
      per_region[2 * region] += 1;
      per_region[2 * region + 1] += e[4 * cur + 0];
      row[2] = e[4 * cur + 1];
      /* the stage this one waited for */
      const uint32_t my_end = e[4 * cur + 2], my_start = e[4 * cur + 1];
      int64_t best = -1;
      for (uint32_t j = 0; j < n_ent; ++j) {
        if (e[4 * j + 3] == 0) continue;
        const uint32_t end_j = e[4 * j + 2];
        const int earlier = end_j < my_end || (end_j == my_end && (int64_t)j < cur);
        if (!earlier || end_j > my_start) continue;
        if (best < 0 || end_j > e[4 * best + 2] || (end_j == e[4 * best + 2] && (int64_t)j > best)) best = j;
      }
      if (best >= 0) bubbles += my_start - e[4 * best + 2];
      cur = best;
    }
    row[0] = n;
    ((uint64_t*)row)[2] = lat;
    ((uint64_t*)row)[3] = bubbles;
    hdr[4] += n; hdr[5] += lat; hdr[6] += bubbles;
  }
  return 0;
}

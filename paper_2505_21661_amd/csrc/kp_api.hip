// Size helpers and per-thread error text of the C ABI.
#include "kp_common.h"

namespace kp {
char* last_error_buf() {
  static thread_local char buf[kLastErrorLen] = {0};
  return buf;
}
}  // namespace kp

extern "C" const char* kp_last_error(void) { return kp::last_error_buf(); }

extern "C" size_t kp_trace_bytes(int n_wg, int waves_per_wg, int cap_per_wg) {
  if (n_wg < 0 || waves_per_wg < 1 || waves_per_wg > KP_MAX_WAVES || cap_per_wg < 0) return 0;
  if (cap_per_wg % waves_per_wg) return 0;
  return sizeof(kp_trace_hdr) + sizeof(kp_wg_hdr) * (size_t)n_wg + (size_t)8 * n_wg * (size_t)cap_per_wg;
}

extern "C" size_t kp_stats_bytes(int n_wg, int waves_per_wg, int n_regions) {
  if (n_wg < 0 || waves_per_wg < 1 || waves_per_wg > KP_MAX_WAVES || n_regions < 1) return 0;
  const size_t R = (size_t)n_regions;
  return sizeof(kp_stats_hdr) + 8 * (KP_HIST_BINS * R + 5 * R + 2 * R * R) +
         sizeof(kp_wave_region_stat) * (size_t)n_wg * waves_per_wg * R;
}

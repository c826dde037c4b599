// Size helpers and per-thread error text of the C ABI.
#include <atomic>

#include "kp_common.h"

namespace kp {
static std::atomic<uint32_t> g_rec_cost{0};
uint32_t rec_cost() { return g_rec_cost.load(std::memory_order_relaxed); }

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

extern "C" void kp_set_rec_cost(uint32_t ticks) { kp::g_rec_cost.store(ticks, std::memory_order_relaxed); }
extern "C" uint32_t kp_get_rec_cost(void) { return kp::rec_cost(); }

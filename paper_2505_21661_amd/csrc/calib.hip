// Calibration kernel (kp_calibrate): regions of known length bracketed by records.
//
// The paper quantifies the cost of one record with a micro-benchmark (Sec. 5.4 "Cycle-level
// Overhead") and compensates measured regions by that constant at replay (Sec. 4.3).  This
// kernel provides both numbers for gfx950: every wave runs n_regions regions back to back,
// region r being a chain of dependent v_fma_f32 (mode 0) or a run of s_sleep (mode 1) whose
// length is given by the caller; a region of length 0 measures the bare cost of a START/END
// record pair.  The decoded durations give ticks per FMA (timer unit) and the record cost.
// The records can carry either of the two clocks the hardware offers (the MetricType of the
// paper's ReadCounterOp, Sec. 3.1): the shader clock or the constant-rate 100 MHz clock; and they
// can be taken per wave or per group of four waves (its Granularity).
#include "kp_common.h"
#include "kp_record.h"

namespace {

struct CalibArgs {
  uint32_t cycles[KP_MAX_REGIONS];
  uint32_t n_regions;
  uint32_t mode;
  uint32_t rec_cost;
  uint32_t collab;  // all lanes store a record, hardware ids go to the workgroup header
};

// n dependent FMAs (rounded down to a multiple of 16); each waits for the previous result.
__device__ __forceinline__ void busy_fma(uint32_t n, float& x) {
  const float c = 1.0000001f;
  for (uint32_t i = n >> 4; i; --i) {
    asm volatile(
        "v_fma_f32 %0, %0, %1, %1\n v_fma_f32 %0, %0, %1, %1\n v_fma_f32 %0, %0, %1, %1\n v_fma_f32 %0, %0, %1, %1\n"
        "v_fma_f32 %0, %0, %1, %1\n v_fma_f32 %0, %0, %1, %1\n v_fma_f32 %0, %0, %1, %1\n v_fma_f32 %0, %0, %1, %1\n"
        "v_fma_f32 %0, %0, %1, %1\n v_fma_f32 %0, %0, %1, %1\n v_fma_f32 %0, %0, %1, %1\n v_fma_f32 %0, %0, %1, %1\n"
        "v_fma_f32 %0, %0, %1, %1\n v_fma_f32 %0, %0, %1, %1\n v_fma_f32 %0, %0, %1, %1\n v_fma_f32 %0, %0, %1, %1\n"
        : "+v"(x)
        : "v"(c));
  }
}

__device__ __forceinline__ void busy_sleep(uint32_t n) {
  for (uint32_t i = n; i; --i) asm volatile("s_sleep 1");
}

__device__ __forceinline__ void busy(uint32_t mode, uint32_t len, float& x) {
  if (mode == 0) busy_fma(len >> 2, x); else busy_sleep(len >> 6);
}

// SITE: the form of the record sites (kp_record.h): 1 generic, 2 lean (records written to LDS at the
// next site), 4 chained (clock reads parked in scalar registers, their clocks stored after the region, the
// records made when the trace is copied out).  The instrumented kernels use all three; a region costs a
// different constant with each.
struct CalibChain {  // site 2 r opens region r, site 2 r + 1 closes it (every region enabled)
  static constexpr bool kDense = false;
  __device__ uint32_t total(uint32_t n, uint32_t) const { return n; }
  __device__ uint32_t end_region(uint32_t site, uint32_t) const { return (site & 1u) ? site >> 1 : kp::kNoRegion; }
  __device__ uint32_t start_region(uint32_t site, uint32_t) const { return (site & 1u) ? kp::kNoRegion : site >> 1; }
};

template <bool REALTIME, bool GROUPS, int SITE>
__global__ __launch_bounds__(1024) void kp_calib_kernel(CalibArgs a, void* trace, uint32_t cap_lds,
                                                        uint32_t cap_hbm, uint32_t flush, uint32_t n_wg,
                                                        uint32_t streams, uint32_t group_log2, float* sink) {
  extern __shared__ __align__(16) uint32_t lds_ring[];  // ring first, the rest only limits occupancy
  __shared__ uint64_t t_begin[2];
  kp::Ring r = kp::ring_init<GROUPS>(lds_ring, t_begin, cap_lds, 0xFFFFFFFFu, flush, cap_hbm, trace, n_wg, streams, blockIdx.x,
                             group_log2);
  if constexpr (REALTIME) kp::ring_use_realtime(r);
  r.collab = a.collab;
  float x = (float)threadIdx.x;
  // Two identical passes: the first warms the instruction cache and is then discarded by
  // resetting the ring state, so that no recorded region pays for a cold code fetch.
  for (int pass = 0; pass < 2; ++pass) {
    if constexpr (SITE == 1) {
      r.cnt = 0;
      r.stored = 0;
      r.pend_tag = kp::kNoPending;
      r.pend_tag2 = kp::kNoPending;
      for (uint32_t rg = 0; rg < a.n_regions; ++rg) {
        kp::record<REALTIME>(r, rg, kp::kPhaseStart);
        busy(a.mode, a.cycles[rg], x);
        kp::record<REALTIME>(r, rg, kp::kPhaseEnd);
      }
      if (pass == 0) kp::store_pending(r);
    } else if constexpr (SITE == 2) {
      kp::lean_begin(r);
      for (uint32_t rg = 0; rg < a.n_regions; ++rg) {
        kp::boundary_fast(r, kp::kNoRegion, rg);
        busy(a.mode, a.cycles[rg], x);
        kp::boundary_fast(r, rg, kp::kNoRegion);
      }
      if (pass == 0) (void)kp::clock_delta(r.pend_t, r.t0_lo);  // the last clock read has to land before the reset
      else kp::lean_end(r);
    } else {
      kp::chain_begin(r);
      for (uint32_t rg = 0; rg < a.n_regions; ++rg) {
        kp::site_chain<0>(r);
        busy(a.mode, a.cycles[rg], x);
        kp::site_chain<1>(r);
        kp::chain_commit<2>(r);
      }
    }
  }
  if (x == 12345.6789f && sink) *sink = x;  // keeps the FMA chain alive
  kp::TraceGeom g{n_wg, streams, a.n_regions, cap_hbm,
                  (flush ? KP_FLAG_FLUSH : 0u) | (REALTIME ? KP_FLAG_REALTIME : 0u) | (a.collab ? KP_FLAG_HW_IDS : 0u)};
  if constexpr (SITE == 4) kp::ring_finish<REALTIME>(r, cap_lds, trace, g, blockIdx.x, a.rec_cost, CalibChain{});
  else kp::ring_finish<REALTIME>(r, cap_lds, trace, g, blockIdx.x, a.rec_cost);
}

}  // namespace

extern "C" kp_status kp_calibrate(const uint32_t* cycles, int n_regions, int n_wg, int waves, int mode,
                                  void* trace_buf, size_t trace_cap, void* stream) {
  kp::clear_error();
  if (!cycles || !trace_buf) return kp::fail(KP_ERR_INVALID_ARG, "NULL argument");
  if (n_regions < 1 || n_regions > KP_MAX_REGIONS || n_wg < 1 || waves < 1 || waves > KP_MAX_WAVES || (mode & ~127))
    return kp::fail(KP_ERR_INVALID_ARG, "n_regions=%d n_wg=%d waves=%d mode=%d", n_regions, n_wg, waves, mode);
  const int site = (mode & 16) ? 2 : ((mode & 32) ? 4 : 1);
  if ((mode & 48) == 48 || (site != 1 && (mode & (2 | 4 | 8 | 64))))
    return kp::fail(KP_ERR_INVALID_ARG, "mode=%d: the lean and chained site forms record per wave, on the shader clock, circular", mode);
  const uint32_t group_log2 = (mode & 8) ? 2u : 0u;
  if (group_log2 && (waves & 3)) return kp::fail(KP_ERR_INVALID_ARG, "wave-group records need a multiple of 4 waves, got %d", waves);
  const size_t streams = (size_t)(waves >> group_log2);
  if (trace_cap % streams) return kp::fail(KP_ERR_TRACE_TOO_SMALL, "trace_cap must be a multiple of the %zu record streams", streams);
  const size_t cap_wave = trace_cap / streams;
  if (!kp::is_pow2(cap_wave) || cap_wave < 2 || cap_wave > (1u << 19))
    return kp::fail(KP_ERR_TRACE_TOO_SMALL, "trace_cap/streams = %zu must be a power of two >= 2", cap_wave);
  const uint32_t flush = (mode & 2) ? 1u : 0u;
  // circular: the LDS sub-ring is the whole segment; flush: a small LDS sub-ring is spilled in chunks
  uint32_t cap_lds = (uint32_t)cap_wave;
  if (flush && cap_lds > 8) cap_lds = 8;
  if ((size_t)cap_lds * 8 * streams > 64 * 1024)
    return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "ring of %zu records per workgroup exceeds 64 KiB of LDS", trace_cap);
  CalibArgs a{};
  for (int i = 0; i < n_regions; ++i) a.cycles[i] = cycles[i];
  a.n_regions = (uint32_t)n_regions;
  a.mode = (uint32_t)(mode & 1);
  a.rec_cost = kp::rec_cost();
  a.collab = (mode & 64) ? 1u : 0u;
  // more than half of the CU's LDS per workgroup: one workgroup per CU, one wave per SIMD for waves <= 4
  const uint32_t lds_bytes = 96 * 1024;
  static thread_local int attr_dev = -1;  // the attribute is kept per device
  int dev = 0;
  KP_HIP_TRY(hipGetDevice(&dev));
  if (attr_dev != dev) {
    for (auto k : {kp_calib_kernel<false, false, 1>, kp_calib_kernel<true, false, 1>, kp_calib_kernel<false, true, 1>,
                   kp_calib_kernel<true, true, 1>, kp_calib_kernel<false, false, 2>, kp_calib_kernel<false, false, 4>})
      KP_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)lds_bytes));
    attr_dev = dev;
  }
  auto kern = site == 2 ? kp_calib_kernel<false, false, 2>
            : site == 4 ? kp_calib_kernel<false, false, 4>
            : group_log2 ? ((mode & 4) ? kp_calib_kernel<true, true, 1> : kp_calib_kernel<false, true, 1>)
                         : ((mode & 4) ? kp_calib_kernel<true, false, 1> : kp_calib_kernel<false, false, 1>);
  hipLaunchKernelGGL(kern, dim3(n_wg), dim3(waves * 64), lds_bytes, static_cast<hipStream_t>(stream),
                     a, trace_buf, cap_lds, (uint32_t)cap_wave, flush, (uint32_t)n_wg, (uint32_t)streams, group_log2,
                     static_cast<float*>(nullptr));
  KP_HIP_TRY(hipGetLastError());
  return KP_OK;
}

// What the two statistics decoders (the LDS-resident one and the one for wide geometries) share: the
// layout of the statistics block and the hand-over between them.
#pragma once
#include "kp_common.h"

namespace kp_reduce {

// positions inside kp_stats_hdr, in u64 words
enum { H_SLOTS_VALID = 0, H_PAIRS, H_ORPHAN_START, H_ORPHAN_END, H_INVALID, H_DROPPED, H_DISORDER,
       H_SPAN_OVF, H_NONMONO, H_OVERLAP_WGS, H_STATUS, H_NWG, H_WAVES, H_NREG, H_CAP, H_RSVD };

struct StatsLayout {  // offsets in u64 words
  size_t hist, cnt, sum, min, max, U, O, F, per, total;
};
__host__ __device__ inline StatsLayout stats_layout(uint32_t n_wg, uint32_t W, uint32_t R) {
  StatsLayout l;
  l.hist = 16;
  l.cnt = l.hist + (size_t)64 * R;
  l.sum = l.cnt + R; l.min = l.sum + R; l.max = l.min + R; l.U = l.max + R;
  l.O = l.U + R;
  l.F = l.O + (size_t)R * R;
  l.per = l.F + (size_t)R * R;
  l.total = l.per + (size_t)2 * n_wg * W * R;
  return l;
}

// The main kernel of the decoder for geometries the LDS-resident one does not take (more than 32
// regions, more than 16384 record slots per workgroup).  Between the init and finalize kernels, on the
// same stream; accumulates into the block exactly as the LDS-resident kernel does (histogram, sums,
// extrema and header counts by atomics, the region-pair sums staged in the F area).  The header has
// been validated by the caller.  wide_supported: KP_ERR_UNSUPPORTED_SHAPE when one workgroup's records
// exceed what the kernel can mark in LDS.
kp_status wide_supported(const kp_trace_hdr& h);
kp_status launch_wide(const uint32_t* wg_hdrs, const void* records, uint64_t* out, const kp_trace_hdr& h,
                      hipStream_t s);

}  // namespace kp_reduce

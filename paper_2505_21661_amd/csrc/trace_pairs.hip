// GPU timeline rows of the trace replay (kp_trace_pairs).
//
// The paper decodes the raw profile buffer into one struct per timed region instance, which
// front ends such as Chrome Trace turn into a timeline (Sec. 3.2), and ties loop iterations to
// the records for its iteration-based timing (Sec. 3.3 "Iteration-based Timing"); records are
// stored unpaired and aligned at replay (Sec. 4.2), and a constant record cost is subtracted
// (Sec. 4.3).  This kernel does that replay on the GPU: one row {start, dur, iter, region} per
// paired START/END of a (workgroup, wave), where iter counts the earlier pairs of the same region
// in that wave.
//
// One decoder workgroup stages one recorded workgroup in LDS as (clock, metadata) pairs, ordered by
// rank.  Then the hardware waves share out the recorded waves in runs of consecutive ranks and walk
// them 64 ranks per round (a run above rank 0 first counts the pairs below it):
//   - an END looks at the four ranks below through DPP wave shifts for the nearest record of its
//     region (deeper only if needed) and is paired iff that record is a START;
//   - its row index is the running count of paired ENDs (ballot + popcount);
//   - its iteration index comes from byte-wide per-region counters packed four to a 32-bit
//     word and prefix-summed across the lanes, on top of the per-region totals of earlier rounds.
#include "kp_stage.h"

namespace {

using namespace kp_stage;

constexpr uint32_t kBelowStride = 128;  // one counter per region

struct PairsOut {
  uint32_t* count;  // pairs per (workgroup, wave)
  u32x4* rows;      // cap/2 rows per (workgroup, wave)
};

template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void kp_pairs_main(Trace p, PairsOut o, uint32_t split_log2) {
  extern __shared__ __align__(16) unsigned char smem[];
  const Lds L = lds_layout(p.nrec);
  const uint2* rec = reinterpret_cast<const uint2*>(smem + L.rec);
  const uint32_t* recw = reinterpret_cast<const uint32_t*>(smem + L.rec);  // word 2p = clock, 2p+1 = metadata
  const uint32_t* sV = reinterpret_cast<const uint32_t*>(smem + L.v);
  uint32_t* below = reinterpret_cast<uint32_t*>(smem + L.end);  // per hardware wave: pairs per region below its run

  const uint32_t tid = threadIdx.x, lane = tid & 63u, hw = tid >> 6;
  const uint32_t W = p.W, R = p.R, cap = p.cap, cl2 = p.cap_log2;
  const uint32_t nwords = (R + 3u) >> 2;
  const unsigned long long lt_mask = (1ull << lane) - 1ull;

  // the padding entries of the count array are part of the output: zero
  if (blockIdx.x == 0 && tid < ((0u - p.n_wg * W) & 3u)) o.count[(size_t)p.n_wg * W + tid] = 0u;
  for (uint32_t i = tid; i < (BLOCK / 64) * kBelowStride; i += BLOCK) below[i] = 0u;
  // stage_workgroup's first barrier orders these stores before any use

  uint32_t iter = 0;
  for (uint32_t wg = blockIdx.x; wg < p.n_wg; wg += gridDim.x, ++iter) {
    stage_workgroup<BLOCK>(p, smem, L, wg, iter);
    const uint32_t live_tag = live_tag_of(iter);
    // ---- walk: 2^split_log2 hardware waves share one recorded wave -----------------------------------
    // Each emits the rows of a run of consecutive ranks.  A run that does not start at rank 0 first
    // counts the pairs below it (total and per region) with the same pairing rounds, so that its row
    // and iteration indices continue those of the runs below; no wave waits for another.
    if (hw < (W << split_log2)) {
      const uint32_t w = hw >> split_log2, part = hw & ((1u << split_log2) - 1u);
      const uint32_t wofs = w << cl2, V = sV[w];
      const uint32_t plen = cap >> split_log2;
      const uint32_t k0 = part * plen, k1 = V < k0 + plen ? V : k0 + plen;  // this wave emits ranks [k0, k1)
      const uint32_t kc = V < k0 ? V : k0;                                   // and counts ranks [0, kc)
      uint32_t* my_below = below + hw * kBelowStride;
      uint32_t base_lo = 0u, base_hi = 0u;  // pairs seen so far: lane r for region r / region 64 + r
      u32x4* my_rows = o.rows + ((size_t)wg * W + w) * (cap / 2);
      uint32_t n_rows = 0;
      uint32_t cm[4] = {0u, 0u, 0u, 0u};  // metadata of the last four ranks of the previous round
      uint2 r_next = rec[wofs + (lane < V ? lane : 0u)];  // one round ahead, to hide the LDS latency
      uint32_t m0, t0, region, pq;
      // One round of 64 ranks from kb, of a walk that ends at k_end: an END is paired iff the nearest
      // earlier record of its region is a START (four ranks through DPP shifts, deeper through LDS).
      auto pair_round = [&](uint32_t kb, uint32_t k_end) __attribute__((always_inline)) -> bool {
        const uint32_t k = kb + lane;
        const bool in = k < k_end;
        const uint32_t q0 = wofs + (in ? k : k_end - 1);
        const uint2 r0 = r_next;
        {
          const uint32_t kn = k + 64;
          r_next = rec[wofs + (kn < V ? kn : 0u)];
        }
        const bool valid = in && is_live(r0.y, live_tag);
        m0 = valid ? r0.y : 0u;
        t0 = r0.x;
        const uint32_t m1 = wave_shr1(m0, cm[0]);
        const uint32_t m2 = wave_shr1(m1, cm[1]);
        const uint32_t m3 = wave_shr1(m2, cm[2]);
        const uint32_t m4 = wave_shr1(m3, cm[3]);
#pragma unroll
        for (int j = 0; j < 4; ++j) cm[j] = (uint32_t)__builtin_amdgcn_readlane((int)m0, 63 - j);
        region = m0 & kMRegion;
        const bool is_end = (m0 & kMEnd) != 0u;  // m0 is 0 for a rank that holds no record
        const uint32_t want = kMValid | region, sel = kMValid | kMRegion;
        const bool h1 = (m1 & sel) == want, h2 = (m2 & sel) == want, h3 = (m3 & sel) == want, h4 = (m4 & sel) == want;
        bool have = h1 || h2 || h3 || h4;  // nearest earlier record of the same region
        uint32_t pm = h1 ? m1 : (h2 ? m2 : (h3 ? m3 : m4));
        pq = q0 - (h1 ? 1u : (h2 ? 2u : (h3 ? 3u : 4u)));
        if (is_end && !have && k > 4) {  // slow path: walk further back
          for (uint32_t kk = k - 4; kk-- > 0;) {
            const uint32_t mq = recw[2 * (wofs + kk) + 1];
            if (is_live(mq, live_tag) && (mq & kMRegion) == region) { have = true; pm = mq; pq = wofs + kk; break; }
          }
        }
        return is_end && have && !(pm & kMEnd);
      };
      // ---- count the pairs below this run ---------------------------------------------------------------
      for (uint32_t kb = 0; kb < kc; kb += 64) {  // kc is a multiple of 64 or the end of the wave
        const bool paired = pair_round(kb, kc);
        n_rows += (uint32_t)__popcll(__builtin_amdgcn_ballot_w64(paired));
        if (paired) atomicAdd(&my_below[region], 1u);
      }
      if (k0 > 0) {  // uniform; LDS operations of one wave complete in order
        base_lo = my_below[lane];
        base_hi = my_below[64 + lane];
        my_below[lane] = 0u;
        my_below[64 + lane] = 0u;
      }
      // ---- emit the rows of this run ------------------------------------------------------------------------
      for (uint32_t kb = k0; kb < k1; kb += 64) {
        const bool paired = pair_round(kb, k1);
        const unsigned long long pb = __builtin_amdgcn_ballot_w64(paired);
        if (pb == 0ull) continue;
        // iteration index: pairs of this region in earlier rounds + earlier lanes of this round.
        // The totals of earlier rounds live in registers: lane r holds the count of region r in
        // base_lo and of region 64 + r in base_hi.  Within the round four regions share a 32-bit
        // word of byte-wide counters (at most 64 per round, so no byte carries into its neighbour and
        // one 32-bit prefix sum counts four regions at once).
        const uint32_t pt = recw[2 * (paired ? pq : wofs)];  // the START's clock, fetched early
        const int from = (int)((region & 63u) << 2);
        uint32_t it = (uint32_t)__builtin_amdgcn_ds_bpermute(from, (int)base_lo);
        if (R > 64u) {  // uniform: every lane takes part in the exchange
          const uint32_t hi = (uint32_t)__builtin_amdgcn_ds_bpermute(from, (int)base_hi);
          if (region >= 64u) it = hi;
        }
        for (uint32_t wd = 0; wd < nwords; ++wd) {
          const bool mine = paired && (region >> 2) == wd;
          if (__builtin_amdgcn_ballot_w64(mine) == 0ull) continue;
          const uint32_t sh = 8u * (region & 3u);
          const uint32_t one = mine ? (1u << sh) : 0u;
          const uint32_t incl = wave_scan_add(one);
          if (mine) it += ((incl - one) >> sh) & 0xFFu;
          const uint32_t tot = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
          // the four lanes that own this word's regions add their byte of the round's totals
          const uint32_t add = (tot >> (8u * (lane & 3u))) & 0xFFu;
          if (wd < 16u) base_lo += (lane >> 2) == wd ? add : 0u;
          else          base_hi += (lane >> 2) == wd - 16u ? add : 0u;
        }
        if (paired) {
          const uint32_t d_raw = t0 - pt;
          const uint32_t d = d_raw > p.rec_cost ? d_raw - p.rec_cost : 0u;
          const uint32_t j = n_rows + (uint32_t)__popcll(pb & lt_mask);
          my_rows[j] = u32x4{pt, d, it, region};
        }
        n_rows += (uint32_t)__popcll(pb);
      }
      // the wave with the last run knows the total
      if (lane == 0 && part + 1u == (1u << split_log2)) o.count[(size_t)wg * W + w] = n_rows;
    }
    __syncthreads();
  }
}

template <int BLOCK>
kp_status launch_pairs(const Trace& p, const PairsOut& o, uint32_t lds_bytes, hipStream_t s) {
  // hardware waves per recorded wave: as many as the block has, while a run keeps at least 64 ranks
  uint32_t split_log2 = 0;
  while ((p.W << (split_log2 + 1)) <= (uint32_t)BLOCK / 64u && (p.cap >> (split_log2 + 1)) >= 64u) ++split_log2;
  auto kern = kp_pairs_main<BLOCK>;
  static thread_local LaunchCache cache;
  uint32_t grid = 0;
  const kp_status st = resident_grid(kern, BLOCK, lds_bytes, &cache, &grid);
  if (st != KP_OK) return st;
  if (grid > p.n_wg) grid = p.n_wg;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(BLOCK), lds_bytes, s, p, o, split_log2);
  KP_HIP_TRY(hipGetLastError());
  return KP_OK;
}

size_t count_bytes(size_t n_seg) { return ((n_seg + 3) / 4) * 16; }

kp_status pairs_impl(const void* raw, size_t n, const kp_trace_hdr& h, void* out_pairs, hipStream_t s) {
  Trace p;
  const kp_status st = trace_from_header(raw, n, h, out_pairs, &p);
  if (st != KP_OK) return st;
  const int block = block_threads(p.W, p.nrec);
  const uint32_t lds = lds_layout(p.nrec).end + (uint32_t)(block / 64) * kBelowStride * 4u;
  if (lds > kMaxLds)
    return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "timeline kernel needs %u B of LDS for this geometry (limit %u)", lds, kMaxLds);
  if (h.n_wg == 0) return KP_OK;

  uint8_t* out = static_cast<uint8_t*>(out_pairs);
  PairsOut o;
  o.count = reinterpret_cast<uint32_t*>(out);
  o.rows = reinterpret_cast<u32x4*>(out + count_bytes((size_t)p.n_wg * p.W));
  return block == 1024 ? launch_pairs<1024>(p, o, lds, s)
       : block == 512  ? launch_pairs<512>(p, o, lds, s)
                       : launch_pairs<256>(p, o, lds, s);
}

}  // namespace

extern "C" size_t kp_pairs_bytes(int n_wg, int waves_per_wg, int cap_per_wg) {
  if (n_wg < 0 || waves_per_wg < 1 || waves_per_wg > KP_MAX_WAVES || cap_per_wg < 0 || cap_per_wg % waves_per_wg) return 0;
  const size_t n_seg = (size_t)n_wg * waves_per_wg, cap_wave = (size_t)cap_per_wg / waves_per_wg;
  return count_bytes(n_seg) + n_seg * (cap_wave / 2) * sizeof(kp_pair_row);
}

extern "C" kp_status kp_trace_pairs_hdr(const void* raw, size_t n, const kp_trace_hdr* hdr_host,
                                        void* out_pairs, void* stream) {
  kp::clear_error();
  if (!raw || !hdr_host || !out_pairs) return kp::fail(KP_ERR_INVALID_ARG, "NULL argument");
  return pairs_impl(raw, n, *hdr_host, out_pairs, static_cast<hipStream_t>(stream));
}

extern "C" kp_status kp_trace_pairs(const void* raw, size_t n, void* out_pairs, void* stream) {
  kp::clear_error();
  if (!raw || !out_pairs) return kp::fail(KP_ERR_INVALID_ARG, "NULL argument");
  kp_trace_hdr h;
  hipStream_t s = static_cast<hipStream_t>(stream);
  KP_HIP_TRY(hipMemcpyAsync(&h, raw, sizeof h, hipMemcpyDeviceToHost, s));
  KP_HIP_TRY(hipStreamSynchronize(s));
  return pairs_impl(raw, n, h, out_pairs, s);
}

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
// One decoder workgroup stages one recorded workgroup in LDS as (clock, metadata) pairs, exactly
// as the statistics decoder does (scatter by rank = seq - first surviving seq; a duplicated rank
// is redone serially so that the later slot wins).  Then hardware wave w walks recorded wave w,
// 64 ranks per round:
//   - an END looks at the four ranks below through DPP wave shifts for the nearest record of its
//     region (deeper only if needed) and is paired iff that record is a START;
//   - its row index is the running count of paired ENDs (ballot + popcount);
//   - its iteration index comes from byte-wide per-region counters packed four to a 32-bit
//     word and prefix-summed across the lanes, on top of the per-region totals of earlier rounds.
#include "kp_common.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr uint32_t kSeqMask = 0xFFFFFu;
// staged metadata: bits 6:0 region, 7 END, 8 valid, 31:16 generation of the staging pass
constexpr uint32_t kMRegion = 0x7Fu, kMEnd = 0x80u, kMValid = 0x100u;
constexpr uint32_t kMaxRecPerWg = 16384;
constexpr uint32_t kMaxLds = 160 * 1024;

enum { T_FIELDVALID = 0, T_OCCUPIED, T_COUNT };

struct PairsParams {
  const uint32_t* wg_hdrs;  // 32 words per recorded workgroup
  const u32x4* records;     // two records per 16-byte load
  uint32_t* count;          // pairs per (workgroup, wave)
  u32x4* rows;              // cap/2 rows per (workgroup, wave)
  uint32_t n_wg, W, R, cap, cap_log2, rec_cost, flush, nrec;
};

struct LdsLayout { uint32_t rec, tmp, v, first, total; };
__host__ __device__ inline uint32_t align16(uint32_t x) { return (x + 15u) & ~15u; }
__host__ __device__ inline LdsLayout lds_layout(uint32_t nrec, uint32_t W, uint32_t R) {
  LdsLayout l;
  uint32_t o = 0;
  l.rec = o; o = align16(o + nrec * 8);
  l.tmp = o; o = align16(o + T_COUNT * 4);
  l.v = o; o = align16(o + 16 * 4);
  l.first = o; o = align16(o + 16 * 4);
  l.total = o;
  return l;
}

__device__ inline uint32_t wave_sum(uint32_t v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
  return v;
}

// Lane l receives the value of lane l-1; lane 0 receives `lane0` (DPP wave shift right by one).
__device__ __forceinline__ uint32_t wave_shr1(uint32_t v, uint32_t lane0) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)lane0, (int)v, 0x138, 0xF, 0xF, false);
}

// Inclusive prefix sum over the 64 lanes: four shifts inside each row of 16, then the last lane of
// row 0/2 into row 1/3 and the last lane of the lower half into the upper half.
__device__ __forceinline__ uint32_t wave_scan_add(uint32_t v) {
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xF, 0xF, false);  // row_shr:1
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xF, 0xF, false);  // row_shr:2
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xF, 0xF, false);  // row_shr:4
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xF, 0xF, false);  // row_shr:8
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xA, 0xF, false);  // row_bcast:15
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xC, 0xF, false);  // row_bcast:31
  return v;
}

template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void kp_pairs_main(PairsParams p) {
  extern __shared__ __align__(16) unsigned char smem[];
  const LdsLayout L = lds_layout(p.nrec, p.W, p.R);
  uint2* rec = reinterpret_cast<uint2*>(smem + L.rec);
  uint32_t* recw = reinterpret_cast<uint32_t*>(smem + L.rec);  // word 2p = clock, 2p+1 = metadata
  uint32_t* tmp = reinterpret_cast<uint32_t*>(smem + L.tmp);
  uint32_t* sV = reinterpret_cast<uint32_t*>(smem + L.v);
  uint32_t* sFirst = reinterpret_cast<uint32_t*>(smem + L.first);

  const uint32_t tid = threadIdx.x, lane = tid & 63u, hw = tid >> 6;
  const uint32_t W = p.W, R = p.R, cap = p.cap, nrec = p.nrec;
  const uint32_t capm = cap - 1, cl2 = p.cap_log2;
  const uint32_t Rpad = (R + 3u) & ~3u, nwords = Rpad >> 2;
  const unsigned long long lt_mask = (1ull << lane) - 1ull;

  // the padding entries of the count array are part of the output: zero
  if (blockIdx.x == 0 && tid < ((0u - p.n_wg * W) & 3u)) p.count[(size_t)p.n_wg * W + tid] = 0u;

  uint32_t iter = 0;
  for (uint32_t wg = blockIdx.x; wg < p.n_wg; wg += gridDim.x, ++iter) {
    const uint32_t* wh = p.wg_hdrs + (size_t)32 * wg;
    // a staged word counts only if it carries the generation of this pass, so the staging area
    // is cleared on the first pass and when the 16-bit generation wraps, not for every workgroup
    const uint32_t gen = 1u + iter % 0xFFFFu;
    const uint32_t live_tag = (gen << 16) | kMValid, live_mask = 0xFFFF0000u | kMValid;
    auto is_live = [&](uint32_t m) { return (m & live_mask) == live_tag; };
    if (tid < W) {
      const uint32_t T = wh[8 + tid];
      const uint32_t V = T < cap ? T : cap;
      sV[tid] = V;
      sFirst[tid] = p.flush ? 0u : T - V;
    }
    if (tid >= 64 && tid < 64 + T_COUNT) tmp[tid - 64] = 0;
    if (gen == 1u) {
      u32x4* z = reinterpret_cast<u32x4*>(rec);
      for (uint32_t i = tid; i < nrec / 2; i += BLOCK) z[i] = u32x4{0u, 0u, 0u, 0u};
    }
    __syncthreads();
    // ---- load and scatter by rank -------------------------------------------------------------
    {
      const u32x4* recs = p.records + (size_t)wg * (nrec / 2);
      const uint32_t n16 = nrec / 2;  // 16-byte units, two records each
      uint32_t c_field = 0;
      for (uint32_t i0 = tid; i0 < n16; i0 += 4 * BLOCK) {
        u32x4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const uint32_t i = i0 + u * BLOCK;
          v[u] = __builtin_nontemporal_load(recs + (i < n16 ? i : i0));
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const uint32_t i = i0 + u * BLOCK;
          const bool live = i < n16;
          const uint32_t f0 = 2 * (live ? i : i0);
          const uint32_t w = f0 >> cl2;
          const uint32_t V = live ? sV[w] : 0u, first = sFirst[w];
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            const uint32_t tag = h ? v[u].z : v[u].x, pay = h ? v[u].w : v[u].y;
            const uint32_t s = (f0 + h) & capm;
            const uint32_t k = ((tag & kSeqMask) - first) & kSeqMask;
            const uint32_t region = (tag >> 24) & 0x7Fu;
            const bool good = s < V && k < V && ((tag >> 20) & 0xFu) == w && region < R;
            c_field += good ? 1u : 0u;
            if (good) rec[(w << cl2) + k] = make_uint2(pay, region | ((tag >> 31) ? kMEnd : 0u) | live_tag);
          }
        }
      }
      c_field = wave_sum(c_field);
      if (lane == 0 && c_field) atomicAdd(&tmp[T_FIELDVALID], c_field);
    }
    __syncthreads();
    // ---- a duplicated seq leaves fewer occupied ranks than valid records ---------------------------
    {
      uint32_t occ = 0;
      for (uint32_t q = tid; q < nrec; q += BLOCK) occ += is_live(recw[2 * q + 1]) ? 1u : 0u;
      occ = wave_sum(occ);
      if (lane == 0 && occ) atomicAdd(&tmp[T_OCCUPIED], occ);
    }
    __syncthreads();
    if (tmp[T_OCCUPIED] != tmp[T_FIELDVALID]) {
      // Rare: some seq occurs twice.  The later slot must win, so redo this workgroup's scatter
      // in slot order, one thread per wave.
      __syncthreads();
      for (uint32_t i = tid; i < nrec; i += BLOCK) recw[2 * i + 1] = 0;
      __syncthreads();
      if (tid < W) {
        const uint32_t w = tid, V = sV[w], first = sFirst[w];
        const uint32_t* seg = reinterpret_cast<const uint32_t*>(p.records) + ((size_t)wg * nrec + (size_t)w * cap) * 2;
        for (uint32_t s = 0; s < V; ++s) {
          const uint32_t tag = seg[2 * s];
          const uint32_t k = ((tag & kSeqMask) - first) & kSeqMask, region = (tag >> 24) & 0x7Fu;
          if (k >= V || ((tag >> 20) & 0xFu) != w || region >= R) continue;
          rec[w * cap + k] = make_uint2(seg[2 * s + 1], region | ((tag >> 31) ? kMEnd : 0u) | live_tag);
        }
      }
      __syncthreads();
    }
    // ---- walk: hardware wave w pairs recorded wave w and emits its rows --------------------------------
    if (hw < W) {
      const uint32_t w = hw, wofs = w << cl2, V = sV[w];
      uint32_t base_lo = 0u, base_hi = 0u;  // pairs seen so far: lane r for region r / region 64 + r
      u32x4* my_rows = p.rows + ((size_t)wg * W + w) * (cap / 2);
      uint32_t n_rows = 0;
      uint32_t cm[4] = {0u, 0u, 0u, 0u};  // metadata of the last four ranks of the previous round
      uint2 r_next = rec[wofs + (lane < V ? lane : 0u)];  // one round ahead, to hide the LDS latency
      for (uint32_t kb = 0; kb < V; kb += 64) {
        const uint32_t k = kb + lane;
        const bool in = k < V;
        const uint32_t q0 = wofs + (in ? k : V - 1);
        const uint2 r0 = r_next;
        {
          const uint32_t kn = k + 64;
          r_next = rec[wofs + (kn < V ? kn : 0u)];
        }
        const bool valid = in && is_live(r0.y);
        const uint32_t m0 = valid ? r0.y : 0u, t0 = r0.x;
        const uint32_t m1 = wave_shr1(m0, cm[0]);
        const uint32_t m2 = wave_shr1(m1, cm[1]);
        const uint32_t m3 = wave_shr1(m2, cm[2]);
        const uint32_t m4 = wave_shr1(m3, cm[3]);
#pragma unroll
        for (int j = 0; j < 4; ++j) cm[j] = (uint32_t)__builtin_amdgcn_readlane((int)m0, 63 - j);
        const uint32_t region = m0 & kMRegion;
        const bool is_end = (m0 & kMEnd) != 0u;  // m0 is 0 for a rank that holds no record
        const uint32_t want = kMValid | region, sel = kMValid | kMRegion;
        const bool h1 = (m1 & sel) == want, h2 = (m2 & sel) == want, h3 = (m3 & sel) == want, h4 = (m4 & sel) == want;
        bool have = h1 || h2 || h3 || h4;  // nearest earlier record of the same region
        uint32_t pm = h1 ? m1 : (h2 ? m2 : (h3 ? m3 : m4));
        uint32_t pq = q0 - (h1 ? 1u : (h2 ? 2u : (h3 ? 3u : 4u)));
        if (is_end && !have && k > 4) {  // slow path: walk further back
          for (uint32_t kk = k - 4; kk-- > 0;) {
            const uint32_t mq = recw[2 * (wofs + kk) + 1];
            if (is_live(mq) && (mq & kMRegion) == region) { have = true; pm = mq; pq = wofs + kk; break; }
          }
        }
        const bool paired = is_end && have && !(pm & kMEnd);
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
      if (lane == 0) p.count[(size_t)wg * W + w] = n_rows;
    }
    __syncthreads();
  }
}

struct LaunchCache { int dev = -1; uint32_t lds = 0; uint32_t max_grid = 0; };

template <int BLOCK>
kp_status launch_pairs(const PairsParams& p, uint32_t lds_bytes, hipStream_t s) {
  auto kern = kp_pairs_main<BLOCK>;
  static thread_local LaunchCache cache;
  int dev = 0;
  KP_HIP_TRY(hipGetDevice(&dev));
  if (cache.dev != dev || cache.lds != lds_bytes) {
    KP_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes));
    int per_cu = 0, cus = 0;
    KP_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, BLOCK, lds_bytes));
    if (per_cu < 1) return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "timeline kernel does not fit one CU (LDS %u B)", lds_bytes);
    KP_HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    cache.dev = dev; cache.lds = lds_bytes; cache.max_grid = (uint32_t)per_cu * (uint32_t)cus;
  }
  uint32_t grid = cache.max_grid;
  if (grid > p.n_wg) grid = p.n_wg;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(BLOCK), lds_bytes, s, p);
  KP_HIP_TRY(hipGetLastError());
  return KP_OK;
}

size_t count_bytes(size_t n_seg) { return ((n_seg + 3) / 4) * 16; }

kp_status pairs_impl(const void* raw, size_t n, const kp_trace_hdr& h, void* out_pairs, hipStream_t s) {
  if (h.magic != KP_TRACE_MAGIC || h.version != KP_TRACE_VERSION)
    return kp::fail(KP_ERR_BAD_TRACE, "trace header: bad magic/version (%08x, %u)", h.magic, h.version);
  if (h.waves_per_wg < 1 || h.waves_per_wg > KP_MAX_WAVES || h.n_regions < 1 || h.n_regions > 128 ||
      !kp::is_pow2(h.cap_wave) || h.cap_wave < 2)
    return kp::fail(KP_ERR_BAD_TRACE, "trace header: waves=%u regions=%u cap_wave=%u", h.waves_per_wg, h.n_regions, h.cap_wave);
  if ((size_t)h.n_wg * h.waves_per_wg * h.cap_wave != n)
    return kp::fail(KP_ERR_BAD_TRACE, "trace header describes %zu record slots, caller passed %zu",
                    (size_t)h.n_wg * h.waves_per_wg * h.cap_wave, n);
  if ((h.flags & ~KP_FLAG_FLUSH) != 0) return kp::fail(KP_ERR_BAD_TRACE, "trace header: unknown flags %x", h.flags);
  const uint32_t W = h.waves_per_wg, R = h.n_regions, cap = h.cap_wave, nrec = W * cap;
  if (nrec > kMaxRecPerWg)
    return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "%u records per workgroup exceed the LDS staging limit %u", nrec, kMaxRecPerWg);
  if (((uintptr_t)raw & 15u) || ((uintptr_t)out_pairs & 15u))
    return kp::fail(KP_ERR_INVALID_ARG, "raw and out_pairs must be 16-byte aligned");
  const LdsLayout L = lds_layout(nrec, W, R);
  if (L.total > kMaxLds)
    return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "timeline kernel needs %u B of LDS for this geometry (limit %u)", L.total, kMaxLds);
  if (h.n_wg == 0) return KP_OK;

  const uint8_t* base = static_cast<const uint8_t*>(raw);
  uint8_t* out = static_cast<uint8_t*>(out_pairs);
  const size_t n_seg = (size_t)h.n_wg * W;
  PairsParams p;
  p.wg_hdrs = reinterpret_cast<const uint32_t*>(base + sizeof(kp_trace_hdr));
  p.records = reinterpret_cast<const u32x4*>(base + sizeof(kp_trace_hdr) + sizeof(kp_wg_hdr) * (size_t)h.n_wg);
  p.count = reinterpret_cast<uint32_t*>(out);
  p.rows = reinterpret_cast<u32x4*>(out + count_bytes(n_seg));
  p.n_wg = h.n_wg; p.W = W; p.R = R; p.cap = cap;
  p.cap_log2 = 0; while ((1u << p.cap_log2) < cap) ++p.cap_log2;
  p.rec_cost = h.rec_cost; p.flush = h.flags & KP_FLAG_FLUSH; p.nrec = nrec;
  // one hardware wave per recorded wave, and enough threads to stage the records quickly
  const int block = (W > 8 || nrec >= 8192) ? 1024 : ((W > 4 || nrec >= 2048) ? 512 : 256);
  return block == 1024 ? launch_pairs<1024>(p, L.total, s)
       : block == 512  ? launch_pairs<512>(p, L.total, s)
                       : launch_pairs<256>(p, L.total, s);
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

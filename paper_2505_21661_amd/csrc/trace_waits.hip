// GPU replay of the waits behind asynchronous operations (kp_trace_waits).
//
// Sec. 4.3 (trace replay, asynchronous instructions): with a START before the asynchronous launch
// (clock CLK0), an END right before the barrier that waits for it (CLK1) and a second START right
// after the barrier (CLK2), the wait is T_wait = CLK2 - CLK1 with the records' own cost cancelled,
// and the figure holds only while what is left of the operation at the barrier outlasts one record.
// This kernel finds every END whose successor in its wave is a START and reduces
//   gap   = (u32)(CLK2 - CLK1)                      per (workgroup, wave, region of the END),
//   gap <= rec_cost                                 counted as "uncovered",
//   whole = (u32)(CLK2 - CLK0) - rec_cost, >= 0     when the END is paired with a START at CLK0.
//
// One decoder workgroup stages one recorded workgroup in LDS, ordered by rank; the hardware waves
// share out the recorded waves in runs of consecutive ranks and walk them 64 ranks per round.  A
// START takes what it needs to know about the rank below -- metadata, clock, whether that END is
// paired and with which clock -- from the lane below through DPP wave shifts (the last lane of the
// previous round stands in for lane 0); only when that rank is empty does it walk back through LDS.  Sums, extrema and the log2 histogram go to LDS
// atomics; totals live in LDS across the recorded workgroups of a persistent decoder workgroup.
#include "kp_stage.h"

namespace {

using namespace kp_stage;

struct WaitsLayout {  // offsets in u64 words
  size_t hist, cnt, sum, min, max, unc, acnt, asum, per, total;
};
__host__ __device__ inline WaitsLayout waits_layout(uint32_t n_wg, uint32_t W, uint32_t R) {
  WaitsLayout l;
  l.hist = 16;
  l.cnt = l.hist + (size_t)64 * R;
  l.sum = l.cnt + R; l.min = l.sum + R; l.max = l.min + R;
  l.unc = l.max + R; l.acnt = l.unc + R; l.asum = l.acnt + R;
  l.per = l.asum + R;
  l.total = l.per + (size_t)2 * n_wg * W * R;
  return l;
}
enum { H_WAITS = 0, H_UNCOVERED, H_ASYNC, H_NWG = 8, H_WAVES, H_NREG, H_CAP, H_COST };

constexpr uint32_t kHistStride = 65;  // regions that hit the same bin land in different LDS banks

struct WaitsLds {
  uint32_t hist, pw_pack, pw_max, pw_min, reg_sum, reg_cnt, reg_max, reg_min, unc, acnt, asum, total;
};
__host__ __device__ inline WaitsLds waits_lds(uint32_t from, uint32_t W, uint32_t R) {
  WaitsLds l;
  uint32_t o = from;
  l.hist = o; o = align16(o + R * kHistStride * 4);
  l.pw_pack = o; o = align16(o + W * R * 8);
  l.pw_max = o; o = align16(o + W * R * 4);
  l.pw_min = o; o = align16(o + W * R * 4);
  l.reg_sum = o; o = align16(o + R * 8);
  l.reg_cnt = o; o = align16(o + R * 8);
  l.reg_max = o; o = align16(o + R * 4);
  l.reg_min = o; o = align16(o + R * 4);
  l.unc = o; o = align16(o + R * 8);
  l.acnt = o; o = align16(o + R * 8);
  l.asum = o; o = align16(o + R * 8);
  l.total = o;
  return l;
}

// init: clear the totals, set min to all-ones, echo the geometry.
__global__ void kp_waits_init(uint64_t* out, uint32_t n_wg, uint32_t W, uint32_t R, uint32_t cap, uint32_t rec_cost) {
  const WaitsLayout l = waits_layout(n_wg, W, R);
  for (size_t i = threadIdx.x + (size_t)blockIdx.x * blockDim.x; i < l.per; i += (size_t)blockDim.x * gridDim.x) {
    uint64_t v = (i >= l.min && i < l.max) ? ~0ull : 0ull;
    if (i == H_NWG) v = n_wg;
    if (i == H_WAVES) v = W;
    if (i == H_NREG) v = R;
    if (i == H_CAP) v = cap;
    if (i == H_COST) v = rec_cost;
    out[i] = v;
  }
}

// finalize: the three header counts are the sums of the per-region counts.
__global__ void kp_waits_finalize(uint64_t* out, uint32_t n_wg, uint32_t W, uint32_t R) {
  const WaitsLayout l = waits_layout(n_wg, W, R);
  if (threadIdx.x < 3) {
    const size_t from = threadIdx.x == 0 ? l.cnt : (threadIdx.x == 1 ? l.unc : l.acnt);
    uint64_t s = 0;
    for (uint32_t r = 0; r < R; ++r) s += out[from + r];
    out[threadIdx.x] = s;
  }
}

template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void kp_waits_main(Trace p, uint64_t* out_words, uint32_t split_log2) {
  extern __shared__ __align__(16) unsigned char smem[];
  const Lds L = lds_layout(p.nrec);
  const WaitsLds X = waits_lds(L.end, p.W, p.R);
  const uint2* rec = reinterpret_cast<const uint2*>(smem + L.rec);
  const uint32_t* sV = reinterpret_cast<const uint32_t*>(smem + L.v);
  uint32_t* hist = reinterpret_cast<uint32_t*>(smem + X.hist);
  unsigned long long* pw_pack = reinterpret_cast<unsigned long long*>(smem + X.pw_pack);
  uint32_t* pw_max = reinterpret_cast<uint32_t*>(smem + X.pw_max);
  uint32_t* pw_min = reinterpret_cast<uint32_t*>(smem + X.pw_min);
  unsigned long long* reg_sum = reinterpret_cast<unsigned long long*>(smem + X.reg_sum);
  unsigned long long* reg_cnt = reinterpret_cast<unsigned long long*>(smem + X.reg_cnt);
  uint32_t* reg_max = reinterpret_cast<uint32_t*>(smem + X.reg_max);
  uint32_t* reg_min = reinterpret_cast<uint32_t*>(smem + X.reg_min);
  unsigned long long* unc = reinterpret_cast<unsigned long long*>(smem + X.unc);
  unsigned long long* acnt = reinterpret_cast<unsigned long long*>(smem + X.acnt);
  unsigned long long* asum = reinterpret_cast<unsigned long long*>(smem + X.asum);

  const uint32_t tid = threadIdx.x, lane = tid & 63u, hw = tid >> 6;
  const uint32_t W = p.W, R = p.R, cl2 = p.cap_log2;
  const WaitsLayout SL = waits_layout(p.n_wg, W, R);

  for (uint32_t i = tid; i < R * kHistStride; i += BLOCK) hist[i] = 0;
  for (uint32_t i = tid; i < W * R; i += BLOCK) { pw_pack[i] = 0; pw_max[i] = 0; pw_min[i] = 0xFFFFFFFFu; }
  for (uint32_t i = tid; i < R; i += BLOCK) {
    reg_sum[i] = 0; reg_cnt[i] = 0; reg_max[i] = 0; reg_min[i] = 0xFFFFFFFFu;
    unc[i] = 0; acnt[i] = 0; asum[i] = 0;
  }
  // stage_workgroup's first barrier orders these stores before any use

  uint32_t iter = 0;
  for (uint32_t wg = blockIdx.x; wg < p.n_wg; wg += gridDim.x, ++iter) {
    stage_workgroup<BLOCK>(p, smem, L, wg, iter);
    const uint32_t live_tag = live_tag_of(iter);
    // ---- walk: 2^split_log2 hardware waves share one recorded wave, each a run of consecutive ranks ----
    // Nothing but the look-back crosses from one run into the next, and the staged records of the
    // earlier run are all in LDS, so the runs are independent.
    if (hw < (W << split_log2)) {
      const uint32_t w = hw >> split_log2, part = hw & ((1u << split_log2) - 1u);
      const uint32_t wofs = w << cl2, V = sV[w];
      const uint32_t plen = p.cap >> split_log2;
      const uint32_t k0 = part * plen, k1 = V < k0 + plen ? V : k0 + plen;
      uint32_t cm[4];                       // metadata of the four ranks below the round
      uint32_t ct = 0u, cpaired = 0u, cpt = 0u;  // clock / paired flag / START clock of the rank just below
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint2 r = rec[wofs + (k0 > (uint32_t)j ? k0 - 1u - j : 0u)];
        cm[j] = (k0 > (uint32_t)j && is_live(r.y, live_tag)) ? r.y : 0u;
        if (j == 0) ct = r.x;
      }
      if (cm[0] & kMEnd) {  // a run that starts right above an END: is that END paired? (uniform)
        for (uint32_t jj = k0 - 1u; jj-- > 0;) {
          const uint2 rj = rec[wofs + jj];
          if (!is_live(rj.y, live_tag) || ((rj.y ^ cm[0]) & kMRegion)) continue;
          if (!(rj.y & kMEnd)) { cpaired = 1u; cpt = rj.x; }
          break;
        }
      }
      uint2 r_next = rec[wofs + (k0 + lane < k1 ? k0 + lane : 0u)];  // one round ahead, to hide the LDS latency
      for (uint32_t kb = k0; kb < k1; kb += 64) {
        const uint32_t k = kb + lane;
        const bool in = k < k1;
        const uint32_t q0 = wofs + (in ? k : k1 - 1);
        const uint2 r0 = r_next;
        {
          const uint32_t kn = k + 64;
          r_next = rec[wofs + (kn < k1 ? kn : 0u)];
        }
        const bool valid = in && is_live(r0.y, live_tag);
        const uint32_t m0 = valid ? r0.y : 0u, t0 = r0.x;
        const uint32_t m1 = wave_shr1(m0, cm[0]);
        const uint32_t m2 = wave_shr1(m1, cm[1]);
        const uint32_t m3 = wave_shr1(m2, cm[2]);
        const uint32_t m4 = wave_shr1(m3, cm[3]);
        const uint32_t t1 = wave_shr1(t0, ct);
#pragma unroll
        for (int j = 0; j < 4; ++j) cm[j] = (uint32_t)__builtin_amdgcn_readlane((int)m0, 63 - j);
        ct = (uint32_t)__builtin_amdgcn_readlane((int)t0, 63);
        // ---- an END is paired iff the nearest earlier record of its region is a START ------------------
        const uint32_t region = m0 & kMRegion;
        const bool is_end = (m0 & kMEnd) != 0u;  // m0 is 0 for a rank that holds no record
        const uint32_t want = kMValid | region, sel = kMValid | kMRegion;
        const bool h1 = (m1 & sel) == want, h2 = (m2 & sel) == want, h3 = (m3 & sel) == want, h4 = (m4 & sel) == want;
        bool have = h1 || h2 || h3 || h4;
        uint32_t pm = h1 ? m1 : (h2 ? m2 : (h3 ? m3 : m4));
        uint32_t pq = q0 - (h1 ? 1u : (h2 ? 2u : (h3 ? 3u : 4u)));
        if (is_end && !have && k > 4) {  // slow path: walk further back
          for (uint32_t kk = k - 4; kk-- > 0;) {
            const uint32_t mq = rec[wofs + kk].y;
            if (is_live(mq, live_tag) && (mq & kMRegion) == region) { have = true; pm = mq; pq = wofs + kk; break; }
          }
        }
        const bool paired = is_end && have && !(pm & kMEnd);
        const uint32_t pt = rec[paired ? pq : wofs].x;  // CLK0 of a paired END
        // ---- a START looks at the record below it -------------------------------------------------------
        uint32_t below_m = m1, below_t = t1;
        uint32_t below_paired = wave_shr1(paired ? 1u : 0u, cpaired);
        uint32_t below_pt = wave_shr1(pt, cpt);
        cpaired = (uint32_t)__builtin_amdgcn_readlane((int)(paired ? 1u : 0u), 63);
        cpt = (uint32_t)__builtin_amdgcn_readlane((int)pt, 63);
        const bool is_start = valid && !is_end;
        if (is_start && k > 0 && !(m1 & kMValid)) {  // the rank below is empty: find the record below it
          below_m = 0u;
          for (uint32_t kk = k - 1; kk-- > 0;) {
            const uint2 rq = rec[wofs + kk];
            if (!is_live(rq.y, live_tag)) continue;
            below_m = rq.y; below_t = rq.x; below_paired = 0u;
            if (rq.y & kMEnd) {  // is that END paired?
              for (uint32_t jj = kk; jj-- > 0;) {
                const uint2 rj = rec[wofs + jj];
                if (!is_live(rj.y, live_tag) || ((rj.y ^ rq.y) & kMRegion)) continue;
                if (!(rj.y & kMEnd)) { below_paired = 1u; below_pt = rj.x; }
                break;
              }
            }
            break;
          }
        }
        if (is_start && (below_m & kMEnd)) {  // below_m is 0 when there is no record below
          const uint32_t a = below_m & kMRegion;
          const uint32_t gap = t0 - below_t;
          const uint32_t e = w * R + a;
          atomicAdd(&pw_pack[e], (1ull << 46) | (unsigned long long)gap);
          atomicMax(&pw_max[e], gap);
          atomicMin(&pw_min[e], gap);
          atomicAdd(&hist[a * kHistStride + (gap ? 31 - __clz(gap) : 0)], 1u);
          if (gap <= p.rec_cost) atomicAdd(&unc[a], 1ull);
          if (below_paired) {
            const uint32_t whole = t0 - below_pt;
            atomicAdd(&acnt[a], 1ull);
            atomicAdd(&asum[a], (unsigned long long)(whole > p.rec_cost ? whole - p.rec_cost : 0u));
          }
        }
      }
    }
    __syncthreads();
    // ---- per-(workgroup, wave, region) output, fold into running totals ------------------------------------
    for (uint32_t e = tid; e < W * R; e += BLOCK) {
      const unsigned long long pk = pw_pack[e];
      const uint32_t n = (uint32_t)(pk >> 46);
      const unsigned long long s = pk & ((1ull << 46) - 1);
      const uint32_t mx = pw_max[e], mn = pw_min[e];
      uint64_t* dst = out_words + SL.per + ((size_t)wg * W * R + e) * 2;
      dst[0] = s;
      dst[1] = (uint64_t)n | ((uint64_t)mx << 32);
      if (n) {
        const uint32_t r = e % R;
        atomicAdd(&reg_sum[r], s);
        atomicAdd(&reg_cnt[r], (unsigned long long)n);
        atomicMax(&reg_max[r], mx);
        atomicMin(&reg_min[r], mn);
      }
      pw_pack[e] = 0; pw_max[e] = 0; pw_min[e] = 0xFFFFFFFFu;
    }
    __syncthreads();
  }

  // ---- flush this decoder workgroup's totals --------------------------------------------------------
  unsigned long long* out = reinterpret_cast<unsigned long long*>(out_words);
  for (uint32_t i = tid; i < R * 64; i += BLOCK) {
    const uint32_t v = hist[(i >> 6) * kHistStride + (i & 63u)];
    if (v) atomicAdd(&out[SL.hist + i], (unsigned long long)v);
  }
  for (uint32_t r = tid; r < R; r += BLOCK) {
    if (reg_cnt[r]) {
      atomicAdd(&out[SL.cnt + r], reg_cnt[r]);
      atomicAdd(&out[SL.sum + r], reg_sum[r]);
      atomicMax(&out[SL.max + r], (unsigned long long)reg_max[r]);
      atomicMin(&out[SL.min + r], (unsigned long long)reg_min[r]);
      if (unc[r]) atomicAdd(&out[SL.unc + r], unc[r]);
      if (acnt[r]) atomicAdd(&out[SL.acnt + r], acnt[r]);
      if (asum[r]) atomicAdd(&out[SL.asum + r], asum[r]);
    }
  }
}

template <int BLOCK>
kp_status launch_waits(const Trace& p, uint64_t* out, uint32_t lds_bytes, hipStream_t s) {
  // hardware waves per recorded wave: as many as the block has, while a run keeps at least 64 ranks
  uint32_t split_log2 = 0;
  while ((p.W << (split_log2 + 1)) <= (uint32_t)BLOCK / 64u && (p.cap >> (split_log2 + 1)) >= 64u) ++split_log2;
  auto kern = kp_waits_main<BLOCK>;
  static thread_local LaunchCache cache;
  uint32_t grid = 0;
  const kp_status st = resident_grid(kern, BLOCK, lds_bytes, &cache, &grid);
  if (st != KP_OK) return st;
  if (grid > p.n_wg) grid = p.n_wg;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(BLOCK), lds_bytes, s, p, out, split_log2);
  KP_HIP_TRY(hipGetLastError());
  return KP_OK;
}

kp_status waits_impl(const void* raw, size_t n, const kp_trace_hdr& h, void* out_waits, hipStream_t s) {
  Trace p;
  const kp_status st = trace_from_header(raw, n, h, out_waits, &p);
  if (st != KP_OK) return st;
  const WaitsLds X = waits_lds(lds_layout(p.nrec).end, p.W, p.R);
  if (X.total > kMaxLds)
    return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "wait replay needs %u B of LDS for this geometry (limit %u)", X.total, kMaxLds);

  uint64_t* out = static_cast<uint64_t*>(out_waits);
  const WaitsLayout SL = waits_layout(p.n_wg, p.W, p.R);
  int init_blocks = (int)((SL.per + 255) / 256);
  if (init_blocks > 64) init_blocks = 64;
  hipLaunchKernelGGL(kp_waits_init, dim3(init_blocks), dim3(256), 0, s, out, p.n_wg, p.W, p.R, p.cap, p.rec_cost);
  KP_HIP_TRY(hipGetLastError());
  if (p.n_wg > 0) {
    const int block = block_threads(p.W, p.nrec);
    const kp_status ls = block == 1024 ? launch_waits<1024>(p, out, X.total, s)
                       : block == 512  ? launch_waits<512>(p, out, X.total, s)
                                       : launch_waits<256>(p, out, X.total, s);
    if (ls != KP_OK) return ls;
  }
  hipLaunchKernelGGL(kp_waits_finalize, dim3(1), dim3(64), 0, s, out, p.n_wg, p.W, p.R);
  KP_HIP_TRY(hipGetLastError());
  return KP_OK;
}

}  // namespace

extern "C" size_t kp_waits_bytes(int n_wg, int waves_per_wg, int n_regions) {
  if (n_wg < 0 || waves_per_wg < 1 || waves_per_wg > KP_MAX_WAVES || n_regions < 1 || n_regions > 128) return 0;
  return waits_layout((uint32_t)n_wg, (uint32_t)waves_per_wg, (uint32_t)n_regions).total * 8;
}

extern "C" kp_status kp_trace_waits_hdr(const void* raw, size_t n, const kp_trace_hdr* hdr_host,
                                        void* out_waits, void* stream) {
  kp::clear_error();
  if (!raw || !hdr_host || !out_waits) return kp::fail(KP_ERR_INVALID_ARG, "NULL argument");
  return waits_impl(raw, n, *hdr_host, out_waits, static_cast<hipStream_t>(stream));
}

extern "C" kp_status kp_trace_waits(const void* raw, size_t n, void* out_waits, void* stream) {
  kp::clear_error();
  if (!raw || !out_waits) return kp::fail(KP_ERR_INVALID_ARG, "NULL argument");
  kp_trace_hdr h;
  hipStream_t s = static_cast<hipStream_t>(stream);
  KP_HIP_TRY(hipMemcpyAsync(&h, raw, sizeof h, hipMemcpyDeviceToHost, s));
  KP_HIP_TRY(hipStreamSynchronize(s));
  return waits_impl(raw, n, h, out_waits, s);
}

// GPU trace decode / pair / reduce (kp_trace_reduce).
//
// The paper stores START/END records unpaired, per warp, in a ring whose tail survives, and
// aligns them at "trace replay" on the host (Sec. 4.2 "SM-level Data Layout", "Shared Memory
// Circular Buffer"; Sec. 4.3).  Here replay runs on the GPU: one decoder workgroup stages one
// recorded workgroup's records in LDS and
//   A  scatters every record to its rank (seq - first surviving seq), which undoes ring
//      rotation and out-of-order flushes in O(1) per record,
//   B  pairs each START with the next record of the same (wave, region) when that is an END,
//      takes d = (u32)(ts_end - ts_start) minus the constant record cost (Sec. 4.3), and
//      accumulates the per-(wave, region) sums and the log2 histogram with LDS atomics,
//   C  XOR-scans the paired region bits of each wave into an "open regions" mask per position,
//   D  builds a coarse time -> position table per wave,
//   E  looks every paired event up in the other waves to find the set of regions active in the
//      workgroup at that instant, and, when the event switches its region on or off for the
//      whole workgroup, adds -t / +t to the region-pair accumulators (the integral of
//      A_a(t)*A_b(t) collapses to a signed sum over its switching times),
//   F  writes the per-(workgroup, wave, region) results and folds them into running totals.
// Decoder workgroups are persistent; totals live in LDS and reach HBM once per workgroup.
#include "kp_common.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr uint32_t kSeqMask = 0xFFFFFu;
constexpr uint32_t kMRegion = 0x1Fu, kMEnd = 0x20u, kMValid = 0x40u, kMPaired = 0x80u;
constexpr uint32_t kMaxRecPerWg = 16384;
constexpr uint32_t kMaxLds = 160 * 1024;

// positions inside kp_stats_hdr, in u64 words
enum { H_SLOTS_VALID = 0, H_PAIRS, H_ORPHAN_START, H_ORPHAN_END, H_INVALID, H_DROPPED, H_DISORDER,
       H_SPAN_OVF, H_NONMONO, H_OVERLAP_WGS, H_STATUS, H_NWG, H_WAVES, H_NREG, H_CAP, H_RSVD };

// per-workgroup temporaries (u32 words in LDS)
enum { T_INVALID = 0, T_FIELDVALID, T_DISORDER, T_OCCUPIED, T_NONMONO, T_PAIRS, T_ORPH_S, T_ORPH_E,
       T_SPANOVF, T_SHIFT, T_COUNT };

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

struct DecodeParams {
  const uint32_t* wg_hdrs;  // 32 words per recorded workgroup
  const u32x4* records;     // two records per 16-byte load
  uint64_t* out;
  uint32_t n_wg, W, R, cap, cap_log2, rec_cost, flush;
  uint32_t nrec, span, ncell;
};

struct LdsLayout {  // byte offsets
  uint32_t ts, om, grid, hist, oacc, reg_sum, reg_max, reg_min, pw_pack, pw_max, pw_min, ctr, tmp,
      v, first, wave_tot, total;
};
__host__ __device__ inline uint32_t align16(uint32_t x) { return (x + 15u) & ~15u; }
__host__ __device__ inline LdsLayout lds_layout(uint32_t nrec, uint32_t W, uint32_t R, uint32_t ncell,
                                                uint32_t mask_bytes, uint32_t block) {
  LdsLayout l;
  uint32_t o = 0;
  l.ts = o; o = align16(o + nrec * 4);
  l.om = o; o = align16(o + nrec * mask_bytes);
  l.grid = o; o = align16(o + W * ncell * 2);
  l.hist = o; o = align16(o + R * 64 * 4);
  l.oacc = o; o = align16(o + R * R * 8);
  l.reg_sum = o; o = align16(o + R * 8);
  l.reg_max = o; o = align16(o + R * 4);
  l.reg_min = o; o = align16(o + R * 4);
  l.pw_pack = o; o = align16(o + W * R * 8);
  l.pw_max = o; o = align16(o + W * R * 4);
  l.pw_min = o; o = align16(o + W * R * 4);
  l.ctr = o; o = align16(o + 16 * 8);
  l.tmp = o; o = align16(o + T_COUNT * 4);
  l.v = o; o = align16(o + 16 * 4);
  l.first = o; o = align16(o + 16 * 4);
  l.wave_tot = o; o = align16(o + (block / 64) * 4);
  l.total = o;
  return l;
}

__device__ inline uint32_t wave_sum(uint32_t v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
  return v;
}

__device__ inline void add_tmp(uint32_t* tmp, int which, uint32_t v) {
  v = wave_sum(v);
  if ((threadIdx.x & 63) == 0 && v) atomicAdd(&tmp[which], v);
}

// ------------------------------------------------------------------------------------------
// init: clear the global totals, set min to all-ones, check the device header against the
// geometry the launch was sized for.
__global__ void kp_reduce_init(const uint32_t* trace_hdr, uint64_t* out, uint32_t n_wg, uint32_t W,
                               uint32_t R, uint32_t cap, uint32_t flags) {
  const StatsLayout l = stats_layout(n_wg, W, R);
  for (size_t i = threadIdx.x + (size_t)blockIdx.x * blockDim.x; i < l.per; i += (size_t)blockDim.x * gridDim.x)
    out[i] = (i >= l.min && i < l.max) ? ~0ull : 0ull;
  __syncthreads();
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    const bool ok = trace_hdr[0] == KP_TRACE_MAGIC && trace_hdr[1] == KP_TRACE_VERSION &&
                    trace_hdr[2] == n_wg && trace_hdr[3] == W && trace_hdr[4] == R &&
                    trace_hdr[5] == cap && trace_hdr[7] == flags;
    out[H_STATUS] = ok ? 0ull : 1ull;
    out[H_NWG] = n_wg; out[H_WAVES] = W; out[H_NREG] = R; out[H_CAP] = cap;
  }
}

// finalize: cnt from the histogram, O = Otmp + Otmp^T off the diagonal, U = diag, F = O/U.
__global__ void kp_reduce_finalize(uint64_t* out, uint32_t n_wg, uint32_t W, uint32_t R) {
  __shared__ uint64_t tmp[KP_MAX_REGIONS * KP_MAX_REGIONS];
  const StatsLayout l = stats_layout(n_wg, W, R);
  const uint32_t tid = threadIdx.x;
  for (uint32_t i = tid; i < R * R; i += blockDim.x) tmp[i] = out[l.F + i];  // staged Otmp
  if (tid < R) {
    uint64_t c = 0;
    for (int b = 0; b < 64; ++b) c += out[l.hist + (size_t)tid * 64 + b];
    out[l.cnt + tid] = c;
  }
  __syncthreads();
  for (uint32_t i = tid; i < R * R; i += blockDim.x) {
    const uint32_t a = i / R, b = i % R;
    const uint64_t u = tmp[a * R + a];
    const uint64_t o = (a == b) ? u : tmp[a * R + b] + tmp[b * R + a];
    out[l.O + i] = o;
    double f = u ? (double)o / (double)u : 0.0;
    reinterpret_cast<double*>(out)[l.F + i] = f;
    if (a == b) out[l.U + a] = u;
  }
}

// ------------------------------------------------------------------------------------------
// Overlap sweep.  One lane owns one time cell and merges the W per-wave record runs that fall
// into it in the total order (clock, wave, rank), carrying every wave's open-region mask.  When
// a paired record switches its region on or off for the whole workgroup (no other wave has it
// open), -t or +t goes to the region-pair accumulators of all regions active at that instant:
// the integral of A_a(t)*A_b(t) collapses to a signed sum over its switching times.
template <int WMAX, typename MaskT>
__device__ __forceinline__ void sweep_cells(const uint32_t* ts, const MaskT* om, const uint16_t* grid,
                                            const uint32_t* sV, unsigned long long* oacc, uint32_t W,
                                            uint32_t R, uint32_t cl2, uint32_t nrec, uint32_t ncell,
                                            uint32_t shift, uint32_t tid, uint32_t nthreads) {
  const uint32_t capm = (1u << cl2) - 1u;
  for (uint32_t c = tid; c < ncell; c += nthreads) {
    unsigned long long key[WMAX];  // (clock << 32) | position of each wave's next record; ~0 = none
    uint32_t msk[WMAX];            // regions each wave has open right now
    uint32_t n = 0;
#pragma unroll
    for (int w = 0; w < WMAX; ++w) {
      key[w] = ~0ull; msk[w] = 0u;
      if ((uint32_t)w < W) {
        const uint32_t V = sV[w];
        const uint32_t g0 = grid[w * ncell + c];
        const uint32_t g1r = grid[w * ncell + (c + 1 < ncell ? c + 1 : c)];
        const uint32_t g1 = (c + 1 < ncell) ? g1r : V;
        const uint32_t i0 = ((uint32_t)w << cl2) + g0;
        const uint32_t ic = i0 < nrec ? i0 : nrec - 1;
        const uint32_t m = om[ic], t = ts[ic];
        msk[w] = g0 < V ? m : 0u;
        key[w] = g0 < g1 ? (((unsigned long long)t << 32) | i0) : ~0ull;
        n += g1 - g0;
      }
    }
    for (; n; --n) {
      unsigned long long best = key[0];
#pragma unroll
      for (int w = 1; w < WMAX; ++w) best = key[w] < best ? key[w] : best;
      const uint32_t idx = (uint32_t)best, tt = (uint32_t)(best >> 32);
      const uint32_t b = idx >> cl2, pos = idx & capm, V = sV[b];
      const uint32_t inx = idx + 1 < nrec ? idx + 1 : idx;
      const uint32_t before = om[idx];
      const uint32_t nm = om[inx], nts = ts[inx];
      const bool more = pos + 1 < V;
      const uint32_t after = more ? nm : 0u;
      const uint32_t nc0 = nts >> shift;
      const uint32_t ncl = nc0 < ncell ? nc0 : ncell - 1;
      const unsigned long long nkey = (more && ncl == c) ? (((unsigned long long)nts << 32) | (idx + 1)) : ~0ull;
      uint32_t others = 0;
#pragma unroll
      for (int w = 0; w < WMAX; ++w) {
        const bool sel = (uint32_t)w == b;
        others |= sel ? 0u : msk[w];
        msk[w] = sel ? after : msk[w];
        key[w] = sel ? nkey : key[w];
      }
      const uint32_t x = before ^ after;  // the region bit this record toggles; 0 if unpaired
      if (x && !(others & x)) {
        const uint32_t a = __ffs(x) - 1;
        const unsigned long long val = (before & x) ? (unsigned long long)tt : (0ull - (unsigned long long)tt);
        atomicAdd(&oacc[a * R + a], val);
        uint32_t set = (others | before) & ~x;
        while (set) {
          const uint32_t bb = __ffs(set) - 1;
          set &= set - 1;
          atomicAdd(&oacc[a * R + bb], val);
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// Position p = wave*cap_wave + rank indexes the LDS arrays.  Every hardware wave of the decoder
// owns `span` consecutive positions and walks them 64 at a time, lane l taking position
// base + 64*round + l, so that neighbouring lanes touch neighbouring LDS words.
template <typename MaskT, int BLOCK>
__global__ __launch_bounds__(BLOCK) void kp_reduce_main(DecodeParams p) {
  extern __shared__ __align__(16) unsigned char smem[];
  const LdsLayout L = lds_layout(p.nrec, p.W, p.R, p.ncell, sizeof(MaskT), BLOCK);
  uint32_t* ts = reinterpret_cast<uint32_t*>(smem + L.ts);
  MaskT* om = reinterpret_cast<MaskT*>(smem + L.om);
  uint16_t* grid = reinterpret_cast<uint16_t*>(smem + L.grid);
  uint32_t* hist = reinterpret_cast<uint32_t*>(smem + L.hist);
  unsigned long long* oacc = reinterpret_cast<unsigned long long*>(smem + L.oacc);
  unsigned long long* reg_sum = reinterpret_cast<unsigned long long*>(smem + L.reg_sum);
  uint32_t* reg_max = reinterpret_cast<uint32_t*>(smem + L.reg_max);
  uint32_t* reg_min = reinterpret_cast<uint32_t*>(smem + L.reg_min);
  unsigned long long* pw_pack = reinterpret_cast<unsigned long long*>(smem + L.pw_pack);
  uint32_t* pw_max = reinterpret_cast<uint32_t*>(smem + L.pw_max);
  uint32_t* pw_min = reinterpret_cast<uint32_t*>(smem + L.pw_min);
  unsigned long long* ctr = reinterpret_cast<unsigned long long*>(smem + L.ctr);
  uint32_t* tmp = reinterpret_cast<uint32_t*>(smem + L.tmp);
  uint32_t* sV = reinterpret_cast<uint32_t*>(smem + L.v);
  uint32_t* sFirst = reinterpret_cast<uint32_t*>(smem + L.first);
  uint32_t* wave_tot = reinterpret_cast<uint32_t*>(smem + L.wave_tot);

  const uint32_t tid = threadIdx.x, lane = tid & 63u, hw = tid >> 6;
  const uint32_t W = p.W, R = p.R, cap = p.cap, nrec = p.nrec, ncell = p.ncell;
  const uint32_t capm = cap - 1, cl2 = p.cap_log2;
  const uint32_t span = p.span;              // positions per hardware wave, power of two >= 64
  const uint32_t pbase = hw * span;
  const uint32_t pend = pbase + span < nrec ? pbase + span : nrec;  // may be <= pbase: idle wave
  const StatsLayout SL = stats_layout(p.n_wg, W, R);
  if (p.out[H_STATUS] != 0) return;  // device header did not match the launch geometry

  for (uint32_t i = tid; i < R * 64; i += BLOCK) hist[i] = 0;
  for (uint32_t i = tid; i < R * R; i += BLOCK) oacc[i] = 0;
  for (uint32_t i = tid; i < R; i += BLOCK) { reg_sum[i] = 0; reg_max[i] = 0; reg_min[i] = 0xFFFFFFFFu; }
  for (uint32_t i = tid; i < W * R; i += BLOCK) { pw_pack[i] = 0; pw_max[i] = 0; pw_min[i] = 0xFFFFFFFFu; }
  if (tid < 16) ctr[tid] = 0;
  __syncthreads();

  for (uint32_t wg = blockIdx.x; wg < p.n_wg; wg += gridDim.x) {
    const uint32_t* wh = p.wg_hdrs + (size_t)32 * wg;
    // ---- workgroup header -----------------------------------------------------------------
    if (tid < W) {
      const uint32_t T = wh[8 + tid];
      const uint32_t V = T < cap ? T : cap;
      sV[tid] = V;
      sFirst[tid] = p.flush ? 0u : T - V;
      atomicAdd(&ctr[H_DROPPED], (unsigned long long)(T - V));
      atomicAdd(&ctr[H_SLOTS_VALID], (unsigned long long)V);
    }
    if (tid >= 64 && tid < 64 + T_COUNT) tmp[tid - 64] = 0;
    if (tid == 32) {
      const uint64_t tb = (uint64_t)wh[2] | ((uint64_t)wh[3] << 32);
      const uint64_t te = (uint64_t)wh[4] | ((uint64_t)wh[5] << 32);
      const uint64_t sp = te - tb;
      uint32_t shift = 0, ovf = 0;
      if (sp >> 32) ovf = 1; else while ((sp >> shift) >= ncell) ++shift;
      wave_tot[0] = ovf;  // parked here until tmp[] has been cleared
      wave_tot[1] = shift;
    }
    {
      u32x4* z = reinterpret_cast<u32x4*>(om);
      const uint32_t nz = (nrec * (uint32_t)sizeof(MaskT) + 15u) / 16u;
      for (uint32_t i = tid; i < nz; i += BLOCK) z[i] = u32x4{0u, 0u, 0u, 0u};
    }
    __syncthreads();
    // table default: "no record of this wave at or after this cell" (ncell is even)
    for (uint32_t i = tid; i < W * ncell / 2; i += BLOCK) {
      const uint32_t V = sV[(2 * i) / ncell];
      reinterpret_cast<uint32_t*>(grid)[i] = V | (V << 16);
    }
    if (tid == 0) { tmp[T_SPANOVF] = wave_tot[0]; tmp[T_SHIFT] = wave_tot[1]; }
    // ---- A: load and scatter by rank ------------------------------------------------------
    {
      const u32x4* rec = p.records + (size_t)wg * (nrec / 2);
      const uint32_t n16 = nrec / 2;  // 16-byte units, two records each
      uint32_t c_invalid = 0, c_field = 0, c_dis = 0;
      for (uint32_t i0 = tid; i0 < n16; i0 += 4 * BLOCK) {
        u32x4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const uint32_t i = i0 + u * BLOCK;
          v[u] = __builtin_nontemporal_load(rec + (i < n16 ? i : i0));
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
            const uint32_t seq = tag & kSeqMask;
            const uint32_t k = (seq - first) & kSeqMask;
            const uint32_t region = (tag >> 24) & 0x7Fu;
            const bool held = s < V;
            const bool good = held && k < V && ((tag >> 20) & 0xFu) == w && region < R;
            c_invalid += (held && !good) ? 1u : 0u;
            c_field += good ? 1u : 0u;
            c_dis += (good && s != (seq & capm)) ? 1u : 0u;
            if (good) {
              ts[(w << cl2) + k] = pay;
              om[(w << cl2) + k] = (MaskT)(region | ((tag >> 31) ? kMEnd : 0u) | kMValid);
            }
          }
        }
      }
      add_tmp(tmp, T_INVALID, c_invalid);
      add_tmp(tmp, T_FIELDVALID, c_field);
      add_tmp(tmp, T_DISORDER, c_dis);
    }
    __syncthreads();
    // ---- occupancy check: a duplicated seq leaves fewer occupied ranks than valid records ----
    {
      uint32_t occ = 0;
      for (uint32_t q = pbase + lane; q < pend; q += 64) occ += (om[q] & kMValid) ? 1u : 0u;
      add_tmp(tmp, T_OCCUPIED, occ);
    }
    __syncthreads();
    if (tmp[T_OCCUPIED] != tmp[T_FIELDVALID]) {
      // Rare: some seq occurs twice.  The later slot must win, so redo this workgroup's
      // scatter in slot order, one thread per wave.
      __syncthreads();
      for (uint32_t i = tid; i < nrec; i += BLOCK) om[i] = 0;
      if (tid == 0) { tmp[T_DISORDER] = 0; tmp[T_OCCUPIED] = 0; }
      __syncthreads();
      if (tid < W) {
        const uint32_t w = tid, V = sV[w], first = sFirst[w];
        const uint32_t* seg = reinterpret_cast<const uint32_t*>(p.records) + ((size_t)wg * nrec + (size_t)w * cap) * 2;
        for (uint32_t s = 0; s < V; ++s) {
          const uint32_t tag = seg[2 * s];
          const uint32_t seq = tag & kSeqMask, k = (seq - first) & kSeqMask, region = (tag >> 24) & 0x7Fu;
          if (k >= V || ((tag >> 20) & 0xFu) != w || region >= R) continue;
          ts[w * cap + k] = s;  // remember the winning slot for now
          om[w * cap + k] = (MaskT)(region | ((tag >> 31) ? kMEnd : 0u) | kMValid);
        }
        uint32_t dis = 0, occ = 0;
        for (uint32_t k = 0; k < V; ++k) {
          if (!(om[w * cap + k] & kMValid)) continue;
          const uint32_t s = ts[w * cap + k];
          dis += (s != ((seg[2 * s] & kSeqMask) & capm));
          ts[w * cap + k] = seg[2 * s + 1];
          ++occ;
        }
        atomicAdd(&tmp[T_DISORDER], dis);
        atomicAdd(&tmp[T_OCCUPIED], occ);
      }
      __syncthreads();
    }
    // ---- B: pairing, durations, per-(wave,region) statistics, monotonicity --------------------
    // An END is paired iff the nearest earlier record of its (wave, region) is a START; every
    // START that is not claimed this way is an orphan, so only ENDs have to search, and in
    // traces of real kernels the START sits a few ranks back.  The four ranks just below are
    // fetched unconditionally (clamped addresses); deeper searches are the rare slow path.
    {
      uint32_t c_nonmono = 0, c_pairs = 0, c_starts = 0, c_ends = 0;
      for (uint32_t qb = pbase; qb < pend; qb += 64) {
        const uint32_t q0 = (qb + lane < pend) ? qb + lane : pend - 1;
        const uint32_t m0 = (qb + lane < pend) ? (uint32_t)om[q0] : 0u;
        const uint32_t t0 = ts[q0];
        const uint32_t w = q0 >> cl2, wofs = w << cl2, k = q0 & capm;
        const bool valid = (m0 & kMValid) != 0;
        const uint32_t region = m0 & kMRegion;
        uint32_t mp[4], tp[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const uint32_t back = k > (uint32_t)j ? (uint32_t)j + 1u : 0u;  // 0: no such rank, reads itself
          const uint32_t mm = om[q0 - back];
          tp[j] = ts[q0 - back];
          mp[j] = back ? mm : 0u;
        }
        // previous record of this wave (ranks can be missing after invalid records)
        uint32_t tprev = t0;
        bool have_prev = false;
#pragma unroll
        for (int j = 3; j >= 0; --j) { const bool v = (mp[j] & kMValid) != 0; tprev = v ? tp[j] : tprev; have_prev |= v; }
        // nearest earlier record of the same region
        uint32_t pm = 0, pt = 0, pq = q0;
        bool have = false;
#pragma unroll
        for (int j = 3; j >= 0; --j) {
          const bool hit = (mp[j] & kMValid) && (mp[j] & kMRegion) == region;
          pm = hit ? mp[j] : pm; pt = hit ? tp[j] : pt; pq = hit ? q0 - 1 - j : pq; have |= hit;
        }
        const bool is_end = valid && (m0 & kMEnd);
        if (valid && k > 4 && (!have_prev || (is_end && !have))) {  // slow path: look further back
          for (uint32_t kk = k - 4; kk-- > 0;) {
            const uint32_t mq = om[wofs + kk];
            if (!(mq & kMValid)) continue;
            if (!have_prev) { have_prev = true; tprev = ts[wofs + kk]; }
            if (!is_end || have) break;
            if ((mq & kMRegion) == region) { have = true; pm = mq; pt = ts[wofs + kk]; pq = wofs + kk; break; }
          }
        }
        c_nonmono += (valid && t0 < tprev) ? 1u : 0u;
        c_starts += (valid && !(m0 & kMEnd)) ? 1u : 0u;
        c_ends += is_end ? 1u : 0u;
        if (is_end && have && !(pm & kMEnd)) {
          ++c_pairs;
          om[pq] = (MaskT)(pm | kMPaired);
          om[q0] = (MaskT)(m0 | kMPaired);
          const uint32_t d_raw = t0 - pt;
          const uint32_t d = d_raw > p.rec_cost ? d_raw - p.rec_cost : 0u;
          const uint32_t e = w * R + region;
          atomicAdd(&pw_pack[e], (1ull << 46) | (unsigned long long)d);
          atomicMax(&pw_max[e], d);
          atomicMin(&pw_min[e], d);
          atomicAdd(&hist[region * 64 + (d ? 31 - __clz(d) : 0)], 1u);
        }
      }
      add_tmp(tmp, T_NONMONO, c_nonmono);
      add_tmp(tmp, T_PAIRS, c_pairs);
      add_tmp(tmp, T_ORPH_S, c_starts);  // turned into orphan counts once T_PAIRS is complete
      add_tmp(tmp, T_ORPH_E, c_ends);
    }
    __syncthreads();
    // ---- C1: XOR of the paired region bits of every span ---------------------------------------
    {
      uint32_t x = 0;
      for (uint32_t q0 = pbase + lane; q0 < pend; q0 += 64) {
        const uint32_t m0 = om[q0];
        if (m0 & kMPaired) x ^= 1u << (m0 & kMRegion);
      }
#pragma unroll
      for (int d = 32; d >= 1; d >>= 1) x ^= __shfl_xor(x, d, 64);
      if (lane == 0) wave_tot[hw] = x;
    }
    __syncthreads();
    const uint32_t wg_invalid = tmp[T_INVALID] + (tmp[T_FIELDVALID] - tmp[T_OCCUPIED]);
    const bool eligible = !tmp[T_SPANOVF] && wg_invalid == 0 && tmp[T_NONMONO] == 0;

    if (eligible) {
      const uint32_t shift = tmp[T_SHIFT];
      // ---- C2: open-region mask before every position (exclusive XOR scan per wave) ------------
      // ---- D : coarse time -> position table ------------------------------------------------------
      {
        uint32_t carry = 0;
        if (span < cap) {  // this span continues a wave that started in an earlier span
          const uint32_t firsthw = ((pbase >> cl2) << cl2) / span;
          for (uint32_t i = firsthw; i < hw; ++i) carry ^= wave_tot[i];
        }
        for (uint32_t qb = pbase; qb < pend; qb += 64) {
          const uint32_t q0 = qb + lane;
          const bool in = q0 < pend;
          const uint32_t m0 = in ? (uint32_t)om[q0] : 0u;
          const uint32_t x = (m0 & kMPaired) ? (1u << (m0 & kMRegion)) : 0u;
          uint32_t v = x;
          if (cap >= 64) {
#pragma unroll
            for (uint32_t d = 1; d < 64; d <<= 1) { const uint32_t y = __shfl_up(v, d, 64); if (lane >= d) v ^= y; }
          } else {
            for (uint32_t d = 1; d < cap; d <<= 1) { const uint32_t y = __shfl_up(v, d, 64); if ((lane & capm) >= d) v ^= y; }
          }
          const uint32_t ex = v ^ x ^ carry;
          if (cap >= 64) {
            carry ^= __shfl(v, 63, 64);
            if (((qb + 64) & capm) == 0) carry = 0;  // next round starts a new wave segment
          }
          // table entry: grid[w][c] = first rank of wave w whose clock falls in cell >= c
          if (in) {
            const uint32_t w = q0 >> cl2, k = q0 & capm, V = sV[w];
            uint16_t* g = grid + w * ncell;
            if (k < V) {
              const uint32_t c0 = ts[q0] >> shift;
              const int32_t c = (int32_t)(c0 < ncell ? c0 : ncell - 1);
              int32_t c_prev = -1;
              if (k > 0) { const uint32_t c1 = ts[q0 - 1] >> shift; c_prev = (int32_t)(c1 < ncell ? c1 : ncell - 1); }
              for (int32_t cc = c_prev + 1; cc <= c; ++cc) g[cc] = (uint16_t)k;
            }
          }
          if (in) om[q0] = (MaskT)ex;  // every lane has read its metadata by now (shuffles above)
        }
      }
      __syncthreads();
      // ---- E: region-pair overlap, one lane per time cell ------------------------------------------
      if (W <= 4)      sweep_cells<4, MaskT>(ts, om, grid, sV, oacc, W, R, cl2, nrec, ncell, shift, tid, BLOCK);
      else if (W <= 8) sweep_cells<8, MaskT>(ts, om, grid, sV, oacc, W, R, cl2, nrec, ncell, shift, tid, BLOCK);
      else             sweep_cells<16, MaskT>(ts, om, grid, sV, oacc, W, R, cl2, nrec, ncell, shift, tid, BLOCK);
    }
    __syncthreads();

    // ---- F: per-(workgroup, wave, region) output, fold into running totals ------------------------
    for (uint32_t e = tid; e < W * R; e += BLOCK) {
      const unsigned long long pk = pw_pack[e];
      const uint32_t n = (uint32_t)(pk >> 46);
      const unsigned long long s = pk & ((1ull << 46) - 1);
      const uint32_t mx = pw_max[e], mn = pw_min[e];
      uint64_t* dst = p.out + SL.per + ((size_t)wg * W * R + e) * 2;
      dst[0] = s;
      dst[1] = (uint64_t)n | ((uint64_t)mx << 32);
      if (n) {
        const uint32_t r = e % R;
        atomicAdd(&reg_sum[r], s);
        atomicMax(&reg_max[r], mx);
        atomicMin(&reg_min[r], mn);
      }
      pw_pack[e] = 0; pw_max[e] = 0; pw_min[e] = 0xFFFFFFFFu;
    }
    if (tid == 0) {
      ctr[H_INVALID] += wg_invalid;
      ctr[H_DISORDER] += tmp[T_DISORDER];
      ctr[H_NONMONO] += tmp[T_NONMONO];
      ctr[H_PAIRS] += tmp[T_PAIRS];
      ctr[H_ORPHAN_START] += tmp[T_ORPH_S] - tmp[T_PAIRS];
      ctr[H_ORPHAN_END] += tmp[T_ORPH_E] - tmp[T_PAIRS];
      ctr[H_SPAN_OVF] += tmp[T_SPANOVF];
      ctr[H_OVERLAP_WGS] += eligible ? 1u : 0u;
    }
    __syncthreads();
  }

  // ---- flush this decoder workgroup's totals --------------------------------------------------
  unsigned long long* out = reinterpret_cast<unsigned long long*>(p.out);
  for (uint32_t i = tid; i < R * 64; i += BLOCK)
    if (hist[i]) atomicAdd(&out[SL.hist + i], (unsigned long long)hist[i]);
  for (uint32_t i = tid; i < R * R; i += BLOCK)
    if (oacc[i]) atomicAdd(&out[SL.F + i], oacc[i]);  // staged in the F area until finalize
  for (uint32_t r = tid; r < R; r += BLOCK) {
    if (reg_min[r] != 0xFFFFFFFFu || reg_max[r] || reg_sum[r]) {
      atomicAdd(&out[SL.sum + r], reg_sum[r]);
      atomicMax(&out[SL.max + r], (unsigned long long)reg_max[r]);
      atomicMin(&out[SL.min + r], (unsigned long long)reg_min[r]);
    }
  }
  if (tid < H_STATUS && ctr[tid]) atomicAdd(&out[tid], ctr[tid]);
}

// Launch shape of one kernel instantiation for one LDS size, queried once per device.
struct LaunchCache { int dev = -1; uint32_t lds = 0; uint32_t max_grid = 0; };

template <typename MaskT, int BLOCK>
kp_status launch_main(const DecodeParams& p, uint32_t lds_bytes, hipStream_t s) {
  auto kern = kp_reduce_main<MaskT, BLOCK>;
  static thread_local LaunchCache cache;
  int dev = 0;
  KP_HIP_TRY(hipGetDevice(&dev));
  if (cache.dev != dev || cache.lds != lds_bytes) {
    KP_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes));
    int per_cu = 0, cus = 0;
    KP_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, BLOCK, lds_bytes));
    if (per_cu < 1) return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "decoder kernel does not fit one CU (LDS %u B)", lds_bytes);
    KP_HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    cache.dev = dev; cache.lds = lds_bytes; cache.max_grid = (uint32_t)per_cu * (uint32_t)cus;
  }
  uint32_t grid = cache.max_grid;
  if (grid > p.n_wg) grid = p.n_wg;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(BLOCK), lds_bytes, s, p);
  KP_HIP_TRY(hipGetLastError());
  return KP_OK;
}

kp_status reduce_impl(const void* raw, size_t n, const kp_trace_hdr& h, void* out_stats, hipStream_t s) {
  if (h.magic != KP_TRACE_MAGIC || h.version != KP_TRACE_VERSION)
    return kp::fail(KP_ERR_BAD_TRACE, "trace header: bad magic/version (%08x, %u)", h.magic, h.version);
  if (h.waves_per_wg < 1 || h.waves_per_wg > KP_MAX_WAVES || h.n_regions < 1 || !kp::is_pow2(h.cap_wave))
    return kp::fail(KP_ERR_BAD_TRACE, "trace header: waves=%u regions=%u cap_wave=%u", h.waves_per_wg, h.n_regions, h.cap_wave);
  if ((size_t)h.n_wg * h.waves_per_wg * h.cap_wave != n)
    return kp::fail(KP_ERR_BAD_TRACE, "trace header describes %zu record slots, caller passed %zu",
                    (size_t)h.n_wg * h.waves_per_wg * h.cap_wave, n);
  if ((h.flags & ~KP_FLAG_FLUSH) != 0) return kp::fail(KP_ERR_BAD_TRACE, "trace header: unknown flags %x", h.flags);
  if (h.n_regions > KP_MAX_REGIONS)
    return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "n_regions=%u exceeds the decoder limit %d", h.n_regions, KP_MAX_REGIONS);
  if (h.cap_wave < 2) return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "cap_wave must be at least 2");
  const uint32_t nrec = h.waves_per_wg * h.cap_wave;
  if (nrec > kMaxRecPerWg)
    return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "%u records per workgroup exceed the LDS staging limit %u", nrec, kMaxRecPerWg);
  if (((uintptr_t)raw & 15u) || ((uintptr_t)out_stats & 15u))
    return kp::fail(KP_ERR_INVALID_ARG, "raw and out_stats must be 16-byte aligned");

  const uint32_t W = h.waves_per_wg, R = h.n_regions, cap = h.cap_wave;
  const int block = nrec >= 8192 ? 1024 : (nrec >= 2048 ? 512 : 256);
  // positions per hardware wave of the decoder: a power of two >= 64 covering nrec
  uint32_t span = 64;
  while (span * (uint32_t)(block / 64) < nrec) span <<= 1;
  const uint32_t ncell = cap < 1024 ? cap : 1024;
  const uint32_t mask_bytes = R <= 16 ? 2 : 4;
  const LdsLayout L = lds_layout(nrec, W, R, ncell, mask_bytes, block);
  if (L.total > kMaxLds)
    return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "decoder needs %u B of LDS for this geometry (limit %u)", L.total, kMaxLds);

  uint64_t* out = static_cast<uint64_t*>(out_stats);
  const uint8_t* base = static_cast<const uint8_t*>(raw);
  const StatsLayout SL = stats_layout(h.n_wg, W, R);
  int init_blocks = (int)((SL.per + 255) / 256);
  if (init_blocks > 64) init_blocks = 64;
  hipLaunchKernelGGL(kp_reduce_init, dim3(init_blocks), dim3(256), 0, s,
                     reinterpret_cast<const uint32_t*>(base), out, h.n_wg, W, R, cap, h.flags);
  KP_HIP_TRY(hipGetLastError());

  if (h.n_wg > 0) {
    DecodeParams p;
    p.wg_hdrs = reinterpret_cast<const uint32_t*>(base + sizeof(kp_trace_hdr));
    p.records = reinterpret_cast<const u32x4*>(base + sizeof(kp_trace_hdr) + sizeof(kp_wg_hdr) * (size_t)h.n_wg);
    p.out = out;
    p.n_wg = h.n_wg; p.W = W; p.R = R; p.cap = cap;
    p.cap_log2 = 0; while ((1u << p.cap_log2) < cap) ++p.cap_log2;
    p.rec_cost = h.rec_cost; p.flush = h.flags & KP_FLAG_FLUSH;
    p.nrec = nrec; p.span = span; p.ncell = ncell;
    kp_status st;
    if (mask_bytes == 2) {
      st = block == 1024 ? launch_main<uint16_t, 1024>(p, L.total, s)
         : block == 512  ? launch_main<uint16_t, 512>(p, L.total, s)
                         : launch_main<uint16_t, 256>(p, L.total, s);
    } else {
      st = block == 1024 ? launch_main<uint32_t, 1024>(p, L.total, s)
         : block == 512  ? launch_main<uint32_t, 512>(p, L.total, s)
                         : launch_main<uint32_t, 256>(p, L.total, s);
    }
    if (st != KP_OK) return st;
  }
  hipLaunchKernelGGL(kp_reduce_finalize, dim3(1), dim3(256), 0, s, out, h.n_wg, W, R);
  KP_HIP_TRY(hipGetLastError());
  return KP_OK;
}

}  // namespace

extern "C" kp_status kp_trace_reduce_hdr(const void* raw, size_t n, const kp_trace_hdr* hdr_host,
                                         void* out_stats, void* stream) {
  kp::clear_error();
  if (!raw || !hdr_host || !out_stats) return kp::fail(KP_ERR_INVALID_ARG, "NULL argument");
  return reduce_impl(raw, n, *hdr_host, out_stats, static_cast<hipStream_t>(stream));
}

extern "C" kp_status kp_trace_reduce(const void* raw, size_t n, void* out_stats, void* stream) {
  kp::clear_error();
  if (!raw || !out_stats) return kp::fail(KP_ERR_INVALID_ARG, "NULL argument");
  kp_trace_hdr h;
  hipStream_t s = static_cast<hipStream_t>(stream);
  KP_HIP_TRY(hipMemcpyAsync(&h, raw, sizeof h, hipMemcpyDeviceToHost, s));
  KP_HIP_TRY(hipStreamSynchronize(s));
  return reduce_impl(raw, n, h, out_stats, s);
}

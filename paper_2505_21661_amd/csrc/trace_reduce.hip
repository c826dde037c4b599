// GPU trace decode / pair / reduce (kp_trace_reduce).
//
// The paper stores START/END records unpaired, per warp, in a ring whose tail survives, and
// aligns them at "trace replay" on the host (Sec. 4.2 "SM-level Data Layout", "Shared Memory
// Circular Buffer"; Sec. 4.3).  Here replay runs on the GPU: one decoder workgroup stages one
// recorded workgroup's records in LDS as (clock, metadata) pairs and
//   A  scatters every record to its rank (seq - first surviving seq), which undoes ring
//      rotation and out-of-order flushes in O(1) per record,
//   B  pairs each START with the next record of the same (wave, region) when that is an END,
//      takes d = (u32)(ts_end - ts_start) minus the constant record cost (Sec. 4.3), and
//      accumulates the per-(wave, region) sums and the log2 histogram with LDS atomics; the
//      four ranks an END looks back at come from neighbouring lanes, not from LDS,
//   C  XOR-scans the paired region bits of each wave into an "open regions" mask per position,
//   D  builds a coarse time -> position table per wave and orders the time cells by how many
//      records they hold, so that the lanes of a wave get cells of similar length,
//   E  sweeps every time cell in clock order, one lane per cell, keeping a bit-sliced count of
//      the waves that have each region open; when a record switches its region on or off for
//      the whole workgroup, -t / +t goes to the region-pair accumulators (the integral of
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
constexpr uint32_t kHistStride = 65;  // histogram rows 65 words apart: equal bins of different regions, different banks

// positions inside kp_stats_hdr, in u64 words
enum { H_SLOTS_VALID = 0, H_PAIRS, H_ORPHAN_START, H_ORPHAN_END, H_INVALID, H_DROPPED, H_DISORDER,
       H_SPAN_OVF, H_NONMONO, H_OVERLAP_WGS, H_STATUS, H_NWG, H_WAVES, H_NREG, H_CAP, H_RSVD };

// per-workgroup temporaries (u32 words in LDS)
enum { T_INVALID = 0, T_FIELDVALID, T_DISORDER, T_OCCUPIED, T_NONMONO, T_PAIRS, T_ORPH_S, T_ORPH_E,
       T_WIDE, T_COUNT };

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
  uint32_t nrec, span, span_log2, ncell, pos_bits;
};

struct LdsLayout {  // byte offsets
  uint32_t rec, grid, perm, cinfo, bucket, hist, oacc, oacc32, reg_sum, reg_max, reg_min, pw_pack, pw_max,
      pw_min, ctr, tmp, misc, v, first, wave_tot, total;
};
__host__ __device__ inline uint32_t align16(uint32_t x) { return (x + 15u) & ~15u; }
__host__ __device__ inline LdsLayout lds_layout(uint32_t nrec, uint32_t W, uint32_t R, uint32_t ncell, uint32_t block) {
  LdsLayout l;
  uint32_t o = 0;
  l.rec = o; o = align16(o + (nrec + 1) * 8);          // one zero entry past the last position
  l.grid = o; o = align16(o + W * (ncell + 1) * 2);    // one entry past the last cell per wave
  l.perm = o; o = align16(o + ncell * 2);
  l.cinfo = o; o = align16(o + ncell * 2);
  l.bucket = o; o = align16(o + 64 * 4);
  l.hist = o; o = align16(o + R * kHistStride * 4);
  l.oacc = o; o = align16(o + R * R * 8);
  l.oacc32 = o; o = align16(o + R * (R | 1u) * 4);
  l.reg_sum = o; o = align16(o + R * 8);
  l.reg_max = o; o = align16(o + R * 4);
  l.reg_min = o; o = align16(o + R * 4);
  l.pw_pack = o; o = align16(o + W * R * 8);
  l.pw_max = o; o = align16(o + W * R * 4);
  l.pw_min = o; o = align16(o + W * R * 4);
  l.ctr = o; o = align16(o + 16 * 8);
  l.tmp = o; o = align16(o + T_COUNT * 4);
  l.misc = o; o = align16(o + 8 * 4);
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

// Lane l receives the value of lane l-1; lane 0 receives `lane0` (DPP wave shift right by one).
__device__ __forceinline__ uint32_t wave_shr1(uint32_t v, uint32_t lane0) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)lane0, (int)v, 0x138, 0xF, 0xF, false);
}

// Inclusive XOR scan over the 64 lanes: four shifts inside each row of 16, then the last lane of
// row 0/2 into row 1/3 and the last lane of the lower half into the upper half.
__device__ __forceinline__ uint32_t wave_xor_scan(uint32_t v) {
  v ^= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xF, 0xF, false);  // row_shr:1
  v ^= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xF, 0xF, false);  // row_shr:2
  v ^= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xF, 0xF, false);  // row_shr:4
  v ^= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xF, 0xF, false);  // row_shr:8
  v ^= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xA, 0xF, false);  // row_bcast:15
  v ^= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xC, 0xF, false);  // row_bcast:31
  return v;
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
// into it in the total order (clock, wave, rank).  The number of waves that have each region open
// is kept bit-sliced: plane k holds bit k of every region's count, so "some wave has it open" is
// the OR of the planes and one record costs a ripple of PLANES steps.  When a paired record takes
// its region's count from 0 to 1 or from 1 to 0, -t or +t goes to the region-pair accumulators of
// all regions active at that instant.
//
// A merge key is (clock, position).  The narrow form keeps the clock relative to the start of the
// cell above `pos_bits` bits of position in one 32-bit word; it needs every clock of the cell to
// be below the cell's end and cell width * positions to fit 32 bits.  The wide form is 64 bits.
template <typename KeyT> struct SweepKey;
template <> struct SweepKey<uint32_t> {
  static __device__ __forceinline__ uint32_t make(uint32_t t, uint32_t pos, uint32_t cbase, uint32_t pb) { return ((t - cbase) << pb) | pos; }
  static __device__ __forceinline__ uint32_t pos(uint32_t k, uint32_t pmask) { return k & pmask; }
  static __device__ __forceinline__ uint32_t clock(uint32_t k, uint32_t cbase, uint32_t pb) { return cbase + (k >> pb); }
};
template <> struct SweepKey<unsigned long long> {
  static __device__ __forceinline__ unsigned long long make(uint32_t t, uint32_t pos, uint32_t, uint32_t) { return ((unsigned long long)t << 32) | pos; }
  static __device__ __forceinline__ uint32_t pos(unsigned long long k, uint32_t) { return (uint32_t)k; }
  static __device__ __forceinline__ uint32_t clock(unsigned long long k, uint32_t, uint32_t) { return (uint32_t)(k >> 32); }
};

template <int WMAX, int PLANES, typename KeyT>
__device__ __forceinline__ void sweep_cells(const uint2* rec, const uint16_t* grid, const uint16_t* perm,
                                            uint32_t* oacc32, uint32_t W, uint32_t R, uint32_t cl2,
                                            uint32_t pb, uint32_t ncell, uint32_t cw, uint32_t tid,
                                            uint32_t nthreads) {
  typedef SweepKey<KeyT> K;
  const KeyT none = ~(KeyT)0;
  const uint32_t capm = (1u << cl2) - 1u, pmask = (1u << pb) - 1u, gstride = ncell + 1;
  for (uint32_t i = tid; i < ncell; i += nthreads) {
    const uint32_t c = perm[i];
    const uint32_t cbase = c * cw;
    KeyT key[WMAX];        // each wave's next record in this cell; all-ones = none
    uint32_t pl[PLANES];   // bit-sliced count of the waves that have each region open
#pragma unroll
    for (int k = 0; k < PLANES; ++k) pl[k] = 0u;
    uint32_t n = 0;
#pragma unroll
    for (int w = 0; w < WMAX; ++w) {
      key[w] = none;
      if ((uint32_t)w < W) {
        const uint32_t g0 = grid[w * gstride + c], g1 = grid[w * gstride + c + 1];
        const uint32_t pos = ((uint32_t)w << cl2) + g0;
        const uint2 r = rec[pos];  // metadata = regions this wave has open before rank g0
        uint32_t carry = r.y;
#pragma unroll
        for (int k = 0; k < PLANES; ++k) { const uint32_t t = pl[k] & carry; pl[k] ^= carry; carry = t; }
        key[w] = g0 < g1 ? K::make(r.x, pos, cbase, pb) : none;
        n += g1 - g0;
      }
    }
    for (; n; --n) {
      KeyT best = key[0];
#pragma unroll
      for (int w = 1; w < WMAX; ++w) best = key[w] < best ? key[w] : best;
      const uint32_t pos = K::pos(best, pmask), tt = K::clock(best, cbase, pb);
      const uint32_t b = pos >> cl2;
      const uint32_t g1 = grid[b * gstride + c + 1];
      const uint2 cur = rec[pos];
      uint2 nxt = rec[pos + 1];
      asm volatile("" : "+v"(nxt.x));  // fetch the next clock with the masks, not behind the test below
      const bool more = (pos & capm) + 1u < g1;
      const KeyT nkey = more ? K::make(nxt.x, pos + 1u, cbase, pb) : none;
#pragma unroll
      for (int w = 0; w < WMAX; ++w) key[w] = key[w] == best ? nkey : key[w];
      const uint32_t x = cur.y ^ nxt.y;  // the region bit this record toggles; 0 if unpaired
      const bool is_end = (cur.y & x) != 0u;
      uint32_t act_before = pl[0];
#pragma unroll
      for (int k = 1; k < PLANES; ++k) act_before |= pl[k];
      {  // count[region] += 1 (START) or -= 1 (END)
        const uint32_t dm = is_end ? 0xFFFFFFFFu : 0u;
        uint32_t carry = x;
#pragma unroll
        for (int k = 0; k < PLANES; ++k) { const uint32_t o = pl[k]; pl[k] = o ^ carry; carry &= o ^ dm; }
      }
      uint32_t act_after = pl[0];
#pragma unroll
      for (int k = 1; k < PLANES; ++k) act_after |= pl[k];
      const uint32_t act = is_end ? act_after : act_before;  // active regions other than this one
      if (x & ~act) {  // the region was off before this START / is off after this END
        // modulo 2^32: the totals of one workgroup lie below its span, which is below 2^32
        uint32_t* row = oacc32 + (__ffs(x) - 1) * (R | 1u);
        const uint32_t val = is_end ? tt : 0u - tt;
        atomicAdd(&row[__ffs(x) - 1], val);
        uint32_t set = act;
        while (set) {
          const uint32_t bb = __ffs(set) - 1;
          set &= set - 1;
          atomicAdd(&row[bb], val);
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// Position p = wave*cap_wave + rank indexes the staged records.  Every hardware wave of the
// decoder owns `span` consecutive positions and walks them 64 at a time, lane l taking position
// base + 64*round + l, so that neighbouring lanes hold neighbouring ranks.
//
// Staged metadata word: bits 4:0 region, 5 END, 6 valid, 7 paired, 31:16 generation.  With at
// most 16 regions the staging area is not cleared between workgroups: a word counts only when
// its generation is the current one (the open-region masks that phase C leaves behind have
// generation 0, which is never current).  With more regions the masks reach into those bits, so
// the area is cleared for every workgroup and the generation stays 0.
template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void kp_reduce_main(DecodeParams p) {
  extern __shared__ __align__(16) unsigned char smem[];
  const LdsLayout L = lds_layout(p.nrec, p.W, p.R, p.ncell, BLOCK);
  uint2* rec = reinterpret_cast<uint2*>(smem + L.rec);
  uint32_t* recw = reinterpret_cast<uint32_t*>(smem + L.rec);  // word 2p = clock, 2p+1 = metadata
  uint16_t* grid = reinterpret_cast<uint16_t*>(smem + L.grid);
  uint16_t* perm = reinterpret_cast<uint16_t*>(smem + L.perm);
  uint16_t* cinfo = reinterpret_cast<uint16_t*>(smem + L.cinfo);
  uint32_t* bucket = reinterpret_cast<uint32_t*>(smem + L.bucket);
  uint32_t* hist = reinterpret_cast<uint32_t*>(smem + L.hist);
  unsigned long long* oacc = reinterpret_cast<unsigned long long*>(smem + L.oacc);
  uint32_t* oacc32 = reinterpret_cast<uint32_t*>(smem + L.oacc32);  // this workgroup's sums modulo 2^32
  unsigned long long* reg_sum = reinterpret_cast<unsigned long long*>(smem + L.reg_sum);
  uint32_t* reg_max = reinterpret_cast<uint32_t*>(smem + L.reg_max);
  uint32_t* reg_min = reinterpret_cast<uint32_t*>(smem + L.reg_min);
  unsigned long long* pw_pack = reinterpret_cast<unsigned long long*>(smem + L.pw_pack);
  uint32_t* pw_max = reinterpret_cast<uint32_t*>(smem + L.pw_max);
  uint32_t* pw_min = reinterpret_cast<uint32_t*>(smem + L.pw_min);
  unsigned long long* ctr = reinterpret_cast<unsigned long long*>(smem + L.ctr);
  uint32_t* tmp = reinterpret_cast<uint32_t*>(smem + L.tmp);
  uint32_t* misc = reinterpret_cast<uint32_t*>(smem + L.misc);  // [0] span overflow, [1] log2 of the power-of-two cell width, [2..4] cell width q << sh and 2^16 / q
  uint32_t* sV = reinterpret_cast<uint32_t*>(smem + L.v);
  uint32_t* sFirst = reinterpret_cast<uint32_t*>(smem + L.first);
  uint32_t* wave_tot = reinterpret_cast<uint32_t*>(smem + L.wave_tot);

  const uint32_t tid = threadIdx.x, lane = tid & 63u, hw = tid >> 6;
  const uint32_t W = p.W, R = p.R, cap = p.cap, nrec = p.nrec, ncell = p.ncell;
  const uint32_t capm = cap - 1, cl2 = p.cap_log2, gstride = ncell + 1;
  const uint32_t span = p.span;              // positions per hardware wave, power of two >= 64
  const uint32_t pbase = hw * span;
  const uint32_t pend = pbase + span < nrec ? pbase + span : nrec;  // may be <= pbase: idle wave
  const StatsLayout SL = stats_layout(p.n_wg, W, R);
  if (p.out[H_STATUS] != 0) return;  // device header did not match the launch geometry

  for (uint32_t i = tid; i < R * kHistStride; i += BLOCK) hist[i] = 0;
  for (uint32_t i = tid; i < R * R; i += BLOCK) oacc[i] = 0;
  for (uint32_t i = tid; i < R * (R | 1u); i += BLOCK) oacc32[i] = 0;
  for (uint32_t i = tid; i < R; i += BLOCK) { reg_sum[i] = 0; reg_max[i] = 0; reg_min[i] = 0xFFFFFFFFu; }
  for (uint32_t i = tid; i < W * R; i += BLOCK) { pw_pack[i] = 0; pw_max[i] = 0; pw_min[i] = 0xFFFFFFFFu; }
  if (tid < 16) ctr[tid] = 0;
  if (tid == 0) rec[nrec] = make_uint2(0u, 0u);
  __syncthreads();

  uint32_t iter = 0;
  for (uint32_t wg = blockIdx.x; wg < p.n_wg; wg += gridDim.x, ++iter) {
    const uint32_t* wh = p.wg_hdrs + (size_t)32 * wg;
    const uint32_t gen = R > 16 ? 0u : 1u + iter % 0xFFFFu;
    const uint32_t live_tag = (gen << 16) | kMValid, live_mask = 0xFFFF0000u | kMValid;
    auto is_live = [&](uint32_t m) { return (m & live_mask) == live_tag; };
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
    if (tid >= 128 && tid < 128 + BLOCK / 64) wave_tot[tid - 128] = 0;
    if (tid >= 192 && tid < 256) bucket[tid - 192] = 0;
    if (tid == 32) {
      const uint64_t tb = (uint64_t)wh[2] | ((uint64_t)wh[3] << 32);
      const uint64_t te = (uint64_t)wh[4] | ((uint64_t)wh[5] << 32);
      const uint64_t sp = te - tb;
      uint32_t shift = 0, ovf = 0;
      if (sp >> 32) ovf = 1; else while ((sp >> shift) >= ncell) ++shift;
      // Cell width q << sh: the narrowest of {5, 6, 7, 8} << (shift - 3) with which ncell cells still
      // cover the span, so that at least four cells in five are in use (a power of two alone may
      // leave half of them empty, and fuller cells make the sweep's longest lane longer).
      uint32_t q = 1u << shift, sh = 0;
      if (!ovf && shift >= 3) {
        sh = shift - 3; q = 8;
        for (uint32_t qq = 5; qq < 8; ++qq)
          if ((uint32_t)(sp >> sh) < ncell * qq) { q = qq; break; }
        if (q == 8) { q = 4; sh = shift - 2; }
      }
      misc[0] = ovf;
      misc[1] = shift;
      misc[2] = sh;
      misc[3] = q;
      misc[4] = 65535u / q + 1u;  // ceil(2^16 / q): (x * m) >> 16 == x / q for x < 8192, q < 8
    }
    if (R > 16 || gen == 1u) {  // clear the staging area (always on this workgroup's first pass)
      u32x4* z = reinterpret_cast<u32x4*>(rec);
      for (uint32_t i = tid; i < nrec / 2; i += BLOCK) z[i] = u32x4{0u, 0u, 0u, 0u};
    }
    __syncthreads();
    // table default: "no record of this wave at or after this cell"
    for (uint32_t i = tid; i < W * gstride; i += BLOCK) grid[i] = (uint16_t)sV[i / gstride];
    // ---- A: load and scatter by rank ------------------------------------------------------
    {
      const u32x4* recs = p.records + (size_t)wg * (nrec / 2);
      const uint32_t n16 = nrec / 2;  // 16-byte units, two records each
      uint32_t c_invalid = 0, c_field = 0, c_dis = 0;
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
            const uint32_t seq = tag & kSeqMask;
            const uint32_t k = (seq - first) & kSeqMask;
            const uint32_t region = (tag >> 24) & 0x7Fu;
            const bool held = s < V;
            const bool good = held && k < V && ((tag >> 20) & 0xFu) == w && region < R;
            c_invalid += (held && !good) ? 1u : 0u;
            c_field += good ? 1u : 0u;
            c_dis += (good && s != (seq & capm)) ? 1u : 0u;
            if (good) rec[(w << cl2) + k] = make_uint2(pay, region | ((tag >> 31) ? kMEnd : 0u) | live_tag);
          }
        }
      }
      add_tmp(tmp, T_INVALID, c_invalid);
      add_tmp(tmp, T_FIELDVALID, c_field);
      add_tmp(tmp, T_DISORDER, c_dis);
    }
    __syncthreads();
    // ---- occupancy check: a duplicated seq leaves fewer occupied ranks than valid records ----
    // Records that all sit in the slot of their own seq have distinct seq modulo the ring size, hence
    // distinct ranks: only a workgroup with a record elsewhere needs the count.
    const bool count_ranks = tmp[T_DISORDER] != 0u;
    if (count_ranks) {
      uint32_t occ = 0;
      for (uint32_t q = pbase + lane; q < pend; q += 64) occ += is_live(recw[2 * q + 1]) ? 1u : 0u;
      add_tmp(tmp, T_OCCUPIED, occ);
      __syncthreads();
    } else if (tid == 0) {
      tmp[T_OCCUPIED] = tmp[T_FIELDVALID];  // read again only after the next barrier
    }
    if (count_ranks && tmp[T_OCCUPIED] != tmp[T_FIELDVALID]) {
      // Rare: some seq occurs twice.  The later slot must win, so redo this workgroup's
      // scatter in slot order, one thread per wave.
      __syncthreads();
      for (uint32_t i = tid; i < nrec; i += BLOCK) recw[2 * i + 1] = 0;
      if (tid == 0) { tmp[T_DISORDER] = 0; tmp[T_OCCUPIED] = 0; }
      __syncthreads();
      if (tid < W) {
        const uint32_t w = tid, V = sV[w], first = sFirst[w];
        const uint32_t* seg = reinterpret_cast<const uint32_t*>(p.records) + ((size_t)wg * nrec + (size_t)w * cap) * 2;
        for (uint32_t s = 0; s < V; ++s) {
          const uint32_t tag = seg[2 * s];
          const uint32_t seq = tag & kSeqMask, k = (seq - first) & kSeqMask, region = (tag >> 24) & 0x7Fu;
          if (k >= V || ((tag >> 20) & 0xFu) != w || region >= R) continue;
          // the clock word remembers the winning slot for now
          rec[w * cap + k] = make_uint2(s, region | ((tag >> 31) ? kMEnd : 0u) | live_tag);
        }
        uint32_t dis = 0, occ = 0;
        for (uint32_t k = 0; k < V; ++k) {
          if (!is_live(recw[2 * (w * cap + k) + 1])) continue;
          const uint32_t s = recw[2 * (w * cap + k)];
          dis += (s != ((seg[2 * s] & kSeqMask) & capm));
          recw[2 * (w * cap + k)] = seg[2 * s + 1];
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
    // traces of real kernels the START sits a few ranks back.  The metadata of the four ranks
    // just below a lane's own comes from the lanes below it (the last four lanes of the previous
    // round stand in for lanes 0..3); deeper searches are the rare slow path.  A pair whose
    // START lies in an earlier hardware wave's span toggles the region bit of both spans'
    // XOR totals, which phase C turns into each span's carry-in.
    {
      uint32_t c_nonmono = 0, c_pairs = 0, c_starts = 0, c_ends = 0, x_span = 0;
      uint32_t cm[4], ct = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t back = pbase > (uint32_t)j ? (uint32_t)j + 1u : 0u;
        const uint2 r = rec[pbase < nrec ? pbase - back : 0u];
        cm[j] = (back && is_live(r.y)) ? r.y : 0u;
        if (j == 0) ct = r.x;
      }
      for (uint32_t qb = pbase; qb < pend; qb += 64) {
        const bool in = qb + lane < pend;
        const uint32_t q0 = in ? qb + lane : pend - 1;
        const uint2 r0 = rec[q0];
        const bool valid = in && is_live(r0.y);
        const uint32_t m0 = valid ? r0.y : 0u, t0 = r0.x;
        uint32_t m1 = wave_shr1(m0, cm[0]);
        uint32_t m2 = wave_shr1(m1, cm[1]);
        uint32_t m3 = wave_shr1(m2, cm[2]);
        uint32_t m4 = wave_shr1(m3, cm[3]);
        const uint32_t t1 = wave_shr1(t0, ct);
#pragma unroll
        for (int j = 0; j < 4; ++j) cm[j] = (uint32_t)__builtin_amdgcn_readlane((int)m0, 63 - j);
        ct = (uint32_t)__builtin_amdgcn_readlane((int)t0, 63);
        const uint32_t k = q0 & capm, wofs = q0 - k, w = q0 >> cl2;
        m1 = k > 0 ? m1 : 0u; m2 = k > 1 ? m2 : 0u; m3 = k > 2 ? m3 : 0u; m4 = k > 3 ? m4 : 0u;
        const uint32_t region = m0 & kMRegion;
        const bool is_end = (m0 & kMEnd) != 0u;  // m0 is 0 for a position that holds no record
        const uint32_t want = kMValid | region, sel = kMValid | kMRegion;
        const bool h1 = (m1 & sel) == want, h2 = (m2 & sel) == want, h3 = (m3 & sel) == want, h4 = (m4 & sel) == want;
        bool have = h1 || h2 || h3 || h4;             // nearest earlier record of the same region
        uint32_t pm = h1 ? m1 : (h2 ? m2 : (h3 ? m3 : m4));
        uint32_t pq = q0 - (h1 ? 1u : (h2 ? 2u : (h3 ? 3u : 4u)));
        bool have_prev = (m1 & kMValid) != 0u;        // previous record of this wave
        uint32_t tprev = t1;
        if (valid && k > 0 && (!have_prev || (is_end && !have && k > 4))) {  // slow path: walk back
          have = false;
          for (uint32_t kk = k; kk-- > 0;) {
            const uint2 rq = rec[wofs + kk];
            if (!is_live(rq.y)) continue;
            if (!have_prev) { have_prev = true; tprev = rq.x; }
            if (!is_end) break;
            if ((rq.y & kMRegion) == region) { have = true; pm = rq.y; pq = wofs + kk; break; }
          }
        }
        c_nonmono += (valid && have_prev && t0 < tprev) ? 1u : 0u;
        c_starts += (valid && !is_end) ? 1u : 0u;
        c_ends += is_end ? 1u : 0u;
        if (is_end && have && !(pm & kMEnd)) {
          ++c_pairs;
          const uint32_t pt = recw[2 * pq];
          recw[2 * pq + 1] = pm | kMPaired;
          recw[2 * q0 + 1] = m0 | kMPaired;
          if (pq < pbase) {
            x_span ^= 1u << region;
            atomicXor(&wave_tot[pq >> p.span_log2], 1u << region);
          }
          const uint32_t d_raw = t0 - pt;
          const uint32_t d = d_raw > p.rec_cost ? d_raw - p.rec_cost : 0u;
          const uint32_t e = w * R + region;
          atomicAdd(&pw_pack[e], (1ull << 46) | (unsigned long long)d);
          atomicMax(&pw_max[e], d);
          atomicMin(&pw_min[e], d);
          atomicAdd(&hist[region * kHistStride + (d ? 31 - __clz(d) : 0)], 1u);
        }
      }
#pragma unroll
      for (int d = 32; d >= 1; d >>= 1) x_span ^= __shfl_xor(x_span, d, 64);
      if (lane == 0 && x_span) atomicXor(&wave_tot[hw], x_span);
      add_tmp(tmp, T_NONMONO, c_nonmono);
      add_tmp(tmp, T_PAIRS, c_pairs);
      add_tmp(tmp, T_ORPH_S, c_starts);  // turned into orphan counts once T_PAIRS is complete
      add_tmp(tmp, T_ORPH_E, c_ends);
    }
    __syncthreads();
    const uint32_t wg_invalid = tmp[T_INVALID] + (tmp[T_FIELDVALID] - tmp[T_OCCUPIED]);
    const bool eligible = !misc[0] && wg_invalid == 0 && tmp[T_NONMONO] == 0;

    if (eligible) {
      const uint32_t shift = misc[1], csh = misc[2], cm = misc[4], xmax = 8u * ncell - 1u;
      const uint32_t cw = misc[3] << csh;  // cell width, at most 1 << shift
      auto cell_of = [&](uint32_t t) -> uint32_t {  // t / cw, or some value >= ncell when t lies past the cells
        uint32_t x = t >> csh;
        x = x < xmax ? x : xmax;
        return (x * cm) >> 16;
      };
      // ---- C: open-region mask before every position (exclusive XOR scan per wave) -------------
      // ---- D: coarse time -> position table: grid[w][c] = first rank of wave w in a cell >= c ----
      {
        uint32_t carry = 0;
        if (span < cap) {  // this span continues a wave that started in an earlier span
          const uint32_t firsthw = ((pbase >> cl2) << cl2) >> p.span_log2;
          for (uint32_t i = firsthw; i < hw; ++i) carry ^= wave_tot[i];
        }
        uint32_t cprev_carry = 0, wide = 0;
        if (pbase > 0 && pbase < nrec) {
          const uint32_t c1 = cell_of(recw[2 * (pbase - 1)]);
          cprev_carry = c1 < ncell ? c1 : ncell - 1;
        }
        for (uint32_t qb = pbase; qb < pend; qb += 64) {
          const bool in = qb + lane < pend;
          const uint32_t q0 = in ? qb + lane : pend - 1;
          const uint2 r0 = rec[q0];
          const bool paired = in && is_live(r0.y) && (r0.y & kMPaired);
          const uint32_t x = paired ? (1u << (r0.y & kMRegion)) : 0u;
          uint32_t v = x;
          if (cap >= 64) {
            v = wave_xor_scan(v);
          } else {
            for (uint32_t d = 1; d < cap; d <<= 1) { const uint32_t y = __shfl_up(v, d, 64); if ((lane & capm) >= d) v ^= y; }
          }
          const uint32_t ex = v ^ x ^ carry;
          if (cap >= 64) {
            carry ^= (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
            if (((qb + 64) & capm) == 0) carry = 0;  // next round starts a new wave segment
          }
          const uint32_t w = q0 >> cl2, k = q0 & capm, V = sV[w];
          const uint32_t c0 = cell_of(r0.x);
          const uint32_t c = c0 < ncell ? c0 : ncell - 1;
          const uint32_t cp = wave_shr1(c, cprev_carry);
          cprev_carry = (uint32_t)__builtin_amdgcn_readlane((int)c, 63);
          if (in && k < V) {
            wide |= c0 >= ncell ? 1u : 0u;
            uint16_t* g = grid + w * gstride;
            for (uint32_t cc = k > 0 ? cp + 1 : 0u; cc <= c; ++cc) g[cc] = (uint16_t)k;
          }
          if (in) recw[2 * q0 + 1] = ex;
        }
        if (wide) tmp[T_WIDE] = 1u;  // some clock lies past the recorded span: narrow merge keys are off
      }
      __syncthreads();
      // ---- order the cells by record count (counting sort, fullest first) --------------------------
      for (uint32_t c = tid; c < ncell; c += BLOCK) {
        uint32_t n = 0;
        for (uint32_t w = 0; w < W; ++w) n += (uint32_t)grid[w * gstride + c + 1] - (uint32_t)grid[w * gstride + c];
        const uint32_t nb = n < 63u ? n : 63u;
        const uint32_t slot = atomicAdd(&bucket[nb], 1u);
        cinfo[c] = (uint16_t)(nb | (slot << 6));
      }
      __syncthreads();
      if (tid < 64) {  // exclusive prefix over the buckets, from 63 down
        const uint32_t mine = bucket[63 - tid];
        uint32_t incl = mine;
#pragma unroll
        for (uint32_t d = 1; d < 64; d <<= 1) { const uint32_t y = __shfl_up(incl, d, 64); if (tid >= d) incl += y; }
        bucket[63 - tid] = incl - mine;
      }
      __syncthreads();
      for (uint32_t c = tid; c < ncell; c += BLOCK) {
        const uint32_t ci = cinfo[c];
        perm[bucket[ci & 63u] + (ci >> 6)] = (uint16_t)c;
      }
      __syncthreads();
      // ---- E: region-pair overlap, one lane per time cell ------------------------------------------
      const uint32_t pb = p.pos_bits;
      if (!tmp[T_WIDE] && shift + pb <= 31u) {  // the all-ones key must stay free
        if (W <= 4)      sweep_cells<4, 3, uint32_t>(rec, grid, perm, oacc32, W, R, cl2, pb, ncell, cw, tid, BLOCK);
        else if (W <= 8) sweep_cells<8, 4, uint32_t>(rec, grid, perm, oacc32, W, R, cl2, pb, ncell, cw, tid, BLOCK);
        else             sweep_cells<16, 5, uint32_t>(rec, grid, perm, oacc32, W, R, cl2, pb, ncell, cw, tid, BLOCK);
      } else {
        if (W <= 4)      sweep_cells<4, 3, unsigned long long>(rec, grid, perm, oacc32, W, R, cl2, pb, ncell, cw, tid, BLOCK);
        else if (W <= 8) sweep_cells<8, 4, unsigned long long>(rec, grid, perm, oacc32, W, R, cl2, pb, ncell, cw, tid, BLOCK);
        else             sweep_cells<16, 5, unsigned long long>(rec, grid, perm, oacc32, W, R, cl2, pb, ncell, cw, tid, BLOCK);
      }
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
    // region-pair sums of this workgroup: the two one-sided sums of a pair add up, modulo 2^32, to the
    // time both regions were open (below the span, hence exact); the upper triangle keeps the totals
    for (uint32_t i = tid; i < R * R; i += BLOCK) {
      const uint32_t a = i / R, b = i - a * R;
      if (a > b) continue;
      uint32_t* ab = oacc32 + a * (R | 1u) + b;
      uint32_t* ba = oacc32 + b * (R | 1u) + a;
      const uint32_t v = a == b ? *ab : *ab + *ba;
      *ab = 0u; *ba = 0u;
      oacc[i] += v;
    }
    if (tid == 0) {
      ctr[H_INVALID] += wg_invalid;
      ctr[H_DISORDER] += tmp[T_DISORDER];
      ctr[H_NONMONO] += tmp[T_NONMONO];
      ctr[H_PAIRS] += tmp[T_PAIRS];
      ctr[H_ORPHAN_START] += tmp[T_ORPH_S] - tmp[T_PAIRS];
      ctr[H_ORPHAN_END] += tmp[T_ORPH_E] - tmp[T_PAIRS];
      ctr[H_SPAN_OVF] += misc[0];
      ctr[H_OVERLAP_WGS] += eligible ? 1u : 0u;
    }
    __syncthreads();
  }

  // ---- flush this decoder workgroup's totals --------------------------------------------------
  unsigned long long* out = reinterpret_cast<unsigned long long*>(p.out);
  for (uint32_t i = tid; i < R * 64; i += BLOCK) {
    const uint32_t h = hist[(i >> 6) * kHistStride + (i & 63u)];
    if (h) atomicAdd(&out[SL.hist + i], (unsigned long long)h);
  }
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

template <int BLOCK>
kp_status launch_main(const DecodeParams& p, uint32_t lds_bytes, hipStream_t s) {
  auto kern = kp_reduce_main<BLOCK>;
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
  uint32_t span_log2 = 0;
  while ((1u << span_log2) < span) ++span_log2;
  // time cells per wave: at most one per record slot, 1024, and 8192 table entries over all waves
  uint32_t ncell = cap < 1024 ? cap : 1024;
  while (W * ncell > 8192) ncell >>= 1;
  const LdsLayout L = lds_layout(nrec, W, R, ncell, block);
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
    p.nrec = nrec; p.span = span; p.span_log2 = span_log2; p.ncell = ncell;
    p.pos_bits = 0; while ((1u << p.pos_bits) < nrec) ++p.pos_bits;
    const kp_status st = block == 1024 ? launch_main<1024>(p, L.total, s)
                       : block == 512  ? launch_main<512>(p, L.total, s)
                                       : launch_main<256>(p, L.total, s);
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

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
constexpr int kMaxChunk = 16;
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
  uint32_t nrec, chunk, ncell;
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

  const uint32_t tid = threadIdx.x;
  const uint32_t W = p.W, R = p.R, cap = p.cap, nrec = p.nrec, CH = p.chunk, ncell = p.ncell;
  const uint32_t capm = cap - 1;
  const StatsLayout SL = stats_layout(p.n_wg, W, R);
  if (p.out[H_STATUS] != 0) return;  // device header did not match the launch geometry

  for (uint32_t i = tid; i < R * 64; i += BLOCK) hist[i] = 0;
  for (uint32_t i = tid; i < R * R; i += BLOCK) oacc[i] = 0;
  for (uint32_t i = tid; i < R; i += BLOCK) { reg_sum[i] = 0; reg_max[i] = 0; reg_min[i] = 0xFFFFFFFFu; }
  for (uint32_t i = tid; i < W * R; i += BLOCK) { pw_pack[i] = 0; pw_max[i] = 0; pw_min[i] = 0xFFFFFFFFu; }
  if (tid < 16) ctr[tid] = 0;

  // this thread's chunk of consecutive ranks (all inside one wave segment)
  const uint32_t nchunks = nrec / CH;
  const bool has_chunk = tid < nchunks;
  const uint32_t cbase = tid * CH;               // flat position of the chunk
  const uint32_t cw = has_chunk ? (cbase >> p.cap_log2) : 0;  // its wave
  const uint32_t ck = cbase & capm;              // rank of its first element
  const uint32_t wofs = cw * cap;
  const uint32_t tps = cap / CH;                 // threads per wave segment (power of two)
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
    if (tid < T_COUNT) tmp[tid] = 0;
    if (tid == 32) {
      const uint64_t tb = (uint64_t)wh[2] | ((uint64_t)wh[3] << 32);
      const uint64_t te = (uint64_t)wh[4] | ((uint64_t)wh[5] << 32);
      const uint64_t span = te - tb;
      uint32_t shift = 0;
      if (span >> 32) {
        tmp[T_SPANOVF] = 1;
      } else {
        while ((span >> shift) >= ncell) ++shift;
      }
      tmp[T_SHIFT] = shift;
    }
    for (uint32_t i = tid; i < nrec; i += BLOCK) om[i] = 0;
    __syncthreads();

    // ---- A: load and scatter by rank ------------------------------------------------------
    {
      const u32x4* rec = p.records + (size_t)wg * (nrec / 2);
      uint32_t c_invalid = 0, c_field = 0, c_dis = 0;
      for (uint32_t i = tid; i < nrec / 2; i += BLOCK) {
        const u32x4 v = __builtin_nontemporal_load(rec + i);
        const uint32_t f0 = 2 * i;
        const uint32_t w = f0 >> p.cap_log2;
        const uint32_t V = sV[w], first = sFirst[w];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const uint32_t tag = h ? v.z : v.x, pay = h ? v.w : v.y;
          const uint32_t s = (f0 + h) & capm;
          if (s < V) {
            const uint32_t seq = tag & kSeqMask;
            const uint32_t k = (seq - first) & kSeqMask;
            const uint32_t region = (tag >> 24) & 0x7Fu;
            if (k >= V || ((tag >> 20) & 0xFu) != w || region >= R) {
              ++c_invalid;
            } else {
              ts[w * cap + k] = pay;
              om[w * cap + k] = (MaskT)(region | ((tag >> 31) ? kMEnd : 0u) | kMValid);
              ++c_field;
              c_dis += (s != (seq & capm));
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
    uint32_t m[kMaxChunk], t[kMaxChunk];
    {
      uint32_t occ = 0;
#pragma unroll
      for (int j = 0; j < kMaxChunk; ++j) {
        m[j] = 0; t[j] = 0;
        if (has_chunk && (uint32_t)j < CH) { m[j] = om[cbase + j]; t[j] = ts[cbase + j]; occ += (m[j] & kMValid) ? 1u : 0u; }
      }
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
#pragma unroll
      for (int j = 0; j < kMaxChunk; ++j)
        if (has_chunk && (uint32_t)j < CH) { m[j] = om[cbase + j]; t[j] = ts[cbase + j]; }
    }

    // ---- B: pairing, durations, per-(wave,region) statistics, monotonicity --------------------
    {
      uint32_t c_nonmono = 0, c_pairs = 0, c_os = 0;
      const uint32_t V = has_chunk ? sV[cw] : 0;
#pragma unroll
      for (int j = 0; j < kMaxChunk; ++j) {
        if (!has_chunk || (uint32_t)j >= CH) continue;
        const uint32_t k = ck + j;
        if (k >= V || !(m[j] & kMValid)) continue;
        // next record of this wave in rank order (ranks can be missing after invalid records)
        uint32_t q = k + 1;
        while (q < V && !(om[wofs + q] & kMValid)) ++q;
        if (q < V && ts[wofs + q] < t[j]) ++c_nonmono;
        if (!(m[j] & kMEnd)) {
          const uint32_t region = m[j] & kMRegion;
          bool paired = false;
          for (; q < V; ++q) {
            const uint32_t mq = om[wofs + q];
            if (!(mq & kMValid) || (mq & kMRegion) != region) continue;
            if (mq & kMEnd) {
              paired = true;
              om[wofs + q] = (MaskT)(mq | kMPaired);
              const uint32_t d_raw = ts[wofs + q] - t[j];
              const uint32_t d = d_raw > p.rec_cost ? d_raw - p.rec_cost : 0u;
              const uint32_t e = cw * R + region;
              atomicAdd(&pw_pack[e], (1ull << 46) | (unsigned long long)d);
              atomicMax(&pw_max[e], d);
              atomicMin(&pw_min[e], d);
              atomicAdd(&hist[region * 64 + (d ? 31 - __clz(d) : 0)], 1u);
            }
            break;
          }
          if (paired) { m[j] |= kMPaired; ++c_pairs; } else { ++c_os; }
        }
      }
      add_tmp(tmp, T_NONMONO, c_nonmono);
      add_tmp(tmp, T_PAIRS, c_pairs);
      add_tmp(tmp, T_ORPH_S, c_os);
    }
    __syncthreads();
    {
      uint32_t c_oe = 0;
      const uint32_t V = has_chunk ? sV[cw] : 0;
#pragma unroll
      for (int j = 0; j < kMaxChunk; ++j) {
        if (!has_chunk || (uint32_t)j >= CH || ck + j >= V) continue;
        if ((m[j] & (kMValid | kMEnd)) == (kMValid | kMEnd)) {
          m[j] = om[cbase + j];
          c_oe += (m[j] & kMPaired) ? 0u : 1u;
        }
      }
      add_tmp(tmp, T_ORPH_E, c_oe);
    }
    __syncthreads();  // every thread is done reading metadata from `om`

    const uint32_t wg_invalid = tmp[T_INVALID] + (tmp[T_FIELDVALID] - tmp[T_OCCUPIED]);
    const bool eligible = !tmp[T_SPANOVF] && wg_invalid == 0 && tmp[T_NONMONO] == 0;

    if (eligible) {
      const uint32_t V = has_chunk ? sV[cw] : 0;
      // ---- C: open-region mask before every position (exclusive XOR scan per wave) ------------
      uint32_t ex[kMaxChunk];
      uint32_t x_tot = 0;
#pragma unroll
      for (int j = 0; j < kMaxChunk; ++j) {
        ex[j] = x_tot;
        if ((uint32_t)j < CH && (m[j] & kMPaired)) x_tot ^= 1u << (m[j] & kMRegion);
      }
      uint32_t carry;
      {
        const uint32_t lane = tid & 63;
        uint32_t v = x_tot;
        if (tps <= 64) {
          for (uint32_t d = 1; d < tps; d <<= 1) {
            const uint32_t y = __shfl_up(v, d, 64);
            if ((lane & (tps - 1)) >= d) v ^= y;
          }
          carry = v ^ x_tot;
        } else {
          for (uint32_t d = 1; d < 64; d <<= 1) {
            const uint32_t y = __shfl_up(v, d, 64);
            if (lane >= d) v ^= y;
          }
          if (lane == 63) wave_tot[tid >> 6] = v;
          __syncthreads();
          const uint32_t hw = tid >> 6, wps = tps >> 6, firsthw = hw & ~(wps - 1);
          uint32_t c = 0;
          for (uint32_t i = firsthw; i < hw; ++i) c ^= wave_tot[i];
          carry = c ^ v ^ x_tot;
        }
      }
#pragma unroll
      for (int j = 0; j < kMaxChunk; ++j) {
        ex[j] ^= carry;
        if (has_chunk && (uint32_t)j < CH) om[cbase + j] = (MaskT)ex[j];
      }
      // ---- D: coarse time -> position table -----------------------------------------------------
      const uint32_t shift = tmp[T_SHIFT];
      if (has_chunk) {
        uint16_t* g = grid + cw * ncell;
        if (V == 0) {
          if (ck == 0) for (uint32_t c = 0; c < ncell; ++c) g[c] = 0;
        } else {
          int32_t c_prev = -1;
          if (ck > 0 && ck < V) { const uint32_t c0 = ts[cbase - 1] >> shift; c_prev = (int32_t)(c0 < ncell ? c0 : ncell - 1); }
#pragma unroll
          for (int j = 0; j < kMaxChunk; ++j) {
            if ((uint32_t)j >= CH || ck + j >= V) continue;
            const uint32_t c0 = t[j] >> shift;
            const int32_t c = (int32_t)(c0 < ncell ? c0 : ncell - 1);
            for (int32_t cc = c_prev + 1; cc <= c; ++cc) g[cc] = (uint16_t)(ck + j);
            c_prev = c;
            if (ck + j == V - 1) for (uint32_t cc = c + 1; cc < ncell; ++cc) g[cc] = (uint16_t)V;
          }
        }
      }
      __syncthreads();
      // ---- E: region-pair overlap from workgroup-level switching times ------------------------------
#pragma unroll
      for (int j = 0; j < kMaxChunk; ++j) {
        if (!has_chunk || (uint32_t)j >= CH || !(m[j] & kMPaired)) continue;
        const uint32_t tt = t[j];
        const uint32_t a = m[j] & kMRegion;
        const uint32_t c0 = tt >> shift;
        const uint32_t cell = c0 < ncell ? c0 : ncell - 1;
        uint32_t others = 0;
        for (uint32_t w2 = 0; w2 < W; ++w2) {
          if (w2 == cw) continue;
          const uint32_t V2 = sV[w2];
          uint32_t pos = grid[w2 * ncell + cell];
          const uint32_t* ts2 = ts + w2 * cap;
          if (w2 < cw) { while (pos < V2 && ts2[pos] <= tt) ++pos; }
          else         { while (pos < V2 && ts2[pos] < tt) ++pos; }
          if (pos < V2) others |= (uint32_t)om[w2 * cap + pos];
        }
        if (!((others >> a) & 1u)) {
          const unsigned long long val = (m[j] & kMEnd) ? (unsigned long long)tt : (0ull - (unsigned long long)tt);
          atomicAdd(&oacc[a * R + a], val);
          uint32_t set = (others | ex[j]) & ~(1u << a);
          while (set) {
            const uint32_t b = __ffs(set) - 1;
            set &= set - 1;
            atomicAdd(&oacc[a * R + b], val);
          }
        }
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
    if (tid == 0) {
      ctr[H_INVALID] += wg_invalid;
      ctr[H_DISORDER] += tmp[T_DISORDER];
      ctr[H_NONMONO] += tmp[T_NONMONO];
      ctr[H_PAIRS] += tmp[T_PAIRS];
      ctr[H_ORPHAN_START] += tmp[T_ORPH_S];
      ctr[H_ORPHAN_END] += tmp[T_ORPH_E];
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

struct DeviceInfo { int cus = 0; };
DeviceInfo& device_info() {
  static thread_local DeviceInfo di;
  return di;
}

template <typename MaskT, int BLOCK>
kp_status launch_main(const DecodeParams& p, uint32_t lds_bytes, hipStream_t s) {
  auto kern = kp_reduce_main<MaskT, BLOCK>;
  KP_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes));
  int per_cu = 0;
  KP_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, BLOCK, lds_bytes));
  if (per_cu < 1) return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "decoder kernel does not fit one CU (LDS %u B)", lds_bytes);
  int dev = 0, cus = 0;
  KP_HIP_TRY(hipGetDevice(&dev));
  KP_HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  uint32_t grid = (uint32_t)per_cu * (uint32_t)cus;
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
  uint32_t chunk = 1;
  while (chunk * (uint32_t)block < nrec) chunk <<= 1;
  if (chunk > cap) chunk = cap;
  if (chunk > (uint32_t)kMaxChunk) return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "internal: chunk %u", chunk);
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
    p.nrec = nrec; p.chunk = chunk; p.ncell = ncell;
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

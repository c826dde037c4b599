// Critical path over the stage table (kp_stages_critical).
//
// The paper reads the critical path of a kernel whose warp groups work on different stages off the
// timeline: a chain of stages each of which could only start when the one before it had finished
// (Sec. 3.3 "Critical-path Analysis"; Sec. 5.2, where a load turns out to be held up by a barrier of another
// warp group), and takes the sum of the latencies along it as the kernel's latency (Table 4, WS model).
// Here the chain is taken per recorded workgroup from its stage table: stages ordered by (max_end,
// index); the path ends in the last one; the stage before X is the latest stage of that order, earlier
// than X, that had ended by the time X started.
//
// One decoder workgroup per recorded workgroup at a time (persistent, grid stride), everything in LDS:
//   1  the entries become 64-bit keys max_end << 32 | index (no stage: all ones) and are sorted with
//      a bitonic network;
//   2  every stage finds the stage before it with one binary search over the sorted ends -- the stages
//      that ended by its start are a prefix of the order -- which gives a forest of "waited for" links;
//   3  the path is the list that starts at the last stage: it is marked by pointer doubling (in round k
//      every marked stage marks the stage 2^k links on and every link is replaced by two), log2(n)
//      rounds instead of a walk of up to n steps;
//   4  marked stages add their latency to their region's totals, and the gaps to the stage before them
//      to the workgroup's bubbles.
#include "kp_common.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBlock = 256;
constexpr uint32_t kMaxEntries = 4096;
constexpr uint32_t kNone = 0xFFFFFFFFu;

struct CriticalParams {
  const u32x4* table;          // [n_wg][R * I] of {max_dur, min_start, max_end, n_waves}
  unsigned long long* hdr;     // 8 words
  unsigned long long* region;  // [R][2]
  u32x4* rows;                 // [n_wg][2]
  uint32_t n_wg, R, I, N, P, log2P;
};

__global__ void kp_critical_init(unsigned long long* out, uint32_t n_wg, uint32_t R, uint32_t I) {
  for (uint32_t i = threadIdx.x; i < 8 + 2 * R; i += blockDim.x) out[i] = i == 0 ? n_wg : (i == 1 ? R : (i == 2 ? I : 0ull));
}

__device__ inline unsigned long long wave_sum64(unsigned long long v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
  return v;
}
__device__ inline uint32_t wave_sum32(uint32_t v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
  return v;
}
__device__ inline uint32_t wave_min32(uint32_t v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) { const uint32_t o = __shfl_xor(v, d, 64); v = o < v ? o : v; }
  return v;
}

// LDS: key[P] u64 | start[N] | lat[N] | jump[2][P] | mark[P] bytes | totals
__global__ __launch_bounds__(kBlock) void kp_critical_main(CriticalParams p) {
  extern __shared__ __align__(16) unsigned char smem[];
  const uint32_t P = p.P, N = p.N, R = p.R, I = p.I;
  unsigned long long* key = reinterpret_cast<unsigned long long*>(smem);
  uint32_t* start = reinterpret_cast<uint32_t*>(smem + 8 * (size_t)P);
  uint32_t* lat = start + P;
  uint32_t* jump0 = lat + P;
  uint32_t* jump1 = jump0 + P;
  uint8_t* mark = reinterpret_cast<uint8_t*>(jump1 + P);
  unsigned long long* reg_tot = reinterpret_cast<unsigned long long*>(smem + 25 * (size_t)P);  // [R][2], 8-byte aligned: P >= 64
  unsigned long long* wg_tot = reg_tot + 2 * R;   // stages, latency, bubbles
  uint32_t* wg_small = reinterpret_cast<uint32_t*>(wg_tot + 3);  // [0] valid stages, [1] min start on the path, [2] a region's keys are out of order
  unsigned long long* all_tot = reinterpret_cast<unsigned long long*>(wg_small + 4);  // paths, stages, latency, bubbles

  const uint32_t tid = threadIdx.x, lane = tid & 63u;
  for (uint32_t i = tid; i < 2 * R; i += kBlock) reg_tot[i] = 0ull;
  if (tid < 4) all_tot[tid] = 0ull;
  __syncthreads();

  for (uint32_t wg = blockIdx.x; wg < p.n_wg; wg += gridDim.x) {
    const u32x4* tab = p.table + (size_t)wg * N;
    if (tid < 3) wg_tot[tid] = 0ull;
    if (tid == 0) { wg_small[0] = 0u; wg_small[1] = 0xFFFFFFFFu; wg_small[2] = 0u; }
    __syncthreads();
    // ---- 1: keys ----------------------------------------------------------------------------------
    // The iterations of a region usually end one after the other, so that the keys of a region (a run of I
    // consecutive entries) are in order as they come; that is checked while the keys are made (an entry that
    // is no stage has the largest key: it must be behind the stages of its run).
    uint32_t n_mine = 0;
    const bool runs = I >= 2u && (I & (I - 1u)) == 0u;  // runs that the merge steps below can start from
    bool disorder = false;
    for (uint32_t i = tid; i < P; i += kBlock) {
      unsigned long long k = ~0ull;
      if (i < N) {
        const u32x4 e = tab[i];
        start[i] = e.y; lat[i] = e.x;
        if (e.w != 0u) { k = ((unsigned long long)e.z << 32) | i; ++n_mine; }
        if (runs && (i & (I - 1u)) != 0u) {
          const u32x4 before = tab[i - 1u];
          const unsigned long long kb = before.w != 0u ? ((unsigned long long)before.z << 32) | (i - 1u) : ~0ull;
          disorder = disorder || kb > k;
        }
      }
      key[i] = k;
      mark[i] = 0;
    }
    n_mine = wave_sum32(n_mine);
    if (lane == 0 && n_mine) atomicAdd(&wg_small[0], n_mine);
    if (__builtin_amdgcn_ballot_w64(disorder) != 0ull && lane == 0) wg_small[2] = 1u;
    __syncthreads();
    // Ascending sort by merging: blocks of k/2 keys in order become blocks of k.  The first step of a merge
    // compares key i of the lower block with key k/2 - 1 - i of the upper one (the smaller k/2 keys of the
    // two end up below, the larger above, each a rising-then-falling sequence), the steps after it are the
    // half-cleaners of a bitonic merge.  With every region's run in order the merging starts at blocks of I.
    // A thread takes the pairs t = tid, tid + 256, ..., so the 64 pairs of a hardware wave lie in one block of
    // 128 consecutive keys whenever the two keys of a pair are at most 64 apart (and, in a first step, the
    // blocks hold at most 128 keys): such steps touch no key of another wave, and since the LDS operations
    // of one wave take effect in order, two of them in a row need no workgroup barrier between them.
    auto between = [&](bool local_before, bool local_after) {
      if (local_before && local_after) { __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront"); __builtin_amdgcn_wave_barrier(); }
      else __syncthreads();
    };
    for (uint32_t k = (runs && wg_small[2] == 0u) ? 2u * I : 2u; k <= P; k <<= 1) {
      const uint32_t half = k >> 1;
      for (uint32_t t = tid; t < P / 2; t += kBlock) {
        const uint32_t blk = (t / half) * k, i = t & (half - 1u), lo = blk + i, hi = blk + k - 1u - i;
        const unsigned long long a = key[lo], b = key[hi];
        if (a > b) { key[lo] = b; key[hi] = a; }
      }
      // (the step after this one: the half-cleaner at distance half / 2, or the first step of the next size)
      between(k <= 128u, half >= 2u ? (half >> 1) <= 64u : 2u * k <= 128u);
      for (uint32_t j = half >> 1; j > 0; j >>= 1) {
        for (uint32_t t = tid; t < P / 2; t += kBlock) {
          const uint32_t lo = ((t & ~(j - 1u)) << 1) | (t & (j - 1u));  // the element of the pair with bit j clear
          const uint32_t hi = lo | j;
          const unsigned long long a = key[lo], b = key[hi];
          if (a > b) { key[lo] = b; key[hi] = a; }
        }
        between(j <= 64u, j >= 2u ? true : 2u * k <= 128u);
      }
    }
    __syncthreads();
    const uint32_t n = wg_small[0];  // the stages are the first n keys
    // ---- 2: the stage each stage waited for -------------------------------------------------------
    for (uint32_t r = tid; r < P; r += kBlock) {
      uint32_t pred = kNone;
      if (r < n) {
        const uint32_t s = start[(uint32_t)key[r]];
        uint32_t lo = 0, hi = n;  // first rank whose end exceeds s
        while (lo < hi) {
          const uint32_t mid = (lo + hi) >> 1;
          if ((uint32_t)(key[mid] >> 32) <= s) lo = mid + 1; else hi = mid;
        }
        const uint32_t c = lo < r ? lo : r;
        pred = c ? c - 1u : kNone;
      }
      jump0[r] = pred;
      if (r + 1u == n) mark[r] = 1;
    }
    // ---- 3: mark the list that starts at the last stage --------------------------------------------
    uint32_t* cur = jump0;
    uint32_t* nxt = jump1;
    for (uint32_t round = 0; (1u << round) < n; ++round) {
      __syncthreads();
      for (uint32_t r = tid; r < n; r += kBlock) {
        const uint32_t j = cur[r];
        // (a stage marked in this very round may already act: it only marks stages of the list)
        if (j != kNone && mark[r]) mark[j] = 1;
        nxt[r] = j != kNone ? cur[j] : kNone;
      }
      uint32_t* t = cur; cur = nxt; nxt = t;
    }
    __syncthreads();
    // ---- 4: totals ---------------------------------------------------------------------------------
    // (the links of one step were overwritten by the doubling: they are found again, one search each)
    uint32_t my_n = 0, my_first = 0xFFFFFFFFu;
    unsigned long long my_lat = 0, my_bub = 0;
    for (uint32_t r = tid; r < n; r += kBlock) {
      if (!mark[r]) continue;
      const uint32_t idx = (uint32_t)key[r];
      const uint32_t s = start[idx], l = lat[idx];
      uint32_t lo = 0, hi = n;
      while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if ((uint32_t)(key[mid] >> 32) <= s) lo = mid + 1; else hi = mid;
      }
      const uint32_t c = lo < r ? lo : r;
      if (c) my_bub += s - (uint32_t)(key[c - 1u] >> 32);
      ++my_n; my_lat += l;
      my_first = s < my_first ? s : my_first;
      const uint32_t region = idx / I;
      atomicAdd(&reg_tot[2 * region], 1ull);
      atomicAdd(&reg_tot[2 * region + 1], (unsigned long long)l);
    }
    my_n = wave_sum32(my_n); my_lat = wave_sum64(my_lat); my_bub = wave_sum64(my_bub); my_first = wave_min32(my_first);
    if (lane == 0 && my_n) {
      atomicAdd(&wg_tot[0], (unsigned long long)my_n);
      atomicAdd(&wg_tot[1], my_lat);
      atomicAdd(&wg_tot[2], my_bub);
      atomicMin(&wg_small[1], my_first);
    }
    __syncthreads();
    if (tid == 0) {
      u32x4 a, b;
      if (n) {
        const unsigned long long last = key[n - 1u];
        const uint32_t idx = (uint32_t)last;
        a = u32x4{(uint32_t)wg_tot[0], ((idx / I) << 16) | (idx % I), wg_small[1], (uint32_t)(last >> 32)};
        all_tot[0] += 1ull;
      } else {
        a = u32x4{0u, 0xFFFFFFFFu, 0u, 0u};
      }
      b = u32x4{(uint32_t)wg_tot[1], (uint32_t)(wg_tot[1] >> 32), (uint32_t)wg_tot[2], (uint32_t)(wg_tot[2] >> 32)};
      p.rows[2 * (size_t)wg] = a;
      p.rows[2 * (size_t)wg + 1] = b;
      all_tot[1] += wg_tot[0]; all_tot[2] += wg_tot[1]; all_tot[3] += wg_tot[2];
    }
    __syncthreads();
  }
  for (uint32_t i = tid; i < 2 * R; i += kBlock)
    if (reg_tot[i]) atomicAdd(&p.region[i], reg_tot[i]);
  if (tid < 4 && all_tot[tid]) atomicAdd(&p.hdr[3 + tid], all_tot[tid]);
}

struct LaunchCache { int dev = -1; uint32_t lds = 0; uint32_t max_grid = 0; };

}  // namespace

extern "C" size_t kp_critical_bytes(int n_wg, int n_regions) {
  if (n_wg < 0 || n_regions < 1 || n_regions > 128) return 0;
  return 64 + 16 * (size_t)n_regions + 32 * (size_t)n_wg;
}

extern "C" kp_status kp_stages_critical(const void* stages, int n_wg, int n_regions, int max_iter, void* out_paths,
                                        void* stream) {
  kp::clear_error();
  if (!stages || !out_paths) return kp::fail(KP_ERR_INVALID_ARG, "NULL argument");
  if (n_wg < 0 || n_regions < 1 || n_regions > 128 || max_iter < 1 || max_iter > 65535)
    return kp::fail(KP_ERR_INVALID_ARG, "n_wg=%d regions=%d max_iter=%d", n_wg, n_regions, max_iter);
  if (((uintptr_t)stages & 15u) || ((uintptr_t)out_paths & 15u))
    return kp::fail(KP_ERR_INVALID_ARG, "stages and out_paths must be 16-byte aligned");
  const uint64_t n_ent = (uint64_t)n_regions * (uint64_t)max_iter;
  if (n_ent > kMaxEntries)
    return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "%d regions x %d iterations exceed %u stages per workgroup", n_regions, max_iter,
                    kMaxEntries);
  hipStream_t s = static_cast<hipStream_t>(stream);
  uint8_t* out = static_cast<uint8_t*>(out_paths);
  CriticalParams p;
  p.table = reinterpret_cast<const u32x4*>(static_cast<const uint8_t*>(stages) + 32);
  p.hdr = reinterpret_cast<unsigned long long*>(out);
  p.region = p.hdr + 8;
  p.rows = reinterpret_cast<u32x4*>(out + 64 + 16 * (size_t)n_regions);
  p.n_wg = (uint32_t)n_wg; p.R = (uint32_t)n_regions; p.I = (uint32_t)max_iter; p.N = (uint32_t)n_ent;
  p.P = 64; p.log2P = 6;
  while (p.P < p.N) { p.P <<= 1; ++p.log2P; }
  hipLaunchKernelGGL(kp_critical_init, dim3(1), dim3(256), 0, s, p.hdr, p.n_wg, p.R, p.I);
  KP_HIP_TRY(hipGetLastError());
  if (n_wg == 0) return KP_OK;
  const uint32_t lds = 25u * p.P + 16u * p.R + 24u + 16u + 32u;
  static thread_local LaunchCache cache;
  int dev = 0;
  KP_HIP_TRY(hipGetDevice(&dev));
  if (cache.dev != dev || cache.lds != lds) {
    KP_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kp_critical_main),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    int per_cu = 0, cus = 0;
    KP_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kp_critical_main, kBlock, lds));
    if (per_cu < 1) return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "critical-path kernel does not fit one CU (LDS %u B)", lds);
    KP_HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    cache.dev = dev; cache.lds = lds; cache.max_grid = (uint32_t)per_cu * (uint32_t)cus;
  }
  const uint32_t grid = cache.max_grid < (uint32_t)n_wg ? cache.max_grid : (uint32_t)n_wg;
  hipLaunchKernelGGL(kp_critical_main, dim3(grid), dim3(kBlock), lds, s, p);
  KP_HIP_TRY(hipGetLastError());
  return KP_OK;
}

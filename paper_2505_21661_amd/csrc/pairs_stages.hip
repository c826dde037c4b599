// Per-iteration stage table from the timeline rows (kp_pairs_stages).
//
// The paper's critical-path analysis and overlap models (Sec. 3.3 "Critical-path Analysis",
// Sec. 5.2 / Table 4) take the latency of every stage in every loop iteration.  A stage that the
// waves of a workgroup run together lasts as long as its slowest wave, so the rows {start, dur,
// iter, region} that kp_trace_pairs wrote for the waves of a workgroup are folded into one entry
// per (workgroup, region, iteration): {max dur, min start, max (start + dur), rows folded}.
//
// A streaming kernel: one decoder workgroup per recorded workgroup at a time (persistent, grid
// stride), its table in LDS.  Hardware wave h reads the rows of recorded waves h, h + 8, ... with
// 16-byte loads, four per lane and step and four steps in flight, and folds them with LDS atomics; the
// table then goes to
// HBM with 16-byte stores and is reset in the same pass.  The rows of a region are kept
// max_iter + 1 entries apart in LDS so that equal iterations of different regions use different banks.
#include "kp_common.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBlock = 512;
constexpr uint32_t kMaxTableBytes = 64 * 1024;

struct StagesParams {
  const uint32_t* count;  // rows per (workgroup, wave)
  const u32x4* rows;      // cap_wave / 2 row slots per (workgroup, wave)
  unsigned long long* hdr;  // n_rows, n_clipped, n_bad_region, 0
  u32x4* table;           // [n_wg][R][max_iter]
  uint32_t n_wg, W, R, half, max_iter;
};

__global__ void kp_stages_init(unsigned long long* hdr) {
  if (threadIdx.x < 4) hdr[threadIdx.x] = 0ull;
}

__device__ inline uint32_t wave_sum(uint32_t v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
  return v;
}

__global__ __launch_bounds__(kBlock) void kp_stages_main(StagesParams p) {
  extern __shared__ __align__(16) unsigned char smem[];
  uint32_t* tab = reinterpret_cast<uint32_t*>(smem);  // entry (r, it) at word 4 * (r * (max_iter + 1) + it)
  u32x4* tab4 = reinterpret_cast<u32x4*>(smem);
  const uint32_t tid = threadIdx.x, lane = tid & 63u, hw = tid >> 6;
  const uint32_t W = p.W, R = p.R, MI = p.max_iter, stride = MI + 1;
  const u32x4 empty = u32x4{0u, 0xFFFFFFFFu, 0u, 0u};

  for (uint32_t i = tid; i < R * stride; i += kBlock) tab4[i] = empty;
  __syncthreads();

  uint32_t n_rows = 0, n_clipped = 0, n_bad = 0;
  auto fold = [&](const u32x4& row) {
    const uint32_t start = row.x, dur = row.y, it = row.z, region = row.w;
    if (region >= R) { ++n_bad; return; }
    if (it >= MI) { ++n_clipped; return; }
    uint32_t* e = tab + 4 * (region * stride + it);
    atomicMax(e + 0, dur);
    atomicMin(e + 1, start);
    atomicMax(e + 2, start + dur);
    atomicAdd(e + 3, 1u);
    ++n_rows;
  };

  for (uint32_t wg = blockIdx.x; wg < p.n_wg; wg += gridDim.x) {
    for (uint32_t w = hw; w < W; w += kBlock / 64) {
      const size_t seg = (size_t)wg * W + w;
      uint32_t cnt = p.count[seg];
      cnt = cnt < p.half ? cnt : p.half;  // a count beyond the wave's slots cannot be honoured
      const u32x4* rows = p.rows + seg * p.half;
      // Four rows per lane and step, and the rows of the next three steps are requested before this
      // step's are folded, so that the folds (LDS atomics) run under the loads and a wave keeps 16 KiB
      // in flight (measured for 1.3e8 rows: 0.595 ms with one step in flight, 0.548 with two, 0.510
      // with three, 0.500 with four).  A row past the count is read from the wave's last valid row (or
      // not at all for an empty wave) and not folded.
      if (cnt == 0) continue;
      auto fetch = [&](uint32_t j0, u32x4 (&r)[4]) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const uint32_t j = j0 + 64u * u;
          r[u] = __builtin_nontemporal_load(rows + (j < cnt ? j : cnt - 1u));
        }
      };
      constexpr int kDepth = 4;
      u32x4 buf[kDepth][4];
#pragma unroll
      for (int d = 0; d < kDepth - 1; ++d)
        if (256u * d < cnt) fetch(lane + 256u * d, buf[d]);
      for (uint32_t j0 = lane; j0 - lane < cnt; j0 += 256) {
        if (j0 - lane + 256u * (kDepth - 1) < cnt) fetch(j0 + 256u * (kDepth - 1), buf[kDepth - 1]);
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (j0 + 64u * u < cnt) fold(buf[0][u]);
#pragma unroll
        for (int d = 0; d + 1 < kDepth; ++d)
#pragma unroll
          for (int u = 0; u < 4; ++u) buf[d][u] = buf[d + 1][u];
      }
    }
    __syncthreads();
    // ---- table to HBM, and reset for the next workgroup ----------------------------------------------
    u32x4* dst = p.table + (size_t)wg * R * MI;
    for (uint32_t i = tid; i < R * MI; i += kBlock) {
      const uint32_t r = i / MI, it = i - r * MI;
      const uint32_t at = r * stride + it;
      dst[i] = tab4[at];
      tab4[at] = empty;
    }
    __syncthreads();
  }

  n_rows = wave_sum(n_rows); n_clipped = wave_sum(n_clipped); n_bad = wave_sum(n_bad);
  if (lane == 0) {
    if (n_rows) atomicAdd(&p.hdr[0], (unsigned long long)n_rows);
    if (n_clipped) atomicAdd(&p.hdr[1], (unsigned long long)n_clipped);
    if (n_bad) atomicAdd(&p.hdr[2], (unsigned long long)n_bad);
  }
}

struct LaunchCache { int dev = -1; uint32_t lds = 0; uint32_t max_grid = 0; };

}  // namespace

extern "C" size_t kp_stages_bytes(int n_wg, int n_regions, int max_iter) {
  if (n_wg < 0 || n_regions < 1 || n_regions > 128 || max_iter < 1) return 0;
  return 32 + sizeof(kp_stage_row) * (size_t)n_wg * (size_t)n_regions * (size_t)max_iter;
}

extern "C" kp_status kp_pairs_stages(const void* pairs, int n_wg, int waves_per_wg, int cap_per_wg, int n_regions,
                                     int max_iter, void* out_stages, void* stream) {
  kp::clear_error();
  if (!pairs || !out_stages) return kp::fail(KP_ERR_INVALID_ARG, "NULL argument");
  if (n_wg < 0 || waves_per_wg < 1 || waves_per_wg > KP_MAX_WAVES || cap_per_wg < 2 * waves_per_wg ||
      cap_per_wg % waves_per_wg || n_regions < 1 || n_regions > 128 || max_iter < 1)
    return kp::fail(KP_ERR_INVALID_ARG, "n_wg=%d waves=%d cap=%d regions=%d max_iter=%d", n_wg, waves_per_wg,
                    cap_per_wg, n_regions, max_iter);
  if (((uintptr_t)pairs & 15u) || ((uintptr_t)out_stages & 15u))
    return kp::fail(KP_ERR_INVALID_ARG, "pairs and out_stages must be 16-byte aligned");
  const uint32_t lds = 16u * (uint32_t)n_regions * ((uint32_t)max_iter + 1u);
  if ((uint64_t)n_regions * ((uint64_t)max_iter + 1u) * 16u > kMaxTableBytes)
    return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "a table of %d regions x %d iterations exceeds %u bytes of LDS",
                    n_regions, max_iter, kMaxTableBytes);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const uint8_t* in = static_cast<const uint8_t*>(pairs);
  uint8_t* out = static_cast<uint8_t*>(out_stages);
  const size_t n_seg = (size_t)n_wg * waves_per_wg;
  StagesParams p;
  p.count = reinterpret_cast<const uint32_t*>(in);
  p.rows = reinterpret_cast<const u32x4*>(in + ((n_seg + 3) / 4) * 16);
  p.hdr = reinterpret_cast<unsigned long long*>(out);
  p.table = reinterpret_cast<u32x4*>(out + 32);
  p.n_wg = (uint32_t)n_wg; p.W = (uint32_t)waves_per_wg; p.R = (uint32_t)n_regions;
  p.half = (uint32_t)(cap_per_wg / waves_per_wg) / 2u; p.max_iter = (uint32_t)max_iter;

  hipLaunchKernelGGL(kp_stages_init, dim3(1), dim3(64), 0, s, p.hdr);
  KP_HIP_TRY(hipGetLastError());
  if (n_wg == 0) return KP_OK;

  static thread_local LaunchCache cache;
  int dev = 0;
  KP_HIP_TRY(hipGetDevice(&dev));
  if (cache.dev != dev || cache.lds != lds) {
    KP_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kp_stages_main),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    int per_cu = 0, cus = 0;
    KP_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kp_stages_main, kBlock, lds));
    if (per_cu < 1) return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "stage kernel does not fit one CU (LDS %u B)", lds);
    KP_HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    cache.dev = dev; cache.lds = lds; cache.max_grid = (uint32_t)per_cu * (uint32_t)cus;
  }
  uint32_t grid = cache.max_grid < (uint32_t)n_wg ? cache.max_grid : (uint32_t)n_wg;
  hipLaunchKernelGGL(kp_stages_main, dim3(grid), dim3(kBlock), lds, s, p);
  KP_HIP_TRY(hipGetLastError());
  return KP_OK;
}

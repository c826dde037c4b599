// Instrumented bf16 GEMM targets (kp_gemm_instrumented): C[M,N] = A[M,K] * B[K,N], fp32 accumulate,
// bf16 (round-to-nearest-even) output, all row-major.
//
// The paper profiles software-pipelined Triton GEMMs by inserting region records around the
// stages of the K loop (Sec. 5.3, GEMM-SWP-2/3; Sec. 2.3 software pipelining).  These kernels
// are this library's own MFMA GEMMs with hand-placed record sites.  Each exists twice from one
// template: INSTR=false compiles every record site away (the uninstrumented baseline),
// INSTR=true records into the LDS ring.  Record sites contain no floating point, so both
// variants produce bit-identical C.
//
//   tile 64x64x32, 4 waves  : regions 0 global load, 1 LDS store, 2 MFMA        (per K step)
//   tile 256x256x64, 8 waves: regions 0 load issue, 1 load wait, 2 LDS write, 3 MFMA (per K step),
//                              4 epilogue (once)
#include "kp_common.h"
#include "kp_record.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

struct GemmArgs {
  const uint16_t* A;
  const uint16_t* B;
  uint16_t* C;
  uint32_t M, N, K;
  uint32_t region_mask;
  void* trace;
  uint32_t cap_lds, cap_hbm, flush, n_wg;
};

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;  // NaN stays NaN
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}

// LDS tiles hold rows of BK bf16 (K contiguous) in 16-byte chunks; chunk c of row r lives at chunk
// position c ^ swz(r) so that the 16-byte reads of 32 different rows spread over all banks.
template <int BK>
__device__ __forceinline__ uint32_t tile_off(uint32_t row, uint32_t chunk) {
  constexpr uint32_t CPR = BK / 8;           // chunks per row
  constexpr uint32_t RPL = 128 / (BK * 2);   // rows per 128-byte bank line (BK <= 64)
  const uint32_t s = (row / RPL) % CPR;
  return row * (BK * 2) + ((chunk ^ s) * 16);  // byte offset
}

#define KP_REC(ring, region, phase) do { if constexpr (INSTR) kp::record(ring, region, phase); } while (0)

// ------------------------------------------------------------------------------------------
// 64x64x32 tile, 4 waves as 2x2, each wave one 32x32 accumulator tile.
template <bool INSTR>
__global__ __launch_bounds__(256) void kp_gemm_small(GemmArgs g) {
  constexpr int BM = 64, BN = 64, BK = 32;
  __shared__ __align__(16) unsigned char sA[BM * BK * 2];
  __shared__ __align__(16) unsigned char sB[BN * BK * 2];
  extern __shared__ __align__(16) uint32_t ring_lds[];
  __shared__ uint64_t t_begin[2];

  const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
  const uint32_t tiles_n = g.N / BN;
  const uint32_t wg = blockIdx.x;
  const uint32_t m0 = (wg / tiles_n) * BM, n0 = (wg % tiles_n) * BN;
  kp::Ring ring{};
  if constexpr (INSTR)
    ring = kp::ring_init(ring_lds, t_begin, g.cap_lds, g.region_mask, g.flush, g.cap_hbm, g.trace, g.n_wg, 4, wg);

  // global -> register mapping
  // A: 64 rows x 4 chunks = 256 chunks, one per thread
  const uint32_t a_row = tid >> 2, a_chunk = tid & 3u;
  const uint16_t* a_src = g.A + (size_t)(m0 + a_row) * g.K + a_chunk * 8;
  // B: 4 k-groups x 32 column pairs = 128 tasks; threads 128..255 idle for B
  const uint32_t b_kg = (tid >> 5) & 3u, b_np = tid & 31u;
  const bool b_on = tid < 128;
  const uint16_t* b_src = g.B + (size_t)(b_kg * 8) * g.N + n0 + b_np * 2;

  const uint32_t wr = wave >> 1, wc = wave & 1u;  // wave position in the 2x2 grid
  f32x16 acc = {0};

  for (uint32_t kt = 0; kt < g.K / BK; ++kt) {
    // ---- region 0: global load ---------------------------------------------------------------
    KP_REC(ring, 0, kp::kPhaseStart);
    const u32x4 av = *reinterpret_cast<const u32x4*>(a_src + (size_t)kt * BK);
    uint32_t bv[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
      bv[i] = b_on ? *reinterpret_cast<const uint32_t*>(b_src + ((size_t)kt * BK + i) * g.N) : 0u;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    KP_REC(ring, 0, kp::kPhaseEnd);
    // ---- region 1: LDS store -----------------------------------------------------------------
    KP_REC(ring, 1, kp::kPhaseStart);
    __syncthreads();  // previous step's MFMA reads are done
    *reinterpret_cast<u32x4*>(sA + tile_off<BK>(a_row, a_chunk)) = av;
    if (b_on) {
      u32x4 lo, hi;  // column 2*b_np and 2*b_np+1, eight consecutive k each
      lo.x = (bv[0] & 0xFFFFu) | (bv[1] << 16); hi.x = (bv[0] >> 16) | (bv[1] & 0xFFFF0000u);
      lo.y = (bv[2] & 0xFFFFu) | (bv[3] << 16); hi.y = (bv[2] >> 16) | (bv[3] & 0xFFFF0000u);
      lo.z = (bv[4] & 0xFFFFu) | (bv[5] << 16); hi.z = (bv[4] >> 16) | (bv[5] & 0xFFFF0000u);
      lo.w = (bv[6] & 0xFFFFu) | (bv[7] << 16); hi.w = (bv[6] >> 16) | (bv[7] & 0xFFFF0000u);
      *reinterpret_cast<u32x4*>(sB + tile_off<BK>(b_np * 2, b_kg)) = lo;
      *reinterpret_cast<u32x4*>(sB + tile_off<BK>(b_np * 2 + 1, b_kg)) = hi;
    }
    __syncthreads();
    KP_REC(ring, 1, kp::kPhaseEnd);
    // ---- region 2: MFMA ------------------------------------------------------------------------
    KP_REC(ring, 2, kp::kPhaseStart);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      // operand layout of v_mfma_f32_32x32x16_bf16: lane l supplies row/column l%32, k = 8*(l/32)..+7
      const uint32_t chunk = ks * 2 + (lane >> 5);
      const bf16x8 af = *reinterpret_cast<const bf16x8*>(sA + tile_off<BK>(wr * 32 + (lane & 31u), chunk));
      const bf16x8 bf = *reinterpret_cast<const bf16x8*>(sB + tile_off<BK>(wc * 32 + (lane & 31u), chunk));
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bf, acc, 0, 0, 0);
    }
    asm volatile("s_nop 0" ::: "memory");
    KP_REC(ring, 2, kp::kPhaseEnd);
  }

  // epilogue: accumulator register v of lane l is C[row, col] with col = l%32,
  // row = 8*(v/4) + 4*(l/32) + v%4 inside the wave's 32x32 tile
  const uint32_t col = n0 + wc * 32 + (lane & 31u);
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const uint32_t row = m0 + wr * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v % 4);
    g.C[(size_t)row * g.N + col] = (uint16_t)f32_to_bf16_rne(acc[v]);
  }
  if constexpr (INSTR) {
    kp::TraceGeom tg{g.n_wg, 4, 3, g.cap_hbm, g.flush ? KP_FLAG_FLUSH : 0u};
    kp::ring_finish(ring, ring_lds, t_begin, g.cap_lds, g.trace, tg, wg, 0u);
  }
}

}  // namespace

// ------------------------------------------------------------------------------------------
namespace {

struct GemmShape { int bm, bn, bk, waves, regions; };

bool pick_shape(int M, int N, int K, GemmShape* s) {
  if (M <= 0 || N <= 0 || K <= 0) return false;
  if (M % 64 == 0 && N % 64 == 0 && K % 32 == 0) { *s = GemmShape{64, 64, 32, 4, 3}; return true; }
  return false;
}

}  // namespace

extern "C" kp_status kp_gemm_launch_shape(int M, int N, int K, int* n_wg, int* waves_per_wg, int* n_regions) {
  kp::clear_error();
  GemmShape s;
  if (!pick_shape(M, N, K, &s))
    return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "GEMM %dx%dx%d: M,N must be multiples of 64 and K of 32", M, N, K);
  if (n_wg) *n_wg = (M / s.bm) * (N / s.bn);
  if (waves_per_wg) *waves_per_wg = s.waves;
  if (n_regions) *n_regions = s.regions;
  return KP_OK;
}

extern "C" kp_status kp_gemm_instrumented(const void* A, const void* B, void* C, int M, int N, int K,
                                          uint32_t region_mask, void* trace_buf, size_t trace_cap,
                                          void* stream) {
  kp::clear_error();
  if (!A || !B || !C) return kp::fail(KP_ERR_INVALID_ARG, "NULL matrix pointer");
  GemmShape s;
  if (!pick_shape(M, N, K, &s))
    return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "GEMM %dx%dx%d: M,N must be multiples of 64 and K of 32", M, N, K);
  if (((uintptr_t)A | (uintptr_t)B | (uintptr_t)C) & 15u) return kp::fail(KP_ERR_INVALID_ARG, "A, B, C must be 16-byte aligned");
  const uint32_t regions = region_mask & 0x7FFFFFFFu;
  const uint32_t flush = region_mask >> 31;
  const int n_wg = (M / s.bm) * (N / s.bn);
  hipStream_t st = static_cast<hipStream_t>(stream);
  GemmArgs g{};
  g.A = static_cast<const uint16_t*>(A); g.B = static_cast<const uint16_t*>(B); g.C = static_cast<uint16_t*>(C);
  g.M = (uint32_t)M; g.N = (uint32_t)N; g.K = (uint32_t)K;
  g.region_mask = regions; g.trace = trace_buf; g.n_wg = (uint32_t)n_wg; g.flush = flush;
  if (regions == 0) {  // uninstrumented baseline: no ring, no record sites
    hipLaunchKernelGGL(kp_gemm_small<false>, dim3(n_wg), dim3(256), 0, st, g);
    KP_HIP_TRY(hipGetLastError());
    return KP_OK;
  }
  if (!trace_buf) return kp::fail(KP_ERR_INVALID_ARG, "trace_buf is NULL but region_mask enables regions");
  if (regions >> s.regions) return kp::fail(KP_ERR_INVALID_ARG, "region_mask enables regions this kernel does not have (%d regions)", s.regions);
  if (((uintptr_t)trace_buf) & 15u) return kp::fail(KP_ERR_INVALID_ARG, "trace_buf must be 16-byte aligned");
  if (trace_cap % (size_t)s.waves) return kp::fail(KP_ERR_TRACE_TOO_SMALL, "trace_cap must be a multiple of %d waves", s.waves);
  const size_t cap_wave = trace_cap / (size_t)s.waves;
  if (!kp::is_pow2(cap_wave) || cap_wave < 2 || cap_wave > (1u << 19))
    return kp::fail(KP_ERR_TRACE_TOO_SMALL, "trace_cap/waves = %zu must be a power of two >= 2", cap_wave);
  uint32_t cap_lds = (uint32_t)cap_wave;
  if (flush && cap_lds > 64) cap_lds = 64;
  const size_t ring_bytes = (size_t)cap_lds * 8 * s.waves;
  if (ring_bytes > 32 * 1024) return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "LDS ring of %zu bytes exceeds the 32 KiB budget", ring_bytes);
  g.cap_lds = cap_lds; g.cap_hbm = (uint32_t)cap_wave;
  hipLaunchKernelGGL(kp_gemm_small<true>, dim3(n_wg), dim3(256), ring_bytes, st, g);
  KP_HIP_TRY(hipGetLastError());
  return KP_OK;
}

// Instrumented bf16 attention forward (kp_attn_instrumented): O = softmax(scale * Q K^T + mask) V,
// fp32 softmax and accumulation, head dimension 128, optional causal mask.
//
// The paper's case study profiles a flash-attention kernel whose regions are the two GEMMs and
// the softmax of every KV iteration (Sec. 5.2, Table 3: GEMM0 = Q K^T, softmax, GEMM1 = P V).
// This is the library's own MFMA kernel with the same three regions per KV tile of 64:
//   region 0  S^T = K Q^T     (MFMA)
//   region 1  online softmax   (VALU, fp32)
//   region 2  O^T += V^T P^T   (MFMA)
// One workgroup = 4 waves = 128 query rows of one (batch, head); each wave owns 32 rows.  The
// products are formed transposed so that a lane holds all scores of ONE query row: the row
// maximum and sum are then in-lane reductions plus one exchange with the lane 32 away, and the
// rescaling of the output accumulators is a per-lane multiply.
#include "kp_common.h"
#include "kp_record.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

struct AttnArgs {
  const uint16_t* Q;
  const uint16_t* K;
  const uint16_t* V;
  uint16_t* O;
  uint32_t B, H, S;
  uint32_t causal;
  float scale_log2;  // scale * log2(e)
  uint32_t region_mask;
  void* trace;
  uint32_t cap_lds, cap_hbm, flush, n_wg;
};

constexpr int kD = 128, kBq = 128, kBkv = 64, kAttnThreads = 256;
constexpr uint32_t kKBytes = kBkv * kD * 2;   // K tile   [64 kv][128 d]
constexpr uint32_t kVBytes = kD * kBkv * 2;   // V^T tile [128 d][64 kv]

// fp32 -> bf16, round to nearest even (v_cvt_pk_bf16_f32 on gfx950)
__device__ __forceinline__ uint32_t bf16_rne(float f) {
  const __bf16 h = (__bf16)f;
  return (uint32_t)__builtin_bit_cast(uint16_t, h);
}

// K tile: rows of 256 bytes (16 chunks of 16 B); V^T tile: rows of 128 bytes (8 chunks).
// Chunk c of row r is stored at chunk position c ^ (r & 7) so 16-byte reads of 8 neighbouring
// rows cover all LDS banks.
__device__ __forceinline__ uint32_t k_off(uint32_t row, uint32_t chunk) { return row * 256u + ((chunk ^ (row & 7u)) << 4); }
__device__ __forceinline__ uint32_t v_off(uint32_t row, uint32_t chunk) { return row * 128u + ((chunk ^ (row & 7u)) << 4); }

// END of one region and/or START of the next with a single clock sample.  INSTR: 0 no record sites,
// 1 generic sites (region mask, either buffer strategy), 2 lean sites (all regions, circular).
#define KP_BOUNDARY(ring, end_r, start_r) do { if constexpr (INSTR != 0) kp::site<INSTR>(ring, end_r, start_r); } while (0)

template <int INSTR>
__global__ __launch_bounds__(kAttnThreads, 2) void kp_attn_fwd(AttnArgs g) {
  extern __shared__ __align__(16) unsigned char smem[];  // [K tile][V^T tile][ring]
  unsigned char* sK = smem;
  unsigned char* sV = smem + kKBytes;
  uint32_t* ring_lds = reinterpret_cast<uint32_t*>(smem + kKBytes + kVBytes);

  const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
  const uint32_t h32 = lane >> 5, l32 = lane & 31u;
  const uint32_t q_blocks = g.S / kBq;
  const uint32_t wg = blockIdx.x;
  // long (late) query blocks first: causal work per block grows with its index
  const uint32_t qb = q_blocks - 1u - (wg % q_blocks);
  const uint32_t bh = wg / q_blocks;
  const size_t head = (size_t)bh * g.S * kD;
  const uint32_t q0 = qb * kBq;

  kp::Ring ring{};
  if constexpr (INSTR != 0)
    ring = kp::ring_init(ring_lds, reinterpret_cast<uint64_t*>(smem), g.cap_lds, g.region_mask, g.flush,
                         g.cap_hbm, g.trace, g.n_wg, 4, wg);

  // Q fragments of this wave's 32 rows stay in registers: step s covers d = 16s .. 16s+15
  const uint32_t qrow = q0 + wave * 32 + l32;
  bf16x8 qf[8];
#pragma unroll
  for (int s = 0; s < 8; ++s)
    qf[s] = *reinterpret_cast<const bf16x8*>(g.Q + head + (size_t)qrow * kD + 16 * s + 8 * h32);

  // global -> LDS mapping
  // K: 64 rows x 16 chunks; thread takes chunk (tid & 15) of rows (tid >> 4) + 16*i
  const uint32_t k_row = tid >> 4, k_chunk = tid & 15u;
  // V: tasks (kv group of 8, d pair): id = tid + 256*j, group = id >> 6, pair = id & 63
  const uint32_t v_pair = tid & 63u, v_grp0 = tid >> 6;  // second task: group + 4
  u32x4 k_reg[4];
  uint32_t v_reg[2][8];
  auto load_tile = [&](uint32_t kv0) {
    const uint16_t* kp_ = g.K + head + (size_t)(kv0 + k_row) * kD + k_chunk * 8;
#pragma unroll
    for (int i = 0; i < 4; ++i) k_reg[i] = *reinterpret_cast<const u32x4*>(kp_ + (size_t)(16 * i) * kD);
    const uint16_t* vp = g.V + head + (size_t)(kv0 + v_grp0 * 8) * kD + v_pair * 2;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 8; ++r) v_reg[j][r] = *reinterpret_cast<const uint32_t*>(vp + (size_t)(32 * j + r) * kD);
  };
  auto store_tile = [&]() {
#pragma unroll
    for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4*>(sK + k_off(k_row + 16 * i, k_chunk)) = k_reg[i];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const uint32_t* bv = v_reg[j];
      u32x4 lo, hi;  // d = 2*pair and 2*pair+1, eight consecutive kv each
      lo.x = (bv[0] & 0xFFFFu) | (bv[1] << 16); hi.x = (bv[0] >> 16) | (bv[1] & 0xFFFF0000u);
      lo.y = (bv[2] & 0xFFFFu) | (bv[3] << 16); hi.y = (bv[2] >> 16) | (bv[3] & 0xFFFF0000u);
      lo.z = (bv[4] & 0xFFFFu) | (bv[5] << 16); hi.z = (bv[4] >> 16) | (bv[5] & 0xFFFF0000u);
      lo.w = (bv[6] & 0xFFFFu) | (bv[7] << 16); hi.w = (bv[6] >> 16) | (bv[7] & 0xFFFF0000u);
      *reinterpret_cast<u32x4*>(sV + v_off(v_pair * 2, v_grp0 + 4 * j)) = lo;
      *reinterpret_cast<u32x4*>(sV + v_off(v_pair * 2 + 1, v_grp0 + 4 * j)) = hi;
    }
  };

  f32x16 oacc[4];  // O^T tiles: rows d = 32*dt + 8j + 4h + i, column q = lane % 32
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) oacc[dt] = f32x16{0};
  float m_run = -INFINITY, l_run = 0.f;

  const uint32_t n_tiles = g.causal ? (q0 + kBq) / kBkv : g.S / kBkv;
  load_tile(0);
  for (uint32_t t = 0; t < n_tiles; ++t) {
    const uint32_t kv0 = t * kBkv;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();  // every wave is done with the previous tile
    store_tile();
    __syncthreads();
    if (t + 1 < n_tiles) load_tile(kv0 + kBkv);  // in flight during the three regions below

    // ---- region 0: S^T = K Q^T --------------------------------------------------------------------
    KP_BOUNDARY(ring, kp::kNoRegion, 0);
    f32x16 sacc[2];
    sacc[0] = f32x16{0}; sacc[1] = f32x16{0};
#pragma unroll
    for (int s = 0; s < 8; ++s) {
#pragma unroll
      for (int tk = 0; tk < 2; ++tk) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(sK + k_off(32 * tk + l32, 2 * s + h32));
        sacc[tk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], sacc[tk], 0, 0, 0);
      }
    }
    KP_BOUNDARY(ring, 0, 1);

    // ---- region 1: online softmax (this lane: query row qrow, 32 of the tile's 64 kv) -------------
    const bool diag = g.causal && (kv0 + kBkv > q0 + wave * 32);  // tile reaches past this wave's first row
    float mx = -INFINITY;
#pragma unroll
    for (int tk = 0; tk < 2; ++tk)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        float sv = sacc[tk][v] * g.scale_log2;
        if (diag) {
          const uint32_t kv = kv0 + 32 * tk + 8 * (v >> 2) + 4 * h32 + (v & 3);
          if (kv > qrow) sv = -INFINITY;
        }
        sacc[tk][v] = sv;
        mx = fmaxf(mx, sv);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);  // m_new is finite: kv = 0 is visible to every row
    float psum = 0.f;
    uint32_t pk[2][8];  // P as packed bf16 pairs, in accumulator order
#pragma unroll
    for (int tk = 0; tk < 2; ++tk)
#pragma unroll
      for (int v = 0; v < 16; v += 2) {
        const float p0 = __builtin_amdgcn_exp2f(sacc[tk][v] - m_new);
        const float p1 = __builtin_amdgcn_exp2f(sacc[tk][v + 1] - m_new);
        const uint32_t b0 = bf16_rne(p0), b1 = bf16_rne(p1);
        // the sum uses the rounded values that enter the P V product
        psum += __uint_as_float(b0 << 16) + __uint_as_float(b1 << 16);
        pk[tk][v >> 1] = b0 | (b1 << 16);
      }
    l_run = l_run * alpha + psum;
    // the running maximum settles after a few tiles; skip the rescale when no row of this wave moved
    if (__builtin_amdgcn_ballot_w64(m_new != m_run) != 0ull) {
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[dt][v] *= alpha;
    }
    m_run = m_new;
    KP_BOUNDARY(ring, 1, 2);

    // ---- region 2: O^T += V^T P^T ---------------------------------------------------------------------
    // The kv order inside an MFMA step follows the accumulator layout of S^T (kv = 16s + 4h + e for
    // e < 4, 16s + 8 + 4h + e - 4 otherwise), so P needs no cross-lane movement; V^T is read to match.
#pragma unroll
    for (int tk = 0; tk < 2; ++tk)
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        u32x4 pw;
        pw.x = pk[tk][4 * s + 0]; pw.y = pk[tk][4 * s + 1]; pw.z = pk[tk][4 * s + 2]; pw.w = pk[tk][4 * s + 3];
        const bf16x8 pf = __builtin_bit_cast(bf16x8, pw);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
          const uint32_t row = 32 * dt + l32;
          const uint32_t c1 = 4 * tk + 2 * s;
          u32x4 vw;
          const u32x2 a = *reinterpret_cast<const u32x2*>(sV + v_off(row, c1) + 8 * h32);
          const u32x2 b = *reinterpret_cast<const u32x2*>(sV + v_off(row, c1 + 1) + 8 * h32);
          vw.x = a.x; vw.y = a.y; vw.z = b.x; vw.w = b.y;
          oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vw), pf, oacc[dt], 0, 0, 0);
        }
      }
    KP_BOUNDARY(ring, 2, kp::kNoRegion);
  }

  // epilogue: O[q][d] = O^T[d][q] / l
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = 1.0f / l_tot;
  uint16_t* orow = g.O + head + (size_t)qrow * kD;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      u32x2 pk2;
      pk2.x = bf16_rne(oacc[dt][4 * q + 0] * inv) | (bf16_rne(oacc[dt][4 * q + 1] * inv) << 16);
      pk2.y = bf16_rne(oacc[dt][4 * q + 2] * inv) | (bf16_rne(oacc[dt][4 * q + 3] * inv) << 16);
      *reinterpret_cast<u32x2*>(orow + 32 * dt + 8 * q + 4 * h32) = pk2;
    }
  if constexpr (INSTR != 0) {
    kp::TraceGeom tg{g.n_wg, 4, 3, g.cap_hbm, g.flush ? KP_FLAG_FLUSH : 0u};
    kp::ring_finish(ring, g.cap_lds, g.trace, tg, wg, 0u);
  }
}

bool attn_shape_ok(int B, int H, int S, int D) {
  return B > 0 && H > 0 && S > 0 && D == kD && S % kBq == 0 && (long long)B * H * (S / kBq) < (1ll << 31);
}

}  // namespace

extern "C" kp_status kp_attn_launch_shape(int B, int H, int S, int D, int* n_wg, int* waves_per_wg, int* n_regions) {
  kp::clear_error();
  if (!attn_shape_ok(B, H, S, D))
    return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "attention B=%d H=%d S=%d D=%d: D must be 128 and S a multiple of 128", B, H, S, D);
  if (n_wg) *n_wg = B * H * (S / kBq);
  if (waves_per_wg) *waves_per_wg = 4;
  if (n_regions) *n_regions = 3;
  return KP_OK;
}

extern "C" kp_status kp_attn_instrumented(const void* Q, const void* K, const void* V, void* O, int B, int H,
                                          int S, int D, int causal, float scale, uint32_t region_mask,
                                          void* trace_buf, size_t trace_cap, void* stream) {
  kp::clear_error();
  if (!Q || !K || !V || !O) return kp::fail(KP_ERR_INVALID_ARG, "NULL tensor pointer");
  if (!attn_shape_ok(B, H, S, D))
    return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "attention B=%d H=%d S=%d D=%d: D must be 128 and S a multiple of 128", B, H, S, D);
  if (((uintptr_t)Q | (uintptr_t)K | (uintptr_t)V | (uintptr_t)O) & 15u)
    return kp::fail(KP_ERR_INVALID_ARG, "Q, K, V, O must be 16-byte aligned");
  if (!(scale > 0.f) || scale > 1e30f) return kp::fail(KP_ERR_INVALID_ARG, "scale must be positive and finite");
  const uint32_t regions = region_mask & 0x7FFFFFFFu, flush = region_mask >> 31;
  const int n_wg = B * H * (S / kBq);
  hipStream_t st = static_cast<hipStream_t>(stream);
  AttnArgs g{};
  g.Q = static_cast<const uint16_t*>(Q); g.K = static_cast<const uint16_t*>(K);
  g.V = static_cast<const uint16_t*>(V); g.O = static_cast<uint16_t*>(O);
  g.B = (uint32_t)B; g.H = (uint32_t)H; g.S = (uint32_t)S; g.causal = causal ? 1u : 0u;
  g.scale_log2 = scale * 1.4426950408889634f;
  g.region_mask = regions; g.trace = trace_buf; g.flush = flush; g.n_wg = (uint32_t)n_wg;
  const uint32_t tile_bytes = kKBytes + kVBytes;
  if (regions == 0) {
    hipLaunchKernelGGL(kp_attn_fwd<0>, dim3(n_wg), dim3(kAttnThreads), tile_bytes, st, g);
    KP_HIP_TRY(hipGetLastError());
    return KP_OK;
  }
  if (!trace_buf) return kp::fail(KP_ERR_INVALID_ARG, "trace_buf is NULL but region_mask enables regions");
  if (regions >> 3) return kp::fail(KP_ERR_INVALID_ARG, "region_mask enables regions this kernel does not have (3 regions)");
  if (((uintptr_t)trace_buf) & 15u) return kp::fail(KP_ERR_INVALID_ARG, "trace_buf must be 16-byte aligned");
  if (trace_cap % 4) return kp::fail(KP_ERR_TRACE_TOO_SMALL, "trace_cap must be a multiple of 4 waves");
  const size_t cap_wave = trace_cap / 4;
  if (!kp::is_pow2(cap_wave) || cap_wave < 2 || cap_wave > (1u << 19))
    return kp::fail(KP_ERR_TRACE_TOO_SMALL, "trace_cap/waves = %zu must be a power of two >= 2", cap_wave);
  uint32_t cap_lds = (uint32_t)cap_wave;
  if (flush && cap_lds > 64) cap_lds = 64;
  const size_t ring_bytes = (size_t)cap_lds * 8 * 4;
  if (ring_bytes > 32 * 1024) return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "LDS ring of %zu bytes exceeds the 32 KiB budget", ring_bytes);
  g.cap_lds = cap_lds; g.cap_hbm = (uint32_t)cap_wave;
  static thread_local bool attr_set = false;
  if (!attr_set) {
    KP_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kp_attn_fwd<1>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024));
    KP_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kp_attn_fwd<2>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024));
    attr_set = true;
  }
  if (!flush && regions == 7u)  // every region, circular: lean record sites
    hipLaunchKernelGGL(kp_attn_fwd<2>, dim3(n_wg), dim3(kAttnThreads), tile_bytes + ring_bytes, st, g);
  else
    hipLaunchKernelGGL(kp_attn_fwd<1>, dim3(n_wg), dim3(kAttnThreads), tile_bytes + ring_bytes, st, g);
  KP_HIP_TRY(hipGetLastError());
  return KP_OK;
}

// Instrumented bf16 attention forward (kp_attn_instrumented): O = softmax(scale * Q K^T + mask) V,
// fp32 softmax and accumulation, head dimension 128, optional causal mask.
//
// The paper's case study profiles a flash-attention kernel whose regions are the two GEMMs and
// the softmax of every KV iteration (Sec. 5.2, Table 3: GEMM0 = Q K^T, softmax, GEMM1 = P V).
// This is the library's own MFMA kernel with the same three regions per KV tile of 64:
//   region 0  S^T = K Q^T     (MFMA); from the second tile on it opens with the barrier that makes
//             the K tile visible
//   region 1  online softmax   (VALU, fp32); opens with the barrier and LDS writes that stage the
//             next K tile, which overlap the other waves' softmax
//   region 2  O^T += V^T P^T   (MFMA)
// One workgroup = 4 waves = 128 query rows of one (batch, head); each wave owns 32 rows.  The
// products are formed transposed so that a lane holds all scores of ONE query row: the row
// maximum and sum are then in-lane reductions plus one exchange with the lane 32 away, and the
// rescaling of the output accumulators is a per-lane multiply.
#include <type_traits>

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
  uint32_t rec_cost;  // ticks the decoder takes off every duration (kp_set_rec_cost)
  uint32_t group_log2;  // 2^group_log2 waves share one record stream
  uint32_t collab;      // 1: all lanes store a record, hardware ids go to the workgroup header
  uint32_t flags;       // kp_trace_hdr.flags of the trace
};

constexpr int kD = 128, kBq = 128, kBkv = 64, kAttnThreads = 256;
constexpr uint32_t kKRow = kD * 2 + 16;        // K tile row: 256 bytes of data + 16 of padding
constexpr uint32_t kKBytes = kBkv * kKRow;    // K tile   [64 kv][128 d]
constexpr uint32_t kVBytes = kD * kBkv * 2;   // V^T tile [128 d][64 kv]
constexpr float kSlack = 8.0f;                // log2 of how far a score may exceed the softmax reference

// two fp32 -> packed bf16 pair (lo in bits 15:0), round to nearest even: one v_cvt_pk_bf16_f32
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t bf16_pack_rne(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// K tile: rows of 256 bytes (16 chunks of 16 B) plus 16 bytes of padding, so that the 16-byte reads
// of 8 neighbouring rows cover all LDS banks and every read address of a lane is a constant away
// from the lane's first one (an XOR swizzle would cost one vector instruction per read).
__device__ __forceinline__ uint32_t k_off(uint32_t row, uint32_t chunk) { return row * kKRow + (chunk << 4); }
// V^T tile: rows of 128 bytes (8 chunks of 16 B).  Within each group of 16 kv the four quads are
// stored in the order 0, 2, 1, 3, so chunk 2g + h holds exactly the eight kv an MFMA step of the
// P V product takes from lane half h.  The position also folds in row >> 3, because the transposing
// writes hit rows that are 8 apart; rows 64..127 keep the two 8-byte halves of a chunk swapped so
// that those writes spread over all banks.
__device__ __forceinline__ uint32_t v_off(uint32_t row, uint32_t chunk) {
  return row * 128u + ((chunk ^ ((row ^ (row >> 3)) & 7u)) << 4);
}

// END of one region and/or START of the next with a single clock sample.  INSTR: 0 no record sites,
// 1 generic sites (region mask, either buffer strategy, either store), 3 the same on the constant-rate clock,
// 4 chained sites (circular strategy, one lane stores; region mask and wave-group records included: the loop
// keeps only the clocks and the records are made when the trace is copied out), 5 chained, constant-rate clock.
#define KP_BOUNDARY(ring, end_r, start_r) do { if constexpr (INSTR == 1 || INSTR == 3) kp::site<INSTR>(ring, end_r, start_r); } while (0)
#define KP_CHAIN(K, ring) do { if constexpr (INSTR >= 4) kp::site_chain<K, (INSTR == 5)>(ring); } while (0)

// The sequence of record sites: one ahead of the loop (opens region 0), three per KV tile, the last only closes.
struct AttnChain {
  static constexpr uint32_t kRegions = 3u, kLead = 0u;
  static constexpr bool kDense = true;
  // n = 3 tiles + 1: every enabled region leaves two records per tile
  __device__ uint32_t total(uint32_t n, uint32_t mask) const { return 2u * ((n - 1u) / 3u) * (uint32_t)__builtin_popcount(mask & 7u); }
  __device__ uint32_t end_region(uint32_t site, uint32_t) const { return site == 0u ? kp::kNoRegion : (site - 1u) % 3u; }
  __device__ uint32_t start_region(uint32_t site, uint32_t n) const { return site + 1u == n ? kp::kNoRegion : site % 3u; }
};

template <int INSTR>
__global__ __launch_bounds__(kAttnThreads, 2) void kp_attn_fwd(AttnArgs g) {
  extern __shared__ __align__(16) unsigned char smem[];  // [K tile][V^T tile][ring]
  unsigned char* sK = smem;
  unsigned char* sV = smem + kKBytes;
  uint32_t* ring_lds = reinterpret_cast<uint32_t*>(smem + kKBytes + kVBytes);

  const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
  const uint32_t h32 = lane >> 5, l32 = lane & 31u;
  const uint32_t q_blocks = g.S / kBq;
  // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  All query blocks of a
  // (batch, head) go to one XCD, one head after the other, so that its K and V (2 MiB) are fetched
  // into one L2 once instead of into all eight.  `wg` is the recorded workgroup: head-major.
  uint32_t wg = blockIdx.x;
  if (((g.n_wg / q_blocks) & 7u) == 0u) {
    const uint32_t xcd = blockIdx.x & 7u, j = blockIdx.x >> 3;
    wg = ((j / q_blocks) * 8u + xcd) * q_blocks + j % q_blocks;
  }
  // long (late) query blocks first: causal work per block grows with its index
  const uint32_t qb = q_blocks - 1u - (wg % q_blocks);
  const uint32_t bh = wg / q_blocks;
  const size_t head = (size_t)bh * g.S * kD;
  const uint32_t q0 = qb * kBq;

  kp::Ring ring{};
  if constexpr (INSTR != 0)
    ring = kp::ring_init<true>(ring_lds, reinterpret_cast<uint64_t*>(smem), g.cap_lds, g.region_mask, g.flush,
                         g.cap_hbm, g.trace, g.n_wg, 4u >> g.group_log2, wg, g.group_log2);
  ring.collab = g.collab;
  if constexpr (INSTR == 3 || INSTR == 5) kp::ring_use_realtime(ring);
  // (with wave groups the host adds 16 bytes behind the ring for the waves that do not record)
  if constexpr (INSTR >= 4) kp::chain_begin(ring, (uint32_t)(uintptr_t)ring_lds + (4u >> g.group_log2) * g.cap_lds * 8u);

  // Q fragments of this wave's 32 rows stay in registers: step s covers d = 16s .. 16s+15
  const uint32_t qrow = q0 + wave * 32 + l32;
  bf16x8 qf[8];
#pragma unroll
  for (int s = 0; s < 8; ++s)
    qf[s] = *reinterpret_cast<const bf16x8*>(g.Q + head + (size_t)qrow * kD + 16 * s + 8 * h32);

  // global -> LDS mapping
  // K: 64 rows x 16 chunks; thread takes chunk (tid & 15) of rows (tid >> 4) + 16*i
  const uint32_t k_row = tid >> 4, k_chunk = tid & 15u;
  // V: thread takes 8 d (group tid & 15) of 4 consecutive kv (quad tid >> 4) and writes them transposed
  const uint32_t v_dg = tid & 15u, v_kq = tid >> 4;
  u32x4 k_reg[4], v_reg[4];
  auto load_k = [&](uint32_t kv0) {
    const uint16_t* kp_ = g.K + head + (size_t)(kv0 + k_row) * kD + k_chunk * 8;
#pragma unroll
    for (int i = 0; i < 4; ++i) k_reg[i] = *reinterpret_cast<const u32x4*>(kp_ + (size_t)(16 * i) * kD);
  };
  auto load_v = [&](uint32_t kv0) {
    const uint16_t* vp = g.V + head + (size_t)(kv0 + v_kq * 4) * kD + v_dg * 8;
#pragma unroll
    for (int i = 0; i < 4; ++i) v_reg[i] = *reinterpret_cast<const u32x4*>(vp + (size_t)i * kD);
  };
  auto store_k = [&]() {
#pragma unroll
    for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4*>(sK + k_off(k_row + 16 * i, k_chunk)) = k_reg[i];
  };
  auto store_v = [&]() {
    const uint32_t chunk = (v_kq >> 2) * 2u + (v_kq & 1u);
    const uint32_t half = ((v_kq >> 1) ^ (v_dg >> 3)) & 1u;
#pragma unroll
    for (int j = 0; j < 4; ++j) {  // word j of every row: d = 8*dg + 2j (low half) and 2j + 1 (high half)
      const uint32_t w0 = v_reg[0][j], w1 = v_reg[1][j], w2 = v_reg[2][j], w3 = v_reg[3][j];
      u32x2 ev, od;
      // low halves / high halves of two words side by side: one v_perm_b32 each (bytes 0-3 of the
      // selector's space are the second operand, 4-7 the first)
      ev.x = __builtin_amdgcn_perm(w1, w0, 0x05040100u); ev.y = __builtin_amdgcn_perm(w3, w2, 0x05040100u);
      od.x = __builtin_amdgcn_perm(w1, w0, 0x07060302u); od.y = __builtin_amdgcn_perm(w3, w2, 0x07060302u);
      const uint32_t d = v_dg * 8u + 2u * (uint32_t)j;
      *reinterpret_cast<u32x2*>(sV + v_off(d, chunk) + 8u * half) = ev;
      *reinterpret_cast<u32x2*>(sV + v_off(d + 1u, chunk) + 8u * half) = od;
    }
  };

  f32x16 oacc[4];  // O^T tiles: rows d = 32*dt + 8j + 4h + i, column q = lane % 32
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) oacc[dt] = f32x16{0};
  float m_run = -INFINITY, l_run = 0.f;

  const uint32_t n_tiles = g.causal ? (q0 + kBq) / kBkv : g.S / kBkv;
  // Staging overlaps arithmetic: the K tile is only read by region 0 and the V^T tile only by
  // region 2, so K tile t+1 is written after the barrier that follows region 0 of tile t (while the
  // softmax runs), and V^T tile t during region 0 of tile t itself, between the MFMAs of K Q^T (every
  // wave left region 2 of tile t-1 before the barrier that precedes it).  Each staging register is
  // refilled from global memory right after it has been written out: a whole tile ahead.
  load_k(0);
  load_v(0);
  store_k();
  load_k(kBkv);  // there are always at least two tiles (S is a multiple of 128)
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
  // One KV tile.  MORE / MORE2 (tile t+1 / t+2 exists) and MASK (the tile may reach past the diagonal)
  // are compile-time: the steady-state body has no branch around its loads and LDS writes, so the
  // compiler can wait for exactly the loads a write needs instead of for all outstanding ones.  The
  // barriers wait for LDS traffic only, never for the global loads of later tiles.
  auto tile = [&](uint32_t t, auto more_c, auto more2_c, auto mask_c) {
    constexpr bool MORE = decltype(more_c)::value, MORE2 = decltype(more2_c)::value, MASK = decltype(mask_c)::value;
    const uint32_t kv0 = t * kBkv;

    // ---- region 0: S^T = K Q^T, with the staging of V^T tile t threaded in ------------------------
    // (opened by the site that closed region 2 of the tile before, or by the one ahead of the loop)
    // The two workgroups of a CU drift apart, so a SIMD usually holds one wave in a matrix region and
    // one in the softmax.  The matrix regions run at a higher wave priority: when both want to issue,
    // the MFMA goes first and the matrix pipe stays fed, while the softmax fills the gaps (measured:
    // 3 % faster than equal priorities, the opposite order 3 % slower).
    __builtin_amdgcn_s_setprio(1);
    store_v();
    if constexpr (MORE) load_v(kv0 + kBkv);
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
    __builtin_amdgcn_s_setprio(0);

    // every wave is done with K tile t and V^T tile t is visible; K tile t+1 goes to LDS while the softmax runs
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    // The site sits behind the barrier, not in front of it: in front, the barrier's wait for LDS traffic
    // would also wait for the two record stores the site has just issued, every tile (measured: 1.5
    // points of overhead).  The wait at the barrier thereby belongs to the region that ends here.
    KP_BOUNDARY(ring, 0, 1);
    KP_CHAIN(1, ring);
    if constexpr (MORE) store_k();
    if constexpr (MORE2) load_k(kv0 + 2 * kBkv);

    // ---- region 1: online softmax (this lane: query row qrow, 32 of the tile's 64 kv) -------------
    const bool diag = MASK && g.causal && (kv0 + kBkv > q0 + wave * 32);  // tile reaches past this wave's first row
    float mx = -INFINITY;  // maximum of the raw scores; the positive scale is applied afterwards
#pragma unroll
    for (int tk = 0; tk < 2; ++tk)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        if (diag) {
          const uint32_t kv = kv0 + 32 * tk + 8 * (v >> 2) + 4 * h32 + (v & 3);
          if (kv > qrow) sacc[tk][v] = -INFINITY;
        }
        mx = fmaxf(mx, sacc[tk][v]);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    // The value the exponentials are taken against only has to keep them in range; it need not be the
    // running maximum.  It moves (and O and l are rescaled) only when some row of the wave exceeds it
    // by more than 2^kSlack, which after the first few tiles practically never happens; until then a
    // probability may be as large as 2^kSlack, which fp32 sums and bf16 operands hold without loss.
    const float mx_s = mx * g.scale_log2;
    if (__builtin_amdgcn_ballot_w64(mx_s > m_run + kSlack) != 0ull) {  // always on the first tile (m_run = -inf)
      const float m_new = fmaxf(m_run, mx_s);  // finite from the first tile on: kv = 0 is visible to every row
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
      l_run *= alpha;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[dt][v] *= alpha;
      m_run = m_new;
    }
    float psum = 0.f;
    uint32_t pk[2][8];  // P as packed bf16 pairs, in accumulator order
#pragma unroll
    for (int tk = 0; tk < 2; ++tk)
#pragma unroll
      for (int v = 0; v < 16; v += 2) {
        const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[tk][v], g.scale_log2, -m_run));
        const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[tk][v + 1], g.scale_log2, -m_run));
        psum += p0 + p1;  // fp32 sum of the unrounded probabilities
        pk[tk][v >> 1] = bf16_pack_rne(p0, p1);
      }
    l_run += psum;
    KP_BOUNDARY(ring, 1, 2);
    KP_CHAIN(2, ring);
    __builtin_amdgcn_s_setprio(2);

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
          u32x4 vw = *reinterpret_cast<const u32x4*>(sV + v_off(row, 4 * tk + 2 * s + h32));
          if (dt >= 2) vw = u32x4{vw.z, vw.w, vw.x, vw.y};  // rows 64.. store the chunk halves swapped
          oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vw), pf, oacc[dt], 0, 0, 0);
        }
      }
    __builtin_amdgcn_s_setprio(0);

    // every wave is done with V^T tile t, and K tile t+1 is visible
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    // One site closes region 2 and opens region 0 of the next tile: a tile costs three sites, not four.
    // Behind the barrier for the same reason as above.
    if constexpr (MORE) KP_BOUNDARY(ring, 2, 0); else KP_BOUNDARY(ring, 2, kp::kNoRegion);
    if constexpr (INSTR >= 4) {
      kp::chain_commit<3>(ring);
      KP_CHAIN(0, ring);
    }
  };
  constexpr std::true_type yes{};
  constexpr std::false_type no{};
  KP_BOUNDARY(ring, kp::kNoRegion, 0);
  KP_CHAIN(0, ring);
  // only the last two tiles of a causal block can reach past the diagonal
  for (uint32_t t = 0; t + 2 < n_tiles; ++t) tile(t, yes, yes, no);
  tile(n_tiles - 2, yes, no, yes);
  tile(n_tiles - 1, no, no, yes);

  // epilogue: O[q][d] = O^T[d][q] / l
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = 1.0f / l_tot;
  uint16_t* orow = g.O + head + (size_t)qrow * kD;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      u32x2 pk2;
      pk2.x = bf16_pack_rne(oacc[dt][4 * q + 0] * inv, oacc[dt][4 * q + 1] * inv);
      pk2.y = bf16_pack_rne(oacc[dt][4 * q + 2] * inv, oacc[dt][4 * q + 3] * inv);
      *reinterpret_cast<u32x2*>(orow + 32 * dt + 8 * q + 4 * h32) = pk2;
    }
  if constexpr (INSTR != 0) {
    kp::TraceGeom tg{g.n_wg, 4u >> g.group_log2, 3, g.cap_hbm, g.flags};
    if constexpr (INSTR >= 4) {
      kp::chain_commit<1>(ring);
      kp::ring_finish<INSTR == 5>(ring, g.cap_lds, g.trace, tg, wg, g.rec_cost, AttnChain{});
    } else {
      kp::ring_finish<INSTR == 3>(ring, g.cap_lds, g.trace, tg, wg, g.rec_cost);
    }
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
  if (region_mask & KP_MASK_PHASES) return kp::fail(KP_ERR_INVALID_ARG, "KP_MASK_PHASES belongs to the GEMM");
  const uint32_t regions = region_mask & ~(KP_MASK_FLUSH | KP_MASK_WAVE_GROUP | KP_MASK_REALTIME | KP_MASK_COLLAB), flush = region_mask >> 31;
  const bool realtime = (region_mask & KP_MASK_REALTIME) != 0u, collab = (region_mask & KP_MASK_COLLAB) != 0u;
  const uint32_t group_log2 = (region_mask & KP_MASK_WAVE_GROUP) ? 2u : 0u;
  const size_t streams = 4u >> group_log2;
  const int n_wg = B * H * (S / kBq);
  hipStream_t st = static_cast<hipStream_t>(stream);
  AttnArgs g{};
  g.Q = static_cast<const uint16_t*>(Q); g.K = static_cast<const uint16_t*>(K);
  g.V = static_cast<const uint16_t*>(V); g.O = static_cast<uint16_t*>(O);
  g.B = (uint32_t)B; g.H = (uint32_t)H; g.S = (uint32_t)S; g.causal = causal ? 1u : 0u;
  g.scale_log2 = scale * 1.4426950408889634f;
  g.region_mask = regions; g.trace = trace_buf; g.flush = flush; g.n_wg = (uint32_t)n_wg;
  g.group_log2 = group_log2;
  g.collab = collab ? 1u : 0u;
  g.flags = (flush ? KP_FLAG_FLUSH : 0u) | (realtime ? KP_FLAG_REALTIME : 0u) | (collab ? KP_FLAG_HW_IDS : 0u);
  const uint32_t tile_bytes = kKBytes + kVBytes;
  if (regions == 0) {
    hipLaunchKernelGGL(kp_attn_fwd<0>, dim3(n_wg), dim3(kAttnThreads), tile_bytes, st, g);
    KP_HIP_TRY(hipGetLastError());
    return KP_OK;
  }
  if (!trace_buf) return kp::fail(KP_ERR_INVALID_ARG, "trace_buf is NULL but region_mask enables regions");
  if (regions >> 3) return kp::fail(KP_ERR_INVALID_ARG, "region_mask enables regions this kernel does not have (3 regions)");
  if (((uintptr_t)trace_buf) & 15u) return kp::fail(KP_ERR_INVALID_ARG, "trace_buf must be 16-byte aligned");
  if (trace_cap % streams) return kp::fail(KP_ERR_TRACE_TOO_SMALL, "trace_cap must be a multiple of %zu record streams", streams);
  const size_t cap_wave = trace_cap / streams;
  if (!kp::is_pow2(cap_wave) || cap_wave < 2 || cap_wave > (1u << 19))
    return kp::fail(KP_ERR_TRACE_TOO_SMALL, "trace_cap/streams = %zu must be a power of two >= 2", cap_wave);
  uint32_t cap_lds = (uint32_t)cap_wave;
  if (flush && cap_lds > 64) cap_lds = 64;
  const size_t ring_bytes = (size_t)cap_lds * 8 * streams + (group_log2 ? 16 : 0);  // (16: see chain_begin)
  if (ring_bytes > 32 * 1024) return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "LDS ring of %zu bytes exceeds the 32 KiB budget", ring_bytes);
  g.cap_lds = cap_lds; g.cap_hbm = (uint32_t)cap_wave; g.rec_cost = kp::rec_cost();
  static thread_local int attr_dev = -1;  // the attribute is kept per device
  int dev = 0;
  KP_HIP_TRY(hipGetDevice(&dev));
  if (attr_dev != dev) {
    KP_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kp_attn_fwd<1>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024));
    KP_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kp_attn_fwd<5>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024));
    KP_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kp_attn_fwd<3>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024));
    KP_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kp_attn_fwd<4>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024));
    attr_dev = dev;
  }
  // circular strategy and one lane stores: chained record sites
  if (!flush && !collab) {
    if (realtime) hipLaunchKernelGGL(kp_attn_fwd<5>, dim3(n_wg), dim3(kAttnThreads), tile_bytes + ring_bytes, st, g);
    else hipLaunchKernelGGL(kp_attn_fwd<4>, dim3(n_wg), dim3(kAttnThreads), tile_bytes + ring_bytes, st, g);
  } else if (realtime) {
    hipLaunchKernelGGL(kp_attn_fwd<3>, dim3(n_wg), dim3(kAttnThreads), tile_bytes + ring_bytes, st, g);
  } else {
    hipLaunchKernelGGL(kp_attn_fwd<1>, dim3(n_wg), dim3(kAttnThreads), tile_bytes + ring_bytes, st, g);
  }
  KP_HIP_TRY(hipGetLastError());
  return KP_OK;
}

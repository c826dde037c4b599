// Instrumented bf16 attention forward (kp_attn_instrumented): O = softmax(scale * Q K^T + mask) V,
// fp32 softmax and accumulation, head dimension 128, optional causal mask.
//
// The paper's case study profiles a flash-attention kernel whose regions are the two GEMMs and
// the softmax of every KV iteration (Sec. 5.2, Table 3: GEMM0 = Q K^T, softmax, GEMM1 = P V).
// This is the library's own MFMA kernel with the same three regions per KV tile of 64:
//   region 0  S^T = K Q^T     (MFMA); closes behind the barrier that follows it
//   region 1  online softmax   (VALU, fp32); opens with the four loads that send this wave's share of the
//             next K tile from global memory straight to LDS
//   region 2  O^T += V^T P^T   (MFMA; V is transposed by the LDS read); closes behind the barrier that
//             follows it, and the next V tile is requested there
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
constexpr uint32_t kRow = kD * 2;             // a row of either tile: one kv, 128 d, 256 bytes in 16 chunks of 16
constexpr uint32_t kKBytes = kBkv * kRow;     // K tile [64 kv][128 d]
constexpr uint32_t kVBytes = kBkv * kRow;     // V tile [64 kv][128 d], as it lies in memory
constexpr float kSlack = 8.0f;                // log2 of how far a score may exceed the softmax reference

// two fp32 -> packed bf16 pair (lo in bits 15:0), round to nearest even: one v_cvt_pk_bf16_f32
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t bf16_pack_rne(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// Both tiles go from global memory straight to LDS (global_load_lds_dwordx4: lane l of a wave lands at byte
// 16 l of a 1 KiB block, i.e. of four rows), so a tile's layout is a permutation of the 16 chunks inside each
// row, which the loading lane applies by fetching the chunk that belongs at its place.
// K tile: chunk c of row kv at position c ^ (kv % 16): the 16-byte operand reads of 16 neighbouring rows (one
// pass of a 16-byte LDS read) cover all banks.
// V tile: chunk c of row kv at position c ^ 4 (kv % 4).  Its operand reads transpose: ds_read_b64_tr_b16 hands
// lane j of a group of 16 lanes the elements j, 16 + j, 32 + j, 48 + j of the 64 that the group's lanes address
// (4 each), so with lane i addressing V[kv0 + i / 4][d0 + 4 (i % 4) ..+3] lane j receives V[kv0 .. kv0 + 3][d0 + j];
// the XOR spreads the four rows and two column groups of a pass over all banks.

// END of one region and/or START of the next with a single clock sample.  INSTR: 0 no record sites,
// 1 generic sites (region mask, either buffer strategy, either store), 3 the same on the constant-rate clock,
// 4 chained sites (circular strategy, one lane stores; region mask and wave-group records included: the loop
// keeps only the clocks and the records are made when the trace is copied out), 5 chained, constant-rate clock.
#define KP_BOUNDARY(ring, end_r, start_r) do { if constexpr (INSTR == 1 || INSTR == 3) kp::site<INSTR>(ring, end_r, start_r); } while (0)
#define KP_CHAIN(K, ring) do { if constexpr (INSTR >= 4) kp::site_chain<K, (INSTR == 5)>(ring); } while (0)

// The sequence of record sites: two that write no record (they fill the first batch), one ahead of the loop
// (opens region 0), three per KV tile, the last only closes.  A tile's three sites are committed as one batch
// inside region 0 of the next tile, once its first MFMAs have been issued: nothing but the clock reads stands
// behind a barrier, where every wave of the workgroup would pay for it at the same time.
struct AttnChain {
  static constexpr uint32_t kRegions = 3u, kLead = 2u;
  static constexpr bool kDense = true;
  // n = 2 + 1 + 3 tiles: every enabled region leaves two records per tile
  __device__ uint32_t total(uint32_t n, uint32_t mask) const { return 2u * ((n - 3u) / 3u) * (uint32_t)__builtin_popcount(mask & 7u); }
  __device__ uint32_t end_region(uint32_t site, uint32_t) const { return site <= kLead ? kp::kNoRegion : (site - 1u - kLead) % 3u; }
  __device__ uint32_t start_region(uint32_t site, uint32_t n) const {
    return (site < kLead || site + 1u == n) ? kp::kNoRegion : (site - kLead) % 3u;
  }
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

  // global -> LDS: either tile is 16 blocks of 1 KiB (four rows); wave w loads blocks 4 w .. 4 w + 3 of it.
  // Lane i of block j is row 4 j + i / 16, chunk position i % 16.
  const uint32_t lds0 = kp::wave_uniform((uint32_t)(uintptr_t)smem + 4096u * wave);
  const uint16_t* k_src[4];
  const uint16_t* v_src[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t row = 16u * wave + 4u * (uint32_t)i + (lane >> 4), pos = lane & 15u;
    k_src[i] = g.K + head + (size_t)row * kD + ((pos ^ (row & 15u)) << 3);
    v_src[i] = g.V + head + (size_t)row * kD + ((pos ^ (4u * (row & 3u))) << 3);
  }
  // One load: M0 (the LDS base) is put back afterwards, the compiler does not expect inline assembly to change
  // it.  From inline assembly because the compiler would make the next LDS access of any kind wait for such a
  // load; hidden from its count of outstanding vector-memory operations the loads still complete in order, and
  // the kernel waits for them itself in front of the barrier that precedes the tile's use.
  auto direct_load = [&](const uint16_t* src, uint32_t dst) {
    uint32_t saved_m0;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off\n\ts_mov_b32 m0, %0"
                 : "=&s"(saved_m0) : "v"(src), "s"(dst) : "memory");
  };
  auto load_k = [&](uint32_t kv0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) direct_load(k_src[i] + (size_t)kv0 * kD, lds0 + (uint32_t)i * 1024u);
  };
  auto load_v = [&](uint32_t kv0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) direct_load(v_src[i] + (size_t)kv0 * kD, lds0 + kKBytes + (uint32_t)i * 1024u);
  };
  // operand reads: K row 32 tk + l32, chunk 2 s + h32; V for the kv of MFMA step (tk, s) and the d of tile dt
  uint32_t k_rd[8], v_rd[4];
#pragma unroll
  for (int sx = 0; sx < 8; ++sx) k_rd[sx] = l32 * kRow + (((2u * (uint32_t)sx + h32) ^ (l32 & 15u)) << 4);
  {
    const uint32_t i = lane & 15u, grp = lane >> 4;  // groups 0, 1: d 0-15, 16-31 of the tile; 2, 3 the same for h = 1
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
      const uint32_t d = 32u * (uint32_t)dt + 16u * (grp & 1u) + 4u * (i & 3u);
      v_rd[dt] = (4u * (grp >> 1) + (i >> 2)) * kRow + (((d >> 3) ^ (4u * (i >> 2))) << 4) + 8u * ((d >> 2) & 1u);
    }
  }
  auto read_v = [&](uint32_t kv_step, int dt) -> bf16x8 {  // kv_step: first kv of the MFMA step (a multiple of 16)
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    typedef __attribute__((address_space(3))) s16x4* lds_s16x4;
    const unsigned char* at = sV + v_rd[dt] + kv_step * kRow;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(at));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(at + 8u * kRow));
    const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
  };

  f32x16 oacc[4];  // O^T tiles: rows d = 32*dt + 8j + 4h + i, column q = lane % 32
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) oacc[dt] = f32x16{0};
  float m_run = -INFINITY, l_run = 0.f;

  const uint32_t n_tiles = g.causal ? (q0 + kBq) / kBkv : g.S / kBkv;
  // Staging overlaps arithmetic: the K tile is only read by region 0 and the V tile only by region 2, so K tile
  // t+1 is requested behind the barrier that follows region 0 of tile t (and travels while softmax and P V run)
  // and V tile t+1 behind the barrier that follows region 2 of tile t; each is waited for in front of the
  // barrier that precedes its use.
  load_k(0);
  load_v(0);
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
  // One KV tile.  MORE (tile t+1 exists) and MASK (the tile may reach past the diagonal) are compile-time: the
  // steady-state body has no branch.  Each barrier waits for this wave's LDS traffic and for the tile it
  // requested one barrier earlier.
  auto tile = [&](uint32_t t, auto more_c, auto mask_c) {
    constexpr bool MORE = decltype(more_c)::value, MASK = decltype(mask_c)::value;
    const uint32_t kv0 = t * kBkv;

    // ---- region 0: S^T = K Q^T, with the staging of V^T tile t threaded in ------------------------
    // (opened by the site that closed region 2 of the tile before, or by the one ahead of the loop)
    // The two workgroups of a CU drift apart, so a SIMD usually holds one wave in a matrix region and
    // one in the softmax.  The matrix regions run at a higher wave priority: when both want to issue,
    // the MFMA goes first and the matrix pipe stays fed, while the softmax fills the gaps (measured:
    // 3 % faster than equal priorities, the opposite order 3 % slower).
    __builtin_amdgcn_s_setprio(1);
    f32x16 sacc[2];
    sacc[0] = f32x16{0}; sacc[1] = f32x16{0};
#pragma unroll
    for (int s = 0; s < 8; ++s) {
#pragma unroll
      for (int tk = 0; tk < 2; ++tk) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(sK + k_rd[s] + (uint32_t)tk * 32u * kRow);
        sacc[tk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], sacc[tk], 0, 0, 0);
      }
      // the three sites of the tile before (ahead of the first tile: the one that opened region 0)
      if constexpr (INSTR >= 4) if (s == 3) kp::chain_commit<3>(ring);
    }
    __builtin_amdgcn_s_setprio(0);

    // every wave is done with K tile t and V tile t has landed; K tile t+1 travels while softmax and P V run
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    // The site sits behind the barrier, not in front of it: in front, the barrier's wait for LDS traffic
    // would also wait for the two record stores the site has just issued, every tile (measured: 1.5
    // points of overhead).  The wait at the barrier thereby belongs to the region that ends here.
    KP_BOUNDARY(ring, 0, 1);
    KP_CHAIN(0, ring);
    if constexpr (MORE) load_k(kv0 + kBkv);

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
    KP_CHAIN(1, ring);
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
          oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_v(32u * (uint32_t)tk + 16u * (uint32_t)s, dt), pf, oacc[dt], 0, 0, 0);
        }
      }
    __builtin_amdgcn_s_setprio(0);

    // every wave is done with V tile t, and K tile t+1 has landed
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    // One site closes region 2 and opens region 0 of the next tile: a tile costs three sites, not four.
    // Behind the barrier for the same reason as above.
    if constexpr (MORE) KP_BOUNDARY(ring, 2, 0); else KP_BOUNDARY(ring, 2, kp::kNoRegion);
    KP_CHAIN(2, ring);
    if constexpr (MORE) load_v(kv0 + kBkv);
  };
  constexpr std::true_type yes{};
  constexpr std::false_type no{};
  KP_BOUNDARY(ring, kp::kNoRegion, 0);
  KP_CHAIN(0, ring);  // (the first two fill the first batch and write no record)
  KP_CHAIN(1, ring);
  KP_CHAIN(2, ring);
  // only the last two tiles of a causal block can reach past the diagonal
  for (uint32_t t = 0; t + 2 < n_tiles; ++t) tile(t, yes, no);
  tile(n_tiles - 2, yes, yes);
  tile(n_tiles - 1, no, yes);

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
      kp::chain_commit<3>(ring);  // the sites of the last tile
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

// Instrumented bf16 GEMM targets (kp_gemm_instrumented): C[M,N] = A[M,K] * B[K,N], fp32 accumulate,
// bf16 (round-to-nearest-even) output, all row-major.
//
// The paper profiles software-pipelined Triton GEMMs by inserting region records around the
// stages of the K loop (Sec. 5.3, GEMM-SWP-2/3; Sec. 2.3 software pipelining).  These kernels
// are this library's own MFMA GEMMs with hand-placed record sites.  Each exists twice from one
// template: INSTR=0 compiles every record site away (the uninstrumented baseline), INSTR=1 and 2
// record into the LDS ring.  Record sites contain no floating point, so all variants produce
// bit-identical C.
//
//   tile 64x64x32, 4 waves  : regions 0 global load, 1 LDS store, 2 MFMA        (per K step)
//   tile 256x256x64, 8 waves: regions 0 / 1 first / second half of a K step's MFMAs with the
//                              staging of the next K step threaded in, 2 barrier wait, 3 epilogue (once);
//                              or (KP_MASK_PHASES) a K step whose stages follow one another, each its own
//                              region: 2 LDS write, 0 global load issue, 3 MFMA, 1 wait; 4 epilogue (once)
#include <type_traits>

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
  uint32_t rec_cost;  // ticks the decoder takes off every duration (kp_set_rec_cost)
  uint32_t group_log2;  // 2^group_log2 waves share one record stream
  uint32_t collab;      // 1: all lanes store a record, hardware ids go to the workgroup header
  uint32_t flags;       // kp_trace_hdr.flags of the trace
};

// fp32 -> bf16, round to nearest even (v_cvt_pk_bf16_f32 on gfx950)
__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
  const __bf16 h = (__bf16)f;
  return (uint32_t)__builtin_bit_cast(uint16_t, h);
}
// two fp32 -> packed bf16 pair (lo in bits 15:0), round to nearest even: one v_cvt_pk_bf16_f32
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t bf16_pack_rne(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// LDS tiles hold rows of BK bf16 (K contiguous) in 16-byte chunks; chunk c of row r lives at chunk
// position c ^ swz(r) so that the 16-byte reads of 32 different rows spread over all banks.
template <int BK>
__device__ __forceinline__ uint32_t tile_off(uint32_t row, uint32_t chunk) {
  constexpr uint32_t CPR = BK / 8;           // chunks per row
  constexpr uint32_t RPL = 128 / (BK * 2);   // rows per 128-byte bank line (BK <= 64)
  // With 128-byte rows (BK = 64) two neighbouring rows already differ in the upper half of the 16 chunk
  // positions of a 256-byte bank line, so the XOR takes row bits 1..3: 16 consecutive rows then cover all
  // 16 positions (with row bits 0..2, rows r and r + 8 shared one, and every operand read took twice as long).
  const uint32_t s = BK == 64 ? (row >> 1) % CPR : (row / RPL) % CPR;
  return row * (BK * 2) + ((chunk ^ s) * 16);  // byte offset
}

// Same, for the transposed B tile of the large kernel (BK = 64): its 16-byte writes come from lanes
// whose rows are 8 apart, so the swizzle also folds in the next three row bits.
__device__ __forceinline__ uint32_t tile_off_bt(uint32_t row, uint32_t chunk) {
  return row * 128u + ((chunk ^ ((row ^ (row >> 3)) & 7u)) << 4);
}

// END of one region and START of the next with a single clock sample.  INSTR: 0 no record sites,
// 1 generic sites (region mask, either buffer strategy, either store), 3 the same on the constant-rate
// clock, 2 lean sites (small kernel: all regions, circular) or chained sites (large kernel: circular, one
// lane stores; the region mask and wave-group records included), 5 chained sites on the constant-rate clock.
// SITE is the form of the sites a kernel uses for INSTR (kp::site<>; 6: chained).
#define KP_BOUNDARY(ring, end_r, start_r) do { if constexpr (INSTR != 0) kp::site<SITE>(ring, end_r, start_r); } while (0)
// The same for the large kernel, whose sites are a fixed sequence: chained, the loop keeps only the clock
// of site K of the batch (kp::site_chain) and KP_COMMIT, which stands right after a wait for all LDS
// traffic, stores the batch's clocks; the records are made when the trace is copied out.
#define KP_SITE_K(ring, K, end_r, start_r) do { if constexpr (INSTR != 0) { \
    if constexpr (SITE == 6) kp::site_chain<K, (INSTR == 5), kMayCross>(ring); else kp::site<SITE>(ring, end_r, start_r); } } while (0)
#define KP_COMMIT(ring, N) do { if constexpr (INSTR != 0 && SITE == 6) kp::chain_commit<N>(ring); } while (0)

// The sequence of the large kernel's record sites (n sites in all).  Default schedule: regions 0, 1, 2 in turn,
// three sites per K step; sites 0 and 1 write no record, they only fill the first two places of the first
// batch, so that every batch of the loop is "the site in the middle of the K step before, the one in front of
// its barrier and the one behind it" and is committed once the first MFMAs of the next K step have been
// issued: no commit waits for a clock it has just asked for, and none stands between a wave and the barrier,
// where its instructions and the latency of its LDS write would be time on the critical path of every K step.  Stages apart: regions 2, 0, 3, 1 in turn, four sites per K step, committed
// behind the barrier (every wave waits there in region 1 anyway); no leading site.  The last site of the loop
// opens the epilogue region instead (3, or 4 with the stages apart), the very last closes it.
template <bool PHASED>
struct GemmChain {
  static constexpr uint32_t kEpilogue = PHASED ? 4u : 3u, kRegions = kEpilogue + 1u, kLead = PHASED ? 0u : 2u;
  static constexpr bool kDense = true;
  // n = kLead + (3 or 4) K steps + 2: every enabled region of the loop leaves two records per K step, the epilogue two
  __device__ uint32_t total(uint32_t n, uint32_t mask) const {
    const uint32_t steps = (n - 2u - kLead) / (PHASED ? 4u : 3u);
    return 2u * steps * (uint32_t)__builtin_popcount(mask & ((1u << kEpilogue) - 1u)) + 2u * ((mask >> kEpilogue) & 1u);
  }
  __device__ static uint32_t in_turn(uint32_t i) {
    if constexpr (PHASED) return (0x1302u >> ((i & 3u) * 4u)) & 0xFu;  // 2, 0, 3, 1
    else return i % 3u;
  }
  __device__ uint32_t end_region(uint32_t site, uint32_t n) const {
    return site <= kLead ? kp::kNoRegion : site + 1u == n ? kEpilogue : in_turn(site - 1u - kLead);
  }
  __device__ uint32_t start_region(uint32_t site, uint32_t n) const {
    return (site < kLead || site + 1u == n) ? kp::kNoRegion : site + 2u == n ? kEpilogue : in_turn(site - kLead);
  }
};

// ------------------------------------------------------------------------------------------
// 64x64x32 tile, 4 waves as 2x2, each wave one 32x32 accumulator tile.
template <int INSTR>
__global__ __launch_bounds__(256) void kp_gemm_small(GemmArgs g) {
  constexpr int SITE = INSTR;
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
  if constexpr (INSTR != 0)
    ring = kp::ring_init<true>(ring_lds, t_begin, g.cap_lds, g.region_mask, g.flush, g.cap_hbm, g.trace, g.n_wg, 4u >> g.group_log2, wg,
                         g.group_log2);
  ring.collab = g.collab;
  if constexpr (INSTR == 3) kp::ring_use_realtime(ring);
  kp::sites_begin<SITE>(ring);

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
    if (kt == 0) KP_BOUNDARY(ring, kp::kNoRegion, 0); else KP_BOUNDARY(ring, 2, 0);
    const u32x4 av = *reinterpret_cast<const u32x4*>(a_src + (size_t)kt * BK);
    uint32_t bv[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
      bv[i] = b_on ? *reinterpret_cast<const uint32_t*>(b_src + ((size_t)kt * BK + i) * g.N) : 0u;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    KP_BOUNDARY(ring, 0, 1);
    // ---- region 1: LDS store -----------------------------------------------------------------
    __syncthreads();  // previous step's MFMA reads are done
    *reinterpret_cast<u32x4*>(sA + tile_off<BK>(a_row, a_chunk)) = av;
    if (b_on) {
      u32x4 lo, hi;  // column 2*b_np and 2*b_np+1, eight consecutive k each
      lo.x = __builtin_amdgcn_perm(bv[1], bv[0], 0x05040100u); hi.x = __builtin_amdgcn_perm(bv[1], bv[0], 0x07060302u);
      lo.y = __builtin_amdgcn_perm(bv[3], bv[2], 0x05040100u); hi.y = __builtin_amdgcn_perm(bv[3], bv[2], 0x07060302u);
      lo.z = __builtin_amdgcn_perm(bv[5], bv[4], 0x05040100u); hi.z = __builtin_amdgcn_perm(bv[5], bv[4], 0x07060302u);
      lo.w = __builtin_amdgcn_perm(bv[7], bv[6], 0x05040100u); hi.w = __builtin_amdgcn_perm(bv[7], bv[6], 0x07060302u);
      *reinterpret_cast<u32x4*>(sB + tile_off<BK>(b_np * 2, b_kg)) = lo;
      *reinterpret_cast<u32x4*>(sB + tile_off<BK>(b_np * 2 + 1, b_kg)) = hi;
    }
    __syncthreads();
    KP_BOUNDARY(ring, 1, 2);
    // ---- region 2: MFMA ------------------------------------------------------------------------
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      // operand layout of v_mfma_f32_32x32x16_bf16: lane l supplies row/column l%32, k = 8*(l/32)..+7
      const uint32_t chunk = ks * 2 + (lane >> 5);
      const bf16x8 af = *reinterpret_cast<const bf16x8*>(sA + tile_off<BK>(wr * 32 + (lane & 31u), chunk));
      const bf16x8 bf = *reinterpret_cast<const bf16x8*>(sB + tile_off<BK>(wc * 32 + (lane & 31u), chunk));
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bf, acc, 0, 0, 0);
    }
    asm volatile("s_nop 0" ::: "memory");
  }
  KP_BOUNDARY(ring, 2, kp::kNoRegion);

  // epilogue: accumulator register v of lane l is C[row, col] with col = l%32,
  // row = 8*(v/4) + 4*(l/32) + v%4 inside the wave's 32x32 tile
  const uint32_t col = n0 + wc * 32 + (lane & 31u);
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const uint32_t row = m0 + wr * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v % 4);
    g.C[(size_t)row * g.N + col] = (uint16_t)f32_to_bf16_rne(acc[v]);
  }
  if constexpr (INSTR != 0) {
    kp::TraceGeom tg{g.n_wg, 4u >> g.group_log2, 3, g.cap_hbm, g.flags};
    kp::sites_end<SITE>(ring);
    kp::ring_finish<INSTR == 3>(ring, g.cap_lds, g.trace, tg, wg, g.rec_cost);
  }
}


// ------------------------------------------------------------------------------------------
// 256x256x64 tile, 8 waves as 2 (M) x 4 (N); each wave owns 128x64 of C as 4x2 MFMA tiles.
// LDS holds two stages of the A tile [256][64] and of the B tile (128 KiB); the K loop is software-pipelined
// over the two stages.  Default schedule: while the MFMAs consume stage s, the tiles of K step +1 travel from
// global memory straight to stage s^1 (no staging registers; B stays row-major and is transposed by the LDS
// read).  Stage-by-stage schedule: K step +1 moves from staging registers to stage s^1 (B transposed in
// registers into a [256 n][64 k] tile) and the global loads of K step +2 are in flight.
// MFMA operands are swapped (B^T rows as the first operand) so that a lane ends up with four
// consecutive columns of one C row per accumulator quad and can store them as 8 bytes.
constexpr int kBigBM = 256, kBigBN = 256, kBigBK = 64;
constexpr uint32_t kBigTileBytes = 2u * (kBigBM + kBigBN) * kBigBK * 2u;  // both stages

template <int INSTR, int WAVES, int SCHEDULE>
__global__ __launch_bounds__(WAVES * 64) void kp_gemm_big(GemmArgs g) {
  // default schedule: vector, scalar and LDS-read instructions may be scheduled across a chained site; the
  // regions are halves of the K step's MFMAs, which stay on their side (stages apart: nothing crosses)
  constexpr int kMayCross = SCHEDULE == 0 ? 0x106 : 0;
  // SCHEDULE 0: staging threaded through the MFMAs; 1: the stages of a K step one after the other; 2: the
  // same source without the scheduling fences between the stages (uninstrumented only)
  constexpr bool PHASED = SCHEDULE != 0;
  static_assert(SCHEDULE != 2 || INSTR == 0, "the unfenced stage-by-stage form has no record sites");
  // INSTR 2 and 5 (constant-rate clock): chained sites; 1 and 3 are the generic sites, which the flush
  // strategy and the 64-lane store need
  static_assert(INSTR != 4, "no such form");
  constexpr int SITE = (INSTR == 2 || INSTR == 5) ? 6 : INSTR;
  constexpr bool REALTIME = INSTR == 3 || INSTR == 5;
  constexpr int BM = kBigBM, BN = kBigBN, BK = kBigBK;
  constexpr int TN = WAVES == 8 ? 2 : 4;   // 32-column MFMA tiles per wave (wave tile 128 x 32*TN)
  static_assert(WAVES == 8 || WAVES == 4, "2 x 4 or 2 x 2 waves");
  constexpr int T = WAVES * 64;             // threads
  constexpr int NA = 2048 / T;              // A chunks per thread and K step
  constexpr int NB = 512 / T;               // B blocks (4 k x 8 n) per thread and K step
  constexpr uint32_t A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE = A_BYTES + B_BYTES;
  extern __shared__ __align__(16) unsigned char smem[];  // [stage0 A|B][stage1 A|B][ring]
  uint32_t* ring_lds = reinterpret_cast<uint32_t*>(smem + 2 * STAGE);

  const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
  const uint32_t tiles_m = g.M / BM, tiles_n = g.N / BN;
  // Workgroups are dealt round-robin to the 8 XCDs; give every XCD a compact block of tiles
  // so that the A and B panels it streams stay in its own L2.
  uint32_t tile_r, tile_c;
  if ((tiles_m % 4u) == 0u && (tiles_n % 2u) == 0u) {
    const uint32_t xcd = blockIdx.x & 7u, j = blockIdx.x >> 3;
    const uint32_t br = tiles_m / 4u, bc = tiles_n / 2u;  // block of tiles per XCD
    tile_r = (xcd >> 1) * br + j / bc;
    tile_c = (xcd & 1u) * bc + j % bc;
  } else {
    tile_r = blockIdx.x / tiles_n;
    tile_c = blockIdx.x % tiles_n;
  }
  const uint32_t wg = tile_r * tiles_n + tile_c;  // recorded workgroup id = tile index
  const uint32_t m0 = tile_r * BM, n0 = tile_c * BN;

  kp::Ring ring{};
  if constexpr (INSTR != 0)
    ring = kp::ring_init<true>(ring_lds, reinterpret_cast<uint64_t*>(smem), g.cap_lds, g.region_mask, g.flush,
                         g.cap_hbm, g.trace, g.n_wg, (uint32_t)WAVES >> g.group_log2, wg, g.group_log2);
  ring.collab = g.collab;
  if constexpr (REALTIME) kp::ring_use_realtime(ring);
  // (with wave groups the host adds 16 bytes behind the ring for the waves that do not record)
  if constexpr (SITE == 6) kp::chain_begin(ring, (uint32_t)(uintptr_t)ring_lds + ((uint32_t)WAVES >> g.group_log2) * g.cap_lds * 8u);
  else kp::sites_begin<SITE>(ring);

  // ---- global -> register -> LDS mapping (stage-by-stage schedule) ---------------------------
  // Every thread stages the same share of a K step, so all waves reach the barrier together:
  //   A: 256 rows x 8 chunks of 16 bytes; thread t takes chunk (t & 7) of rows (t >> 3) + (T/8)*i;
  //   B: blocks of 4 k x 8 n, 16 x 32 of them; thread t takes blocks t + T*j (k quad id >> 5, n block
  //      id & 31), loads the four rows of each (16 bytes each) and transposes them in registers into
  //      eight 8-byte k-runs, one per column of the transposed tile.
  // 2048/T + 4*(512/T) 16-byte global loads per thread and K step: vector-memory instructions are
  // issued at a fixed rate per CU whatever their width, so wide loads keep the issue time short.
  const uint32_t a_row = tid >> 3, a_chunk = tid & 7u;
  const uint16_t* src_a = g.A + (size_t)(m0 + a_row) * g.K + a_chunk * 8;
  uint32_t a_dst[NA];  // LDS byte offsets inside a stage
#pragma unroll
  for (int i = 0; i < NA; ++i) a_dst[i] = tile_off<BK>(a_row + (T / 8) * i, a_chunk);
  // column c of a block goes to row 8*nb + c of the transposed tile, chunk kq / 2, half kq % 2
  const uint32_t b_nb = tid & 31u;
  const uint16_t* src_b = g.B + (size_t)((tid >> 5) * 4) * g.N + n0 + b_nb * 8;

  u32x4 la[NA], lb[NB][4];  // staging registers: A chunks, B rows
  auto load_a = [&](uint32_t kt, int i) {
    la[i] = *reinterpret_cast<const u32x4*>(src_a + (size_t)kt * BK + (size_t)((T / 8) * i) * g.K);
  };
  auto load_b = [&](uint32_t kt, int j, int i) {  // block j of this thread starts T/32 k quads further down
    lb[j][i] = *reinterpret_cast<const u32x4*>(src_b + ((size_t)kt * BK + (size_t)((T / 32) * 4 * j + i)) * g.N);
  };
  auto store_a = [&](uint32_t stage, int i) {
    *reinterpret_cast<u32x4*>(smem + stage * STAGE + a_dst[i]) = la[i];
  };
  // word w of the four rows holds columns 2w (low halves) and 2w+1 (high halves)
  auto store_b = [&](uint32_t stage, int j, int w) {
    unsigned char* sB = smem + stage * STAGE + A_BYTES;
    const uint32_t kq = (tid >> 5) + (T / 32) * (uint32_t)j;
    const uint32_t w0 = lb[j][0][w], w1 = lb[j][1][w], w2 = lb[j][2][w], w3 = lb[j][3][w];
    u32x2 ev, od;
    // low halves / high halves of two words side by side: one v_perm_b32 each (bytes 0-3 of the
    // selector's space are the second operand, 4-7 the first)
    ev.x = __builtin_amdgcn_perm(w1, w0, 0x05040100u); ev.y = __builtin_amdgcn_perm(w3, w2, 0x05040100u);
    od.x = __builtin_amdgcn_perm(w1, w0, 0x07060302u); od.y = __builtin_amdgcn_perm(w3, w2, 0x07060302u);
    const uint32_t n = b_nb * 8u + 2u * (uint32_t)w;
    *reinterpret_cast<u32x2*>(sB + tile_off_bt(n, kq >> 1) + (kq & 1u) * 8u) = ev;
    *reinterpret_cast<u32x2*>(sB + tile_off_bt(n + 1u, kq >> 1) + (kq & 1u) * 8u) = od;
  };

  // ---- global -> LDS (default schedule) ------------------------------------------------------
  // The A tile goes from global memory straight to LDS (global_load_lds_dwordx4: lane l of
  // a wave lands at byte 16 l of a 1 KiB block whose base M0 holds), without staging registers and LDS write
  // instructions.  Wave w fills blocks 4 w .. 4 w + 3 of a stage's A tile, 8 rows each: lane l is row l / 8 of
  // the block and chunk position l % 8, and fetches the chunk that the tile's swizzle puts there.  The loads
  // are issued from inline assembly: the compiler would make the next LDS access of any kind wait for such a
  // load (it cannot tell the load's destination from the tile being read).  They are therefore not in its
  // count of outstanding vector-memory operations; they complete in order with the others, so its own waits
  // stay sufficient (they may wait for more), and the kernel waits for them itself before the barrier.
  constexpr bool DIRECT = !PHASED;
  const uint32_t d_lds0 = kp::wave_uniform((uint32_t)(uintptr_t)smem + 4096u * wave);
  uint32_t d_off[4];  // byte offsets from the tile's first element (the base stays in scalar registers)
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t row = 32u * wave + 8u * (uint32_t)i + (lane >> 3);
    const uint32_t chunk = (lane & 7u) ^ ((row >> 1) & 7u);  // tile_off<64>: position = chunk ^ (row / 2) % 8
    d_off[i] = (row * g.K + chunk * 8u) * 2u;
  }
  const uint16_t* a_base = g.A + (size_t)m0 * g.K;
  // The B tile likewise, as it lies in memory: 64 rows (k) of 256 n, 512 bytes each; chunk c (8 n) of row k at
  // chunk position c ^ 4 (k % 4).  Wave w fills blocks 4 w .. 4 w + 3 of 1 KiB, two rows each.
  uint32_t db_off[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t row = 8u * wave + 2u * (uint32_t)i + (lane >> 5);
    const uint32_t chunk = (lane & 31u) ^ (4u * (row & 3u));
    db_off[i] = (row * g.N + chunk * 8u) * 2u;
  }
  const uint16_t* b_base = g.B + n0;
  // One load, its global address a scalar base (the tile's first element in this K step) plus the lane's 32-bit
  // byte offset, which never changes: no vector arithmetic per load (with a 64-bit pointer per lane and load
  // the kernel was 3.5 % slower).  M0 (the LDS base) is put back afterwards, the compiler does not expect
  // inline assembly to change it; one wait state between the write of M0 and the load that uses it.  The eight loads of a K step stay
  // separate statements: issued back to back from one block of assembly they made the uninstrumented kernel 4 %
  // slower (the address arithmetic of the next load no longer sits between two loads).
  auto direct_load = [&](const uint16_t* base, uint32_t off, uint32_t dst) {
    uint32_t saved_m0;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %3\n\ts_mov_b32 m0, %0"
                 : "=&s"(saved_m0) : "v"(off), "s"(dst), "s"(base) : "memory");
  };
  auto direct_one = [&](uint32_t kt, uint32_t stage, int idx) {
    const uint32_t dst = d_lds0 + stage * STAGE;
    if (idx < 4) direct_load(a_base + (size_t)kt * BK, d_off[idx], dst + (uint32_t)idx * 1024u);
    else direct_load(b_base + (size_t)kt * BK * g.N, db_off[idx - 4], dst + A_BYTES + (uint32_t)(idx - 4) * 1024u);
  };
  auto direct_tiles = [&](uint32_t kt, uint32_t stage) {
    const uint32_t dst = d_lds0 + stage * STAGE;
#pragma unroll
    for (int i = 0; i < 4; ++i) direct_load(a_base + (size_t)kt * BK, d_off[i], dst + (uint32_t)i * 1024u);
#pragma unroll
    for (int i = 0; i < 4; ++i) direct_load(b_base + (size_t)kt * BK * g.N, db_off[i], dst + A_BYTES + (uint32_t)i * 1024u);
  };

  const uint32_t wm = WAVES == 8 ? wave >> 2 : wave >> 1;  // wave position: 2 x 4 or 2 x 2
  const uint32_t wn = WAVES == 8 ? wave & 3u : wave & 1u;
  // Operand reads of the row-major B tile: ds_read_b64_tr_b16 hands lane j of a group of 16 lanes the elements
  // j, 16 + j, 32 + j, 48 + j of the 64 that the group's lanes address (4 each, lane after lane).  With lane i
  // of a group addressing B[k0 + i / 4][n0 + 4 (i % 4) ..+3], lane j receives B[k0 .. k0 + 3][n0 + j]: four
  // consecutive k of one column; two such reads make the eight k of the lane's MFMA operand.  Groups 0 and 1 are
  // columns 0-15 and 16-31 of the k octet 0, groups 2 and 3 the same columns of octet 1.
  uint32_t b_rd[TN];
  {
    const uint32_t bi = lane & 15u, bg = lane >> 4;
    const uint32_t k = 8u * (bg >> 1) + (bi >> 2);
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
      const uint32_t n = wn * (32 * TN) + (uint32_t)tn * 32u + 16u * (bg & 1u) + 4u * (bi & 3u);
      b_rd[tn] = k * 512u + ((((n >> 3) ^ (4u * (bi >> 2)))) << 4) + 8u * ((n >> 2) & 1u);
    }
  }
  auto read_b = [&](const unsigned char* sBt, int ks, int tn) -> bf16x8 {
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) s16x4* lds_s16x4;
    const unsigned char* at = sBt + b_rd[tn] + (uint32_t)(16 * ks) * 512u;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(at));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(at + 4u * 512u));
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
  };

  f32x16 acc[TN][4];                               // [tn][tm], transposed tiles (rows = n, cols = m)
#pragma unroll
  for (int a = 0; a < TN; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) acc[a][b] = f32x16{0};

  // prologue: K step 0 into stage 0 (and, stage by stage, K step 1 into the staging registers)
  const uint32_t KT = g.K / BK;
  if constexpr (DIRECT) {
    static_assert(WAVES == 8 && BK == 64, "four 1 KiB blocks of either tile per wave");
    direct_tiles(0, 0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the tiles of K step 0 have landed
  } else {
#pragma unroll
    for (int i = 0; i < NA; ++i) load_a(0, i);
#pragma unroll
    for (int i = 0; i < 4 * NB; ++i) load_b(0, i >> 2, i & 3);
#pragma unroll
    for (int i = 0; i < NA; ++i) store_a(0, i);
#pragma unroll
    for (int i = 0; i < 4 * NB; ++i) store_b(0, i >> 2, i & 3);
    if (KT > 1) {
#pragma unroll
      for (int i = 0; i < NA; ++i) load_a(1, i);
#pragma unroll
      for (int i = 0; i < 4 * NB; ++i) load_b(1, i >> 2, i & 3);
    }
  }
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");

  // Default schedule.  Iteration kt runs the MFMAs of K step kt on LDS stage kt & 1.  It starts by sending
  // both tiles of K step kt+1 from global memory to the other stage, eight loads per wave that have the whole
  // iteration to land; the wave waits for them, and for its LDS reads, right before the barrier.  The operands
  // of MFMA step ks+1 are requested before the MFMAs of step ks are issued, and the MFMAs of a K step's last
  // step are issued behind the barrier, after the loads and the first operand reads of the next iteration:
  // a wave comes back from the barrier with matrix work at hand while the first operands of the new stage
  // are on their way.
  // MORE (K step kt+1 exists) is compile-time so that the steady-state body is one basic block.
  // operands of the last MFMA step of a K step: its MFMAs are issued behind the barrier, in the next iteration
  bf16x8 af_p[4], bf_p[TN];
#pragma unroll
  for (int i = 0; i < 4; ++i) af_p[i] = bf16x8{0};
#pragma unroll
  for (int i = 0; i < TN; ++i) bf_p[i] = bf16x8{0};
  constexpr int kLoadEvery = 2;  // (measured: 1 and 3 are 3 to 7 % slower)
  auto mfma_pending = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
      for (int tm = 0; tm < 4; ++tm)
        acc[tn][tm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf_p[tn], af_p[tm], acc[tn][tm], 0, 0, 0);
  };
  auto iteration = [&](uint32_t kt, auto more_c, auto more2_c) {
    constexpr bool MORE = decltype(more_c)::value;
    const uint32_t stage = kt & 1u;
    const unsigned char* sA = smem + stage * STAGE;
    const unsigned char* sB = sA + A_BYTES;
    // operands of MFMA step ks + 1 are requested before the MFMAs of step ks are issued
    bf16x8 af[2][4], bfr[2][TN];
    auto read_step = [&](int ks, int buf) __attribute__((always_inline)) {
      const uint32_t chunk = (uint32_t)ks * 2u + (lane >> 5);
#pragma unroll
      for (int tm = 0; tm < 4; ++tm)
        af[buf][tm] = *reinterpret_cast<const bf16x8*>(sA + tile_off<BK>(wm * 128 + tm * 32 + (lane & 31u), chunk));
#pragma unroll
      for (int tn = 0; tn < TN; ++tn) bfr[buf][tn] = read_b(sB, ks, tn);
    };
    // load d of the next K step's tiles goes behind MFMA kLoadEvery * d + kLoadEvery - 1 of the iteration's 32
    auto load_behind = [&](uint32_t kt_, uint32_t stage_, int mfma) __attribute__((always_inline)) {
      if (mfma % kLoadEvery == kLoadEvery - 1 && mfma / kLoadEvery < 8) {
        __builtin_amdgcn_sched_barrier(0);
        direct_one(kt_ + 1, stage_ ^ 1u, mfma / kLoadEvery);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    read_step(0, 0);
    // the last MFMA step of the K step before (zeros the first time).  The loads of the next K step's tiles go
    // behind every second MFMA of the first sixteen: the loads of all waves queue up in one unit of the CU, and a
    // wave that issues its eight in a row waits there with no matrix work in flight; spread further, the last
    // ones land too late
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
      for (int tm = 0; tm < 4; ++tm) {
        acc[tn][tm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf_p[tn], af_p[tm], acc[tn][tm], 0, 0, 0);
        if constexpr (MORE) load_behind(kt, stage, tn * 4 + tm);
      }
    KP_COMMIT(ring, 3);  // the sites of the K step before: in its middle, in front of its barrier and behind it
#pragma unroll
    for (int ks = 0; ks + 1 < BK / 16; ++ks) {
      // ---- region 0: first half of the K step; region 1: second half
      if (ks == 1) KP_SITE_K(ring, 0, 0, 1);  // 16 MFMAs on either side
      read_step(ks + 1, (ks + 1) & 1);
#pragma unroll
      for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int tm = 0; tm < 4; ++tm) {
          acc[tn][tm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[ks & 1][tn], af[ks & 1][tm], acc[tn][tm], 0, 0, 0);
          if constexpr (MORE) load_behind(kt, stage, 8 * (ks + 1) + tn * 4 + tm);
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) af_p[i] = af[(BK / 16 - 1) & 1][i];
#pragma unroll
    for (int i = 0; i < TN; ++i) bf_p[i] = bfr[(BK / 16 - 1) & 1][i];
    // the tiles of the next K step have landed (no other vector-memory operation is in flight in the loop)
    if constexpr (MORE) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    KP_SITE_K(ring, 1, 1, 2);
    // ---- region 2: every wave is done with the stage ----------------------------------------------
    // (chained sites: nothing behind the barrier uses the clock just asked for, so nothing waits for it there)
    if constexpr (SITE == 1 || SITE == 3) asm volatile("s_barrier\n\ts_waitcnt lgkmcnt(0)" ::: "memory");
    else asm volatile("s_barrier" ::: "memory");
    if constexpr (MORE) KP_SITE_K(ring, 2, 2, 0); else KP_SITE_K(ring, 2, 2, 3);
  };
  // The same K step with its stages one after the other, each a region of its own (the stage-by-stage
  // instrumentation of a software-pipelined GEMM, Sec. 5.3): 2 the staging registers (K step kt+1) go to
  // the other LDS stage, 0 the global loads of K step kt+2 are issued, 3 the MFMAs of K step kt, 1 the
  // wait for this wave's LDS traffic and for the other waves.  Four sites and eight records per K step.
  // A record site pins its place in the instruction stream (it is a scheduling fence: nothing moves across
  // the clock read).  Without sites the compiler would be free to thread the stages through one another
  // again, and "the same schedule without record sites" would be another, faster schedule (measured: 135.5
  // against 140 us): so the uninstrumented form has a bare scheduling fence wherever the instrumented one
  // has a site.  SCHEDULE 2 leaves them out, for that comparison.
  auto stage_fence = [] { if constexpr (INSTR == 0 && SCHEDULE == 1) __builtin_amdgcn_sched_barrier(0); };
  auto iteration_phased = [&](uint32_t kt, auto more_c, auto more2_c) {
    constexpr bool MORE = decltype(more_c)::value, MORE2 = decltype(more2_c)::value;
    const uint32_t stage = kt & 1u;
    const unsigned char* sA = smem + stage * STAGE;
    const unsigned char* sB = sA + A_BYTES;
    if constexpr (MORE) {
#pragma unroll
      for (int i = 0; i < NA; ++i) store_a(stage ^ 1u, i);
#pragma unroll
      for (int i = 0; i < 4 * NB; ++i) store_b(stage ^ 1u, i >> 2, i & 3);
    }
    KP_SITE_K(ring, 1, 2, 0);
    stage_fence();
    if constexpr (MORE2) {
#pragma unroll
      for (int i = 0; i < NA; ++i) load_a(kt + 2, i);
#pragma unroll
      for (int i = 0; i < 4 * NB; ++i) load_b(kt + 2, i >> 2, i & 3);
    }
    KP_SITE_K(ring, 2, 0, 3);
    stage_fence();
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      const uint32_t chunk = ks * 2 + (lane >> 5);
      bf16x8 af[4], bfr[TN];
#pragma unroll
      for (int tm = 0; tm < 4; ++tm)
        af[tm] = *reinterpret_cast<const bf16x8*>(sA + tile_off<BK>(wm * 128 + tm * 32 + (lane & 31u), chunk));
#pragma unroll
      for (int tn = 0; tn < TN; ++tn)
        bfr[tn] = *reinterpret_cast<const bf16x8*>(sB + tile_off_bt(wn * (32 * TN) + tn * 32 + (lane & 31u), chunk));
#pragma unroll
      for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int tm = 0; tm < 4; ++tm)
          acc[tn][tm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[tn], af[tm], acc[tn][tm], 0, 0, 0);
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // (nothing of this wave's is in flight any more: see above)
    KP_SITE_K(ring, 3, 3, 1);
    stage_fence();
    asm volatile("s_barrier\n\ts_waitcnt lgkmcnt(0)" ::: "memory");
    KP_COMMIT(ring, 4);
    if constexpr (MORE) KP_SITE_K(ring, 0, 1, 2); else KP_SITE_K(ring, 0, 1, 4);
    stage_fence();
  };
  constexpr std::true_type yes{};
  constexpr std::false_type no{};
  if constexpr (PHASED) {
    KP_SITE_K(ring, 0, kp::kNoRegion, 2);
    for (uint32_t kt = 0; kt + 2 < KT; ++kt) iteration_phased(kt, yes, yes);
    if (KT >= 2) iteration_phased(KT - 2, yes, no);
    iteration_phased(KT - 1, no, no);
  } else {
    if constexpr (SITE == 6) {  // (they fill the first two places of the first batch)
      kp::site_chain<0, REALTIME>(ring);
      kp::site_chain<1, REALTIME>(ring);
    }
    KP_SITE_K(ring, 2, kp::kNoRegion, 0);
    for (uint32_t kt = 0; kt + 2 < KT; ++kt) iteration(kt, yes, yes);
    if (KT >= 2) iteration(KT - 2, yes, no);
    iteration(KT - 1, no, no);
    mfma_pending();
    KP_COMMIT(ring, 3);
  }

  // ---- region 3 (4 with the stages apart): epilogue ---------------------------------------------------
  // transposed tile: register v of lane l is C[m, n] with m = l%32 and n = 8*(v/4) + 4*(l/32) + v%4
#pragma unroll
  for (int tm = 0; tm < 4; ++tm) {
    const uint32_t row = m0 + wm * 128 + tm * 32 + (lane & 31u);
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint32_t col = n0 + wn * (32 * TN) + tn * 32 + 8 * q + 4 * (lane >> 5);
        u32x2 pk;
        pk.x = bf16_pack_rne(acc[tn][tm][4 * q + 0], acc[tn][tm][4 * q + 1]);
        pk.y = bf16_pack_rne(acc[tn][tm][4 * q + 2], acc[tn][tm][4 * q + 3]);
        *reinterpret_cast<u32x2*>(g.C + (size_t)row * g.N + col) = pk;
      }
    }
  }
  KP_SITE_K(ring, PHASED ? 1 : 0, PHASED ? 4 : 3, kp::kNoRegion);
  if constexpr (INSTR != 0) {
    kp::TraceGeom tg{g.n_wg, (uint32_t)WAVES >> g.group_log2, PHASED ? 5u : 4u, g.cap_hbm, g.flags};
    if constexpr (SITE == 6) {
      // the site that closed the epilogue and, with the stages apart, the one that opened it
      kp::chain_commit<PHASED ? 2 : 1>(ring);
      kp::ring_finish<REALTIME>(ring, g.cap_lds, g.trace, tg, wg, g.rec_cost, GemmChain<PHASED>{});
    } else {
      kp::sites_end<SITE>(ring);
      kp::ring_finish<REALTIME>(ring, g.cap_lds, g.trace, tg, wg, g.rec_cost);
    }
  }
}

}  // namespace

// ------------------------------------------------------------------------------------------
namespace {

struct GemmShape { int bm, bn, bk, waves, regions; };

// Waves per workgroup of the 256x256x64 kernel.  The kernel template also builds with 4 waves
// (128x128 of C per wave, accumulators in AGPRs, one wave per SIMD); on MI355X that variant measured
// about the same speed (146 vs 137-142 us at 4096^3: a third less LDS read traffic and a short
// barrier, but a single wave per SIMD hides less), so only the 8-wave form is instantiated.
constexpr int kBigWaves = 8;

bool pick_shape(int M, int N, int K, GemmShape* s) {
  if (M <= 0 || N <= 0 || K <= 0) return false;
  // the large tile only pays off once there are enough tiles to spread over the chip
  if (M % 256 == 0 && N % 256 == 0 && K % 64 == 0 && (M / 256) * (N / 256) >= 16) { *s = GemmShape{256, 256, 64, kBigWaves, 4}; return true; }
  if (M % 64 == 0 && N % 64 == 0 && K % 32 == 0) { *s = GemmShape{64, 64, 32, 4, 3}; return true; }
  return false;
}

template <int INSTR, int WAVES, int SCHEDULE>
kp_status launch_big(const GemmArgs& g, int n_wg, size_t ring_bytes, hipStream_t st) {
  static thread_local int attr_dev = -1;  // the attribute is kept per device
  int dev = 0;
  KP_HIP_TRY(hipGetDevice(&dev));
  if (attr_dev != dev) {
    KP_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kp_gemm_big<INSTR, WAVES, SCHEDULE>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
    attr_dev = dev;
  }
  hipLaunchKernelGGL((kp_gemm_big<INSTR, WAVES, SCHEDULE>), dim3(n_wg), dim3(WAVES * 64), kBigTileBytes + ring_bytes, st, g);
  KP_HIP_TRY(hipGetLastError());
  return KP_OK;
}

template <int INSTR>
kp_status launch_big_w(bool phased, const GemmArgs& g, int n_wg, size_t ring_bytes, hipStream_t st) {
  return phased ? launch_big<INSTR, kBigWaves, 1>(g, n_wg, ring_bytes, st)
                : launch_big<INSTR, kBigWaves, 0>(g, n_wg, ring_bytes, st);
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
  const uint32_t regions = region_mask & ~(KP_MASK_FLUSH | KP_MASK_WAVE_GROUP | KP_MASK_PHASES | KP_MASK_REALTIME | KP_MASK_COLLAB | KP_MASK_UNFENCED);
  const bool unfenced = (region_mask & KP_MASK_UNFENCED) != 0u;
  const bool realtime = (region_mask & KP_MASK_REALTIME) != 0u, collab = (region_mask & KP_MASK_COLLAB) != 0u;
  const bool phased = (region_mask & KP_MASK_PHASES) != 0u;
  if (phased) {
    if (s.bm != 256) return kp::fail(KP_ERR_INVALID_ARG, "KP_MASK_PHASES: only the 256x256x64 kernel has the stage-by-stage K step");
    s.regions = 5;
  }
  if (unfenced && (!phased || regions != 0u))
    return kp::fail(KP_ERR_INVALID_ARG, "KP_MASK_UNFENCED goes with KP_MASK_PHASES and no region");
  const uint32_t flush = region_mask >> 31;
  const uint32_t group_log2 = (region_mask & KP_MASK_WAVE_GROUP) ? 2u : 0u;
  const int streams = s.waves >> group_log2;
  const int n_wg = (M / s.bm) * (N / s.bn);
  hipStream_t st = static_cast<hipStream_t>(stream);
  GemmArgs g{};
  g.A = static_cast<const uint16_t*>(A); g.B = static_cast<const uint16_t*>(B); g.C = static_cast<uint16_t*>(C);
  g.M = (uint32_t)M; g.N = (uint32_t)N; g.K = (uint32_t)K;
  g.region_mask = regions; g.trace = trace_buf; g.n_wg = (uint32_t)n_wg; g.flush = flush;
  g.group_log2 = group_log2;
  g.collab = collab ? 1u : 0u;
  g.flags = (flush ? KP_FLAG_FLUSH : 0u) | (realtime ? KP_FLAG_REALTIME : 0u) | (collab ? KP_FLAG_HW_IDS : 0u);
  const bool big = s.bm == 256;
  if (regions == 0) {  // uninstrumented baseline: no ring, no record sites
    if (big && unfenced) return launch_big<0, kBigWaves, 2>(g, n_wg, 0, st);
    if (big) return launch_big_w<0>(phased, g, n_wg, 0, st);
    hipLaunchKernelGGL(kp_gemm_small<0>, dim3(n_wg), dim3(256), 0, st, g);
    KP_HIP_TRY(hipGetLastError());
    return KP_OK;
  }
  if (!trace_buf) return kp::fail(KP_ERR_INVALID_ARG, "trace_buf is NULL but region_mask enables regions");
  if (regions >> s.regions) return kp::fail(KP_ERR_INVALID_ARG, "region_mask enables regions this kernel does not have (%d regions)", s.regions);
  if (((uintptr_t)trace_buf) & 15u) return kp::fail(KP_ERR_INVALID_ARG, "trace_buf must be 16-byte aligned");
  if (trace_cap % (size_t)streams) return kp::fail(KP_ERR_TRACE_TOO_SMALL, "trace_cap must be a multiple of %d record streams", streams);
  const size_t cap_wave = trace_cap / (size_t)streams;
  if (!kp::is_pow2(cap_wave) || cap_wave < 2 || cap_wave > (1u << 19))
    return kp::fail(KP_ERR_TRACE_TOO_SMALL, "trace_cap/streams = %zu must be a power of two >= 2", cap_wave);
  uint32_t cap_lds = (uint32_t)cap_wave;
  if (flush && cap_lds > 64) cap_lds = 64;
  const size_t ring_bytes = (size_t)cap_lds * 8 * streams + (group_log2 ? 16 : 0);  // (16: see chain_begin)
  if (ring_bytes > 32 * 1024) return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "LDS ring of %zu bytes exceeds the 32 KiB budget", ring_bytes);
  g.cap_lds = cap_lds; g.cap_hbm = (uint32_t)cap_wave; g.rec_cost = kp::rec_cost();
  // small kernel: every region, circular, and fewer than 2^20 records per wave (6 per K step): lean record sites
  const bool lean = !flush && !group_log2 && !realtime && !collab && regions == (1u << s.regions) - 1u && K <= (1 << 22);
  // The large kernel chains its sites whenever the strategy is circular and one lane stores: the region mask,
  // wave-group records and the constant-rate clock all keep that form.
  const bool chained = !flush && !collab;
  if (big) return chained ? (realtime ? launch_big_w<5>(phased, g, n_wg, ring_bytes, st) : launch_big_w<2>(phased, g, n_wg, ring_bytes, st))
                          : (realtime ? launch_big_w<3>(phased, g, n_wg, ring_bytes, st) : launch_big_w<1>(phased, g, n_wg, ring_bytes, st));
  if (lean) hipLaunchKernelGGL(kp_gemm_small<2>, dim3(n_wg), dim3(256), ring_bytes, st, g);
  else if (realtime) hipLaunchKernelGGL(kp_gemm_small<3>, dim3(n_wg), dim3(256), ring_bytes, st, g);
  else      hipLaunchKernelGGL(kp_gemm_small<1>, dim3(n_wg), dim3(256), ring_bytes, st, g);
  KP_HIP_TRY(hipGetLastError());
  return KP_OK;
}

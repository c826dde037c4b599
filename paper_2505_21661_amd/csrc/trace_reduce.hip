// GPU trace decode / pair / reduce (kp_trace_reduce).
//
// The paper stores START/END records unpaired, per warp, in a ring whose tail survives, and
// aligns them at "trace replay" on the host (Sec. 4.2 "SM-level Data Layout", "Shared Memory
// Circular Buffer"; Sec. 4.3).  Here replay runs on the GPU: one persistent decoder workgroup
// takes one recorded workgroup at a time and keeps it in LDS as a clock word and a metadata byte
// per record.
//   A  every record is scattered to its rank (seq - first surviving seq), which undoes ring
//      rotation and out-of-order flushes in O(1) per record; the records of the next workgroup
//      are requested before the results of the current one are written;
//   B  a lane takes the records of 8 rounds of 128 consecutive ranks, two neighbours per round;
//      an END is paired iff the nearest earlier record of its (wave, region) is a START --
//      usually the rank just below, in the same lane or the lane below (DPP);
//      d = (u32)(ts_end - ts_start) minus the constant record cost (Sec. 4.3) goes to the
//      per-(wave, region) sums and the log2 histogram with LDS atomics;
//   C  the paired records of all waves are sorted by clock: counting sort into time cells (one
//      LDS atomic per record gives cell and arrival slot) and a prefix sum over the cells put
//      them in cell order;
//   D  every lane takes 16 consecutive records of that sequence and finishes the order in
//      registers (a sorting network over its own records, then a merge of its outer halves with
//      the neighbouring lanes').  The number of waves that have each region open is kept
//      bit-sliced (plane k = bit k of every region's count); a first pass gives each lane's net
//      change, a prefix sum over lanes and waves the state at the start of each lane's stretch,
//      and the second pass the set of open regions after every record.  The time two regions
//      are both open is the sum over the stretches between records of length * open(a) * open(b):
//      a matrix product, taken by the matrix cores 64 stretches at a time;
//   E  the per-(workgroup, wave, region) results go to HBM and into running totals, which live in
//      LDS and reach HBM once per decoder workgroup.
// Traces outside what the register sort covers (more than 16 regions, a span of 2^26 ticks or
// more, a time cell with more than 17 records) rank the records inside their cell by comparing
// clocks and add every switch of a region to the region-pair sums with LDS atomics.
// A workgroup with a corrupt record (bad field, duplicated seq) has holes in its ranks; it is rare,
// takes no part in the overlap statistics and is paired by a plain serial walk per (wave, region).
#include "kp_reduce.h"

#include <type_traits>

namespace {

using namespace kp_reduce;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr uint32_t kSeqMask = 0xFFFFFu;
// staged metadata byte: bits 5:0 region (63 = no record), 6 paired, 7 END
constexpr uint32_t kRegion = 0x3Fu, kEmpty = 0x3Fu, kPaired = 0x40u, kEnd = 0x80u;
constexpr int kNR = 16;                       // positions per lane
constexpr uint32_t kWaveSpan = 64 * kNR;      // positions per hardware wave
constexpr uint32_t kMaxCellWindow = 17;       // fullest time cell the sweep's register sort covers
constexpr uint32_t kMaxRecPerWg = 16384;
constexpr uint32_t kMaxLds = 160 * 1024;
constexpr uint32_t kHistStride = 65;  // histogram rows 65 words apart: equal bins of different regions, different banks

// steps after which kp_trace_reduce_steps can leave a workgroup
enum { kStepOrdered = 1, kStepPaired, kStepCounted, kStepCellSums, kStepPlaced, kStepRanked, kStepSorted, kStepSwept };

// per-workgroup temporaries (u32 words in LDS)
enum { T_INVALID = 0, T_FIELDVALID, T_DISORDER, T_OCCUPIED, T_NONMONO, T_PAIRS, T_STARTS, T_ENDS,
       T_EVENTS, T_MARKS, T_WIDE, T_MAXCELL, T_HELD, T_COUNT };  // T_HELD stays last

struct DecodeParams {
  const uint32_t* wg_hdrs;  // 32 words per recorded workgroup
  const u32x4* records;     // two records per 16-byte load
  uint64_t* out;
  uint32_t n_wg, W, R, cap, cap_log2, rec_cost, flush;
  uint32_t nrec;            // record slots per recorded workgroup
  uint32_t ncopy;           // copies of the per-(wave, region) sums: 1, 2 or 4
  uint32_t stop_after;      // 0: everything; else leave each workgroup after this step (timing only), see kStep*
};

__host__ __device__ constexpr uint32_t align16(uint32_t x) { return (x + 15u) & ~15u; }
constexpr uint32_t kMaxPerWave = 1024;  // entries of the per-(wave, region) sums, copies included

// LDS of a decoder workgroup of BLOCK threads, byte offsets.  Every array is sized for the largest
// geometry the kernel takes, so that all addresses are compile-time constants.
template <int BLOCK>
struct Lds {
  static constexpr uint32_t npos = BLOCK * kNR;
  static constexpr uint32_t clk = 0;                                       // 4 words of padding after every 64
  static constexpr uint32_t meta = align16(clk + (npos + npos / 16) * 4);
  static constexpr uint32_t cells = align16(meta + npos + 16);             // one 16-bit counter per time cell, npos cells, + the total
  static constexpr uint32_t ctr = align16(cells + (npos / 2 + 4) * 4);
  static constexpr uint32_t tmp = ctr + 16 * 8;
  static constexpr uint32_t misc = align16(tmp + T_COUNT * 4);
  static constexpr uint32_t vf = misc + 4 * 4;
  static constexpr uint32_t wtot = vf + 32 * 8;
  static constexpr uint32_t ptot = wtot + 16 * 4;
  static constexpr uint32_t hist = ptot + 16 * 8 * 4;
  static constexpr uint32_t oacc = align16(hist + KP_MAX_REGIONS * kHistStride * 4);
  static constexpr uint32_t oacc32 = oacc + KP_MAX_REGIONS * KP_MAX_REGIONS * 8;
  static constexpr uint32_t reg_sum = align16(oacc32 + KP_MAX_REGIONS * (KP_MAX_REGIONS + 1) * 4);
  static constexpr uint32_t reg_max = reg_sum + KP_MAX_REGIONS * 8;
  static constexpr uint32_t reg_min = reg_max + KP_MAX_REGIONS * 4;
  static constexpr uint32_t pw_pack = reg_min + KP_MAX_REGIONS * 4;
  static constexpr uint32_t pw_max = pw_pack + kMaxPerWave * 8;
  static constexpr uint32_t pw_min = pw_max + kMaxPerWave * 4;
  static constexpr uint32_t total = pw_min + kMaxPerWave * 4;
  static_assert(total <= kMaxLds, "decoder LDS exceeds one CU");
};

// Word of the clock array that holds position i: 4 words of padding after every 64, so that the
// 64 lanes of a wave reading 16 consecutive words each (64 bytes apart) spread over all banks.
__device__ __forceinline__ uint32_t clk_word(uint32_t i) { return i + ((i >> 6) << 2); }

// Lane l receives the value of lane l-1; lane 0 receives `lane0` (DPP wave shift right by one).
__device__ __forceinline__ uint32_t wave_shr1(uint32_t v, uint32_t lane0) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)lane0, (int)v, 0x138, 0xF, 0xF, false);
}

// The DPP steps of an inclusive scan over the 64 lanes: four shifts inside each row of 16, then the
// last lane of row 0/2 into row 1/3 and the last lane of the lower half into the upper half.  Lanes
// without a source read 0.
template <int STEP> __device__ __forceinline__ uint32_t scan_src(uint32_t v) {
  if (STEP == 0) return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xF, 0xF, false);  // row_shr:1
  if (STEP == 1) return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xF, 0xF, false);  // row_shr:2
  if (STEP == 2) return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xF, 0xF, false);  // row_shr:4
  if (STEP == 3) return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xF, 0xF, false);  // row_shr:8
  if (STEP == 4) return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xA, 0xF, false);  // row_bcast:15
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xC, 0xF, false);                 // row_bcast:31
}

__device__ __forceinline__ uint32_t wave_scan_add(uint32_t v) {
  v += scan_src<0>(v); v += scan_src<1>(v); v += scan_src<2>(v);
  v += scan_src<3>(v); v += scan_src<4>(v); v += scan_src<5>(v);
  return v;
}

// Sum over the wave, added to tmp[which] by the last lane.
__device__ __forceinline__ void add_tmp(uint32_t* tmp, int which, uint32_t v) {
  v = wave_scan_add(v);
  if ((threadIdx.x & 63u) == 63u && v) atomicAdd(&tmp[which], v);
}

// a += b for bit-sliced numbers: plane k holds bit k of 32 independent counters, modulo 2^PLANES.
template <int PLANES>
__device__ __forceinline__ void planes_add(uint32_t (&a)[PLANES], const uint32_t (&b)[PLANES]) {
  uint32_t c = 0;
#pragma unroll
  for (int k = 0; k < PLANES; ++k) {
    const uint32_t s = a[k] ^ b[k];
    const uint32_t g = a[k] & b[k];
    a[k] = s ^ c;
    c = g | (s & c);
  }
}

// counter[bit of x] += 1 (dm = 0) or -= 1 (dm = all ones); x is zero or one-hot.
template <int PLANES>
__device__ __forceinline__ void planes_step(uint32_t (&pl)[PLANES], uint32_t x, uint32_t dm) {
  uint32_t carry = x;
#pragma unroll
  for (int k = 0; k < PLANES; ++k) { const uint32_t o = pl[k]; pl[k] = o ^ carry; carry &= o ^ dm; }
}

// Batcher's odd-even merge sort of N registers: a fixed network (63 exchanges for 16 words, 384 for 48),
// every index known at compile time.
template <int N>
__device__ __forceinline__ void network_sort(uint32_t (&key)[N]) {
#pragma unroll
  for (int pp = 1; pp < N; pp <<= 1) {
#pragma unroll
    for (int k = pp; k >= 1; k >>= 1) {
#pragma unroll
      for (int j = k % pp; j + k < N; j += 2 * k) {
#pragma unroll
        for (int i = 0; i < (k < N - j - k ? k : N - j - k); ++i) {
          if ((i + j) / (2 * pp) == (i + j + k) / (2 * pp)) {
            const uint32_t x = key[i + j], y = key[i + j + k];
            key[i + j] = x < y ? x : y;
            key[i + j + k] = x < y ? y : x;
          }
        }
      }
    }
  }
}

// Ascending order of 8 registers that first rise and then fall (or the reverse): 12 exchanges.
__device__ __forceinline__ void bitonic_merge8(uint32_t (&v)[8]) {
#pragma unroll
  for (int k = 4; k >= 1; k >>= 1) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if ((i & k) == 0) {
        const uint32_t x = v[i], y = v[i + k];
        v[i] = x < y ? x : y;
        v[i + k] = x < y ? y : x;
      }
    }
  }
}

// The sweep works on one word per record of the sequence: clock << 6 | region << 1 | END; records with
// equal words are interchangeable.  A place past the end of the sequence holds `fake`: the largest
// clock of the workgroup with a region number that no record has, so that it sorts last, opens no
// region and the stretch in front of it has an honest length.
// Fields of such a word.
__device__ __forceinline__ uint32_t key_clock(uint32_t k) { return k >> 6; }
__device__ __forceinline__ uint32_t key_region_bit(uint32_t k) { return 1u << ((k >> 1) & 31u); }  // bit 31 for a place past the end: above every region
__device__ __forceinline__ uint32_t key_end_mask(uint32_t k) { return (uint32_t)__builtin_amdgcn_sbfe((int)k, 0, 1); }  // all ones for an END

// The 16 records of the clock-sorted sequence that lane `tid` of the sweep owns, from a sequence that
// is only ordered cell by cell (inside a cell the records stand in arrival order).  Cells follow one
// another in clock order, so sorting the words sorts every cell and moves no record out of its cell.
//
// Form for cells of at most 9 records: the lane sorts its own 16 places and puts them back; a cell that
// lies across the boundary to the next lane then has at most 8 records on either side, all of them in
// the upper half here and in the lower half there, so merging these two halves (both sorted) and
// handing the lower 8 back to this lane, the upper 8 to the next one finishes the job.  Each lane does
// that for its lower half with the lane below and for its upper half with the lane above: the larger
// (smaller) of element i of one run and element 7 - i of the other are the upper (lower) 8 of the two
// runs, in rising-then-falling order.  Contains one workgroup barrier.
template <uint32_t NPOS>
__device__ __forceinline__ void sorted_own(uint32_t* clk, uint32_t tid, uint32_t n_events, uint32_t fake, uint32_t (&key)[kNR]) {
  const uint32_t g0 = tid * kNR;
  u32x4* own = reinterpret_cast<u32x4*>(clk + clk_word(g0));
#pragma unroll
  for (int x = 0; x < kNR / 4; ++x) {
    const u32x4 v = own[x];
    key[4 * x] = v.x; key[4 * x + 1] = v.y; key[4 * x + 2] = v.z; key[4 * x + 3] = v.w;
  }
  if (__builtin_amdgcn_ballot_w64(g0 + kNR > n_events)) {
#pragma unroll
    for (int y = 0; y < kNR; ++y) key[y] = g0 + y < n_events ? key[y] : fake;
  }
  network_sort<kNR>(key);
  own[0] = u32x4{key[0], key[1], key[2], key[3]};
  own[1] = u32x4{key[4], key[5], key[6], key[7]};
  own[2] = u32x4{key[8], key[9], key[10], key[11]};
  own[3] = u32x4{key[12], key[13], key[14], key[15]};
  __syncthreads();
  {
    const u32x4* below = reinterpret_cast<const u32x4*>(clk + clk_word((tid > 0 ? tid - 1 : 0) * kNR));
    const u32x4* above = reinterpret_cast<const u32x4*>(clk + clk_word((tid + 1 < NPOS / kNR ? tid + 1 : tid) * kNR));
    const u32x4 b0 = below[2], b1 = below[3], a0 = above[0], a1 = above[1];
    const uint32_t lo_gate = tid > 0 ? 0xFFFFFFFFu : 0u;               // no lane below: nothing comes up
    const uint32_t hi_fill = tid + 1 < NPOS / kNR ? 0u : 0xFFFFFFFFu;  // no lane above: nothing comes down
    const uint32_t bw[8] = {b0.x & lo_gate, b0.y & lo_gate, b0.z & lo_gate, b0.w & lo_gate,
                            b1.x & lo_gate, b1.y & lo_gate, b1.z & lo_gate, b1.w & lo_gate};
    const uint32_t aw[8] = {a0.x | hi_fill, a0.y | hi_fill, a0.z | hi_fill, a0.w | hi_fill,
                            a1.x | hi_fill, a1.y | hi_fill, a1.z | hi_fill, a1.w | hi_fill};
    uint32_t lo[8], hi[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      lo[i] = key[7 - i] > bw[i] ? key[7 - i] : bw[i];         // upper 8 of (upper half below, own lower half)
      hi[i] = key[8 + i] < aw[7 - i] ? key[8 + i] : aw[7 - i];  // lower 8 of (own upper half, lower half above)
    }
    bitonic_merge8(lo);
    bitonic_merge8(hi);
#pragma unroll
    for (int i = 0; i < 8; ++i) { key[i] = lo[i]; key[8 + i] = hi[i]; }
  }
}

// Ascending order of 16 registers that first rise and then fall (or the reverse): 32 exchanges.
__device__ __forceinline__ void bitonic_merge16(uint32_t (&v)[kNR]) {
#pragma unroll
  for (int k = 8; k >= 1; k >>= 1) {
#pragma unroll
    for (int i = 0; i < kNR; ++i) {
      if ((i & k) == 0) {
        const uint32_t x = v[i], y = v[i + k];
        v[i] = x < y ? x : y;
        v[i + k] = x < y ? y : x;
      }
    }
  }
}

// Form for cells of up to 17 records: a cell then lies in at most two neighbouring lanes, with up to 16
// records in either.  The lane sorts its own 16 places; then lanes 2m and 2m + 1 merge their runs (the
// lower lane keeps the lower 16 of the 32, the upper lane the upper 16), and after that lanes 2m + 1 and
// 2m + 2 do the same.  The second merge moves no record across the boundary the first one settled: what
// it hands down to lane 2m + 1 belongs to the cell that lies across the boundary above, and that cell
// has no record in lane 2m (it would hold 18).  Contains three workgroup barriers.
template <uint32_t NPOS>
__device__ __forceinline__ void sorted_pairs(uint32_t* clk, uint32_t tid, uint32_t n_events, uint32_t fake, uint32_t (&key)[kNR]) {
  const uint32_t g0 = tid * kNR;
  u32x4* own = reinterpret_cast<u32x4*>(clk + clk_word(g0));
#pragma unroll
  for (int x = 0; x < kNR / 4; ++x) {
    const u32x4 v = own[x];
    key[4 * x] = v.x; key[4 * x + 1] = v.y; key[4 * x + 2] = v.z; key[4 * x + 3] = v.w;
  }
  if (__builtin_amdgcn_ballot_w64(g0 + kNR > n_events)) {
#pragma unroll
    for (int y = 0; y < kNR; ++y) key[y] = g0 + y < n_events ? key[y] : fake;
  }
  network_sort<kNR>(key);
#pragma unroll
  for (int round = 0; round < 2; ++round) {
    own[0] = u32x4{key[0], key[1], key[2], key[3]};
    own[1] = u32x4{key[4], key[5], key[6], key[7]};
    own[2] = u32x4{key[8], key[9], key[10], key[11]};
    own[3] = u32x4{key[12], key[13], key[14], key[15]};
    __syncthreads();
    // round 0: partner of lane t is t ^ 1; round 1: the other neighbour (the first and the last lane have none)
    const bool upper = ((tid ^ (uint32_t)round) & 1u) != 0u;  // this lane keeps the upper 16 of the merge
    const bool alone = round == 1 && (tid == 0u || tid + 1u == NPOS / kNR);
    const uint32_t partner = upper ? tid - 1u : tid + 1u;
    const u32x4* other = reinterpret_cast<const u32x4*>(clk + clk_word((alone ? tid : partner) * kNR));
    const u32x4 p0 = other[0], p1 = other[1], p2 = other[2], p3 = other[3];
    const uint32_t pw[kNR] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w, p2.x, p2.y, p2.z, p2.w, p3.x, p3.y, p3.z, p3.w};
    // the larger (smaller) of element i of one run and element 15 - i of the other: the upper (lower) 16
    const uint32_t neutral = upper ? 0u : 0xFFFFFFFFu;
#pragma unroll
    for (int i = 0; i < kNR; ++i) {
      const uint32_t x = key[i], y = alone ? neutral : pw[kNR - 1 - i];
      const uint32_t lo = x < y ? x : y, hi = x < y ? y : x;
      key[i] = upper ? hi : lo;
    }
    bitonic_merge16(key);
    if (round == 0) __syncthreads();  // every lane has read its partner's run before it is overwritten
  }
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

// finalize (one workgroup): cnt from the histogram, O = Otmp + Otmp^T off the diagonal, U = diag,
// F = O/U.  Otmp is what the main kernels staged in the F area.
__global__ void kp_reduce_finalize(uint64_t* out, uint32_t n_wg, uint32_t W, uint32_t R) {
  const StatsLayout l = stats_layout(n_wg, W, R);
  const uint32_t tid = threadIdx.x;
  for (uint32_t r = tid; r < R; r += blockDim.x) {
    uint64_t c = 0;
    for (int b = 0; b < 64; ++b) c += out[l.hist + (size_t)r * 64 + b];
    out[l.cnt + r] = c;
    out[l.U + r] = out[l.F + (size_t)r * R + r];
  }
  for (uint32_t i = tid; i < R * R; i += blockDim.x) {
    const uint32_t a = i / R, b = i % R;
    out[l.O + i] = a == b ? out[l.F + i] : out[l.F + i] + out[l.F + (size_t)b * R + a];
  }
  __syncthreads();  // (a workgroup's own global stores are visible to it after the barrier)
  for (uint32_t i = tid; i < R * R; i += blockDim.x) {
    const uint64_t u = out[l.U + i / R], o = out[l.O + i];
    reinterpret_cast<double*>(out)[l.F + i] = u ? (double)o / (double)u : 0.0;
  }
}

// ------------------------------------------------------------------------------------------
// Position p = wave*cap_wave + rank indexes the staged records.  Hardware wave h of the decoder
// owns positions [h*1024, h*1024 + 1024) and lane l takes position h*1024 + 64*j + l in round j,
// so that neighbouring lanes hold neighbouring ranks.
template <int BLOCK, int PLANES>
__global__ __launch_bounds__(BLOCK) void kp_reduce_main(DecodeParams p) {
  using L = Lds<BLOCK>;
  __shared__ __align__(16) unsigned char smem[L::total];
  uint32_t* clk = reinterpret_cast<uint32_t*>(smem + L::clk);
  uint8_t* meta = smem + L::meta;
  uint32_t* cells = reinterpret_cast<uint32_t*>(smem + L::cells);  // cell c: half (c & 1) of word c >> 1
  uint32_t* hist = reinterpret_cast<uint32_t*>(smem + L::hist);
  unsigned long long* oacc = reinterpret_cast<unsigned long long*>(smem + L::oacc);
  uint32_t* oacc32 = reinterpret_cast<uint32_t*>(smem + L::oacc32);  // this workgroup's sums modulo 2^32
  unsigned long long* reg_sum = reinterpret_cast<unsigned long long*>(smem + L::reg_sum);
  uint32_t* reg_max = reinterpret_cast<uint32_t*>(smem + L::reg_max);
  uint32_t* reg_min = reinterpret_cast<uint32_t*>(smem + L::reg_min);
  unsigned long long* pw_pack = reinterpret_cast<unsigned long long*>(smem + L::pw_pack);
  uint32_t* pw_max = reinterpret_cast<uint32_t*>(smem + L::pw_max);
  uint32_t* pw_min = reinterpret_cast<uint32_t*>(smem + L::pw_min);
  unsigned long long* ctr = reinterpret_cast<unsigned long long*>(smem + L::ctr);
  uint32_t* tmp = reinterpret_cast<uint32_t*>(smem + L::tmp);
  uint32_t* misc = reinterpret_cast<uint32_t*>(smem + L::misc);  // [0] span overflow, [1] cell scale, [2] span
  uint2* sVF = reinterpret_cast<uint2*>(smem + L::vf);           // per wave: records held, first surviving seq
  uint32_t* wtot = reinterpret_cast<uint32_t*>(smem + L::wtot);
  uint32_t* ptot = reinterpret_cast<uint32_t*>(smem + L::ptot);

  constexpr uint32_t NPOS = BLOCK * kNR, NCELL = NPOS;
  // The last four words of the clock array are padding that no position maps to, and the metadata
  // array has 16 spare bytes: stores of lanes that have nothing to store go there instead of branching.
  constexpr uint32_t kSpareWord = NPOS + NPOS / 16 - 1;
  const uint32_t tid_k = threadIdx.x;
  // The kernel arguments arrive as one block of scalar registers.  Each one used in the loop gets a
  // register of its own through an opaque move: when scalar registers run short the compiler then parks
  // and fetches single values instead of the whole block.
  auto own_reg = [](uint32_t x) -> uint32_t { uint32_t y; asm("s_mov_b32 %0, %1" : "=s"(y) : "s"(x)); return y; };
  const uint32_t W = own_reg(p.W), R = own_reg(p.R), cap = own_reg(p.cap), nrec = own_reg(p.nrec);
  const uint32_t capm = cap - 1, cl2 = own_reg(p.cap_log2);
  const uint32_t n_wg = own_reg(p.n_wg), n_copies = own_reg(p.ncopy), stop_after = own_reg(p.stop_after);
  const uint32_t rec_cost = own_reg(p.rec_cost), flush = own_reg(p.flush);
  const StatsLayout SL = stats_layout(n_wg, W, R);
  if (p.out[H_STATUS] != 0) return;  // device header did not match the launch geometry

  for (uint32_t i = tid_k; i < R * kHistStride; i += BLOCK) hist[i] = 0;
  for (uint32_t i = tid_k; i < R * R; i += BLOCK) oacc[i] = 0;
  for (uint32_t i = tid_k; i < R * (R | 1u); i += BLOCK) oacc32[i] = 0;
  for (uint32_t i = tid_k; i < R; i += BLOCK) { reg_sum[i] = 0; reg_max[i] = 0; reg_min[i] = 0xFFFFFFFFu; }
  for (uint32_t i = tid_k; i < n_copies * W * R; i += BLOCK) { pw_pack[i] = 0; pw_max[i] = 0; pw_min[i] = 0xFFFFFFFFu; }
  if (tid_k < 16) ctr[tid_k] = 0;
  __syncthreads();

  // The records of a workgroup (eight 16-byte units, two records each, per thread) and the words of its
  // header are requested one workgroup ahead, before the previous workgroup's results are written, so
  // that the memory latency runs under that tail and under the clearing of the staging state.
  u32x4 v[8];
  uint32_t h_total;  // lane & 15 -> records written by that wave
  uint2 h_begin, h_end;
  constexpr int kEarly = 6;  // units requested before the matrix products of the sweep of the workgroup before
  auto request_units = [&](uint32_t g, uint32_t t, auto first, auto last) {
    const u32x4* recs = p.records + (size_t)g * (nrec / 2);
#pragma unroll
    for (int u = decltype(first)::value; u < decltype(last)::value; ++u) {
      const uint32_t i = t + u * BLOCK;
      v[u] = __builtin_nontemporal_load(recs + (i < nrec / 2 ? i : nrec / 2 - 1));
    }
  };
  auto request_header = [&](uint32_t g, uint32_t t) {
    const uint32_t* whn = p.wg_hdrs + (size_t)32 * g;
    h_total = whn[8 + (t & 15u)];
    h_begin = *reinterpret_cast<const uint2*>(whn + 2);
    h_end = *reinterpret_cast<const uint2*>(whn + 4);
  };
  request_units(blockIdx.x, tid_k, std::integral_constant<int, 0>{}, std::integral_constant<int, kEarly>{});
  request_header(blockIdx.x, tid_k);

  for (uint32_t wg = blockIdx.x; wg < n_wg; wg += gridDim.x) {
    // A fresh copy of the thread index per workgroup that the optimiser cannot see through: without it
    // the address arithmetic of all 16 rounds is computed once before the loop and held in registers
    // for the whole kernel.
    uint32_t tid = tid_k;
    asm volatile("" : "+v"(tid));
    const uint32_t lane = tid & 63u, hw = (uint32_t)__builtin_amdgcn_readfirstlane((int)(tid >> 6));
    const uint32_t pbase = hw * kWaveSpan;
    const uint32_t qe = pbase + 2u * lane;     // even position of round 0; round j: qe + 128 j
    // its clock word; round j: cwe + 136 j (pbase is a multiple of 1024, lanes 32.. are past one padding)
    const uint32_t cwe = qe + (pbase >> 4) + ((lane >> 5) << 2);
    // the last units of this workgroup's records: they travel while the staging state is cleared
    request_units(wg, tid, std::integral_constant<int, kEarly>{}, std::integral_constant<int, 8>{});
    // ---- workgroup header, clear the staging state -----------------------------------------------
    if (tid <= KP_MAX_WAVES) {  // (entries from W up: no records)
      const uint32_t T = tid < W ? h_total : 0u;
      const uint32_t V = T < cap ? T : cap;
      sVF[tid] = make_uint2(V, flush ? 0u : T - V);
      atomicAdd(&ctr[H_DROPPED], (unsigned long long)(T - V));
      atomicAdd(&ctr[H_SLOTS_VALID], (unsigned long long)V);
    }
    if (tid < 64) {  // clear the temporaries; the last one takes the records the waves hold together
      const uint32_t held = wave_scan_add(tid < W ? (h_total < cap ? h_total : cap) : 0u);
      if (tid >= 64 - T_COUNT) tmp[tid - (64 - T_COUNT)] = tid == 63u ? held : 0u;
    }
    if (tid == 32) {
      const uint64_t tb = (uint64_t)h_begin.x | ((uint64_t)h_begin.y << 32);
      const uint64_t te = (uint64_t)h_end.x | ((uint64_t)h_end.y << 32);
      const uint64_t sp = te - tb;
      // cell of clock t: (t * scale) >> 32, i.e. the span divided into NCELL cells (clamped below).  Any
      // scale near NCELL * 2^32 / (span + 1) orders the cells by time, so a floating-point quotient does:
      // a 64-bit integer division is some 150 instructions that every wave of the workgroup waits for.
      const double scale = (double)NCELL * 4294967296.0 / ((double)(uint32_t)sp + 1.0);
      misc[0] = (sp >> 32) ? 1u : 0u;
      misc[1] = scale >= 4294967295.0 ? 0xFFFFFFFFu : (uint32_t)scale;
      misc[2] = (uint32_t)sp;
    }
    reinterpret_cast<u32x4*>(meta)[tid] = u32x4{0x3F3F3F3Fu, 0x3F3F3F3Fu, 0x3F3F3F3Fu, 0x3F3F3F3Fu};
    {  // a position without a record reads as the largest clock: it never counts as a step back in time
      u32x4* own = reinterpret_cast<u32x4*>(clk + clk_word(tid * kNR));
      const u32x4 ones{0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu};
      own[0] = ones; own[1] = ones; own[2] = ones; own[3] = ones;
    }
    reinterpret_cast<u32x4*>(cells)[2 * tid] = u32x4{0u, 0u, 0u, 0u};
    reinterpret_cast<u32x4*>(cells)[2 * tid + 1] = u32x4{0u, 0u, 0u, 0u};
    if (tid == 0) reinterpret_cast<u32x4*>(cells)[2 * BLOCK] = u32x4{0u, 0u, 0u, 0u};
    __syncthreads();

    uint32_t wg_invalid = 0;
    bool eligible = false;
    uint32_t products = 0;  // limbs of the stretch lengths when the sweep hands its sets to the matrix cores, else 0
    const uint32_t wg_ahead = wg + gridDim.x < n_wg ? wg + gridDim.x : wg;  // (the last one asks for its own again)
    do {  // (left early only when single steps are timed)
    // ---- A: scatter by rank ------------------------------------------------------------------
    // Eight 16-byte units (two records each) per thread cover the workgroup.  Two records that go to an
    // even rank and the rank above it (the usual case: both sit in the slot of their seq) leave with one
    // 8-byte and one 2-byte store.
    // (Slots that hold a record and fail a check are what is left of the header's record count.)
    {
      uint32_t c_field = 0, c_dis = 0;
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const uint32_t f0 = 2u * (tid + u * BLOCK);
        // a unit past the last record slot falls into a wave past the last one, which holds no records
        const uint32_t wv = f0 >> cl2, w = wv < KP_MAX_WAVES ? wv : KP_MAX_WAVES, s0 = f0 & capm;
        const uint2 vf = sVF[w];
        const uint32_t V = vf.x, first = vf.y;
        const uint32_t tag0 = v[u].x, pay0 = v[u].y, tag1 = v[u].z, pay1 = v[u].w;
        // rank: the low 20 bits of tag - first are those of seq - first
        const uint32_t k0 = (tag0 - first) & kSeqMask, k1 = (tag1 - first) & kSeqMask;
        const bool good0 = s0 < V && k0 < V && ((tag0 >> 20) & 0xFu) == w && ((tag0 >> 24) & 0x7Fu) < R;
        const bool good1 = s0 + 1u < V && k1 < V && ((tag1 >> 20) & 0xFu) == w && ((tag1 >> 24) & 0x7Fu) < R;
        c_field += (good0 ? 1u : 0u) + (good1 ? 1u : 0u);
        c_dis += ((good0 && ((tag0 ^ s0) & capm) != 0u) ? 1u : 0u) + ((good1 && ((tag1 ^ (s0 + 1u)) & capm) != 0u) ? 1u : 0u);
        const uint32_t base = f0 - s0;  // first position of the recorded wave
        const uint32_t pos0 = base + k0, pos1 = base + k1;
        // an even rank and the one above it: k1 - k0 == 1 and k0 even
        const bool twin = good0 && good1 && (((k1 - k0) ^ 1u) | (k0 & 1u)) == 0u;
        if (twin) {
          uint32_t* dst = clk + clk_word(pos0);
          dst[0] = pay0; dst[1] = pay1;
          *reinterpret_cast<uint16_t*>(meta + pos0) = (uint16_t)__builtin_amdgcn_perm(tag1, tag0, 0x0C0C0703u);  // END flag and region of both
        } else {
          if (good0) { clk[clk_word(pos0)] = pay0; meta[pos0] = (uint8_t)(tag0 >> 24); }
          if (good1) { clk[clk_word(pos1)] = pay1; meta[pos1] = (uint8_t)(tag1 >> 24); }
        }
      }
      add_tmp(tmp, T_FIELDVALID, c_field);
      add_tmp(tmp, T_DISORDER, c_dis);
    }
    __syncthreads();
    if (stop_after == kStepOrdered) break;

    // ---- a duplicated seq leaves fewer occupied ranks than valid records ---------------------------
    // Records that all sit in the slot of their own seq have distinct seq modulo the ring size, hence
    // distinct ranks: only a workgroup with a record elsewhere needs the count.
    uint32_t n_occupied = tmp[T_FIELDVALID];
    if (tmp[T_DISORDER] != 0u) {
      const u32x4 mv = reinterpret_cast<const u32x4*>(meta)[tid];
      const uint32_t mw[4] = {mv.x, mv.y, mv.z, mv.w};
      uint32_t occ = 0;
#pragma unroll
      for (int i = 0; i < 4; ++i)  // bytes whose region field is not the "no record" code
        occ += __popc((((mw[i] & 0x3F3F3F3Fu) ^ 0x3F3F3F3Fu) + 0x7F7F7F7Fu) & 0x80808080u);
      add_tmp(tmp, T_OCCUPIED, occ);
      __syncthreads();
      n_occupied = tmp[T_OCCUPIED];
      if (n_occupied != tmp[T_FIELDVALID]) {
        // Rare: some seq occurs twice.  The later slot must win, so redo this workgroup's
        // scatter in slot order, one thread per wave.
        __syncthreads();
        reinterpret_cast<u32x4*>(meta)[tid] = u32x4{0x3F3F3F3Fu, 0x3F3F3F3Fu, 0x3F3F3F3Fu, 0x3F3F3F3Fu};
        if (tid == 0) { tmp[T_DISORDER] = 0; tmp[T_OCCUPIED] = 0; }
        __syncthreads();
        if (tid < W) {
          const uint32_t w = tid, V = sVF[w].x, first = sVF[w].y;
          const uint32_t* seg = reinterpret_cast<const uint32_t*>(p.records) + ((size_t)wg * nrec + (size_t)w * cap) * 2;
          for (uint32_t s = 0; s < V; ++s) {
            const uint32_t tag = seg[2 * s];
            const uint32_t seq = tag & kSeqMask, k = (seq - first) & kSeqMask, region = (tag >> 24) & 0x7Fu;
            if (k >= V || ((tag >> 20) & 0xFu) != w || region >= R) continue;
            // the clock word remembers the winning slot for now
            clk[clk_word(w * cap + k)] = s;
            meta[w * cap + k] = (uint8_t)(tag >> 24);
          }
          uint32_t dis = 0, occ2 = 0;
          for (uint32_t k = 0; k < V; ++k) {
            if ((meta[w * cap + k] & kRegion) == kEmpty) continue;
            const uint32_t s = clk[clk_word(w * cap + k)];
            dis += (s != ((seg[2 * s] & kSeqMask) & capm));
            clk[clk_word(w * cap + k)] = seg[2 * s + 1];
            ++occ2;
          }
          atomicAdd(&tmp[T_DISORDER], dis);
          atomicAdd(&tmp[T_OCCUPIED], occ2);
        }
        __syncthreads();
        n_occupied = tmp[T_OCCUPIED];
      }
    }
    // ---- this lane's 16 positions: in round j the even position qe + 128 j and the one above it ---------
    // (The arrays below are only ever assigned outside of branches: a conditional assignment makes the
    // compiler carry each array through the branch as one 16-register value, copied at every merge.)
    uint32_t t[kNR], mq[kNR / 4];  // clocks; metadata bytes, record i in byte i & 3 of word i >> 2
#pragma unroll
    for (int j = 0; j < kNR / 4; ++j) mq[j] = 0u;
#pragma unroll
    for (int j = 0; j < kNR / 2; ++j) {
      const uint2 tt = *reinterpret_cast<const uint2*>(clk + cwe + 136u * j);
      t[2 * j] = tt.x; t[2 * j + 1] = tt.y;
      // positions past the last record slot stay cleared
      mq[j >> 1] |= (uint32_t)*reinterpret_cast<const uint16_t*>(meta + qe + 128u * j) << (16 * (j & 1));
    }
    auto meta_of = [&](int i) -> uint32_t { return (mq[i >> 2] >> (8 * (i & 3))) & 0xFFu; };
    auto set_paired = [&](int i, uint32_t yes) { mq[i >> 2] |= (yes << 6) << (8 * (i & 3)); };  // yes: 0 or 1
    wg_invalid = tmp[T_HELD] - n_occupied;  // slots that hold a record and did not make it into the ordered sequence

    // One pair: duration into the per-(wave, region) sums and the histogram.  The sums exist in up to
    // four copies, one per quarter of the wave: lanes 16 apart tend to hold the same region, and LDS
    // atomics of one instruction that hit one address are processed one after the other.
    const uint32_t copy = (lane >> 4) & (n_copies - 1u);
    auto account_pair = [&](uint32_t w, uint32_t region, uint32_t d_raw) {
      const uint32_t d = d_raw > rec_cost ? d_raw - rec_cost : 0u;
      const uint32_t e = __umul24(__umul24(w, R) + region, n_copies) + copy;
      atomicAdd(&pw_pack[e], (1ull << 46) | (unsigned long long)d);
      atomicMax(&pw_max[e], d);
      atomicMin(&pw_min[e], d);
      atomicAdd(&hist[__umul24(region, kHistStride) + (31 - __clz(d | 1u))], 1u);
    };

    if (wg_invalid == 0u) {
      // ---- B: pairing, durations, per-(wave,region) statistics, monotonicity ------------------------
      // Every rank below a wave's record count holds a record here.  An END is paired iff the nearest
      // earlier record of its (wave, region) is a START; every START that is not claimed this way is an
      // orphan, so only ENDs search.  In traces of kernels whose regions follow one another the START
      // sits one rank below: in the lane's own even position, or, for an END in the even position, in
      // the odd position of the lane below (DPP; the last lane of the previous round stands in for lane
      // 0).  Both positions of a round are tested at once on the two metadata bytes side by side.  An
      // END whose lower neighbour belongs to another region walks back through LDS.
      // A START learns that it is paired from its END: in the same lane directly, one lane up through a
      // DPP shift of the claims, and when the END is in another hardware wave or found the START by
      // walking, through a mark in the START's metadata byte that is read back after the barrier.
      uint32_t n_nonmono = 0;  // wave-uniform count
      uint32_t claims = 0;
      bool marked = false;
      uint32_t cm = kEmpty, ct = 0;
      if (pbase > 0 && pbase < nrec) { cm = meta[pbase - 1]; ct = clk[clk_word(pbase - 1)]; }
      auto count = [](bool b) -> uint32_t { return (uint32_t)__popcll(__builtin_amdgcn_ballot_w64(b)); };
      auto walk_back = [&](uint32_t qq, uint32_t mine, bool& have, uint32_t& sm, uint32_t& sq, uint32_t& sts) {
        const uint32_t k = qq & capm, wofs = qq - k;
        for (uint32_t kk = k - 1; kk-- > 0;) {
          const uint32_t mm = meta[wofs + kk];
          if (((mm ^ mine) & kRegion) == 0u) { have = true; sm = mm; sq = wofs + kk; sts = clk[clk_word(sq)]; break; }
        }
      };
#pragma unroll
      for (int j = 0; j < kNR / 2; ++j) {
        const uint32_t q = qe + 128u * j;  // even position; the odd one is q + 1
        const uint32_t m2 = (mq[j >> 1] >> (16 * (j & 1))) & 0xFFFFu;  // byte 0: even position, byte 1: odd
        const uint32_t t0 = t[2 * j], t1 = t[2 * j + 1];
        uint32_t pm = wave_shr1(m2 >> 8, cm);
        const uint32_t pt = wave_shr1(t1, ct);
        cm = (uint32_t)__builtin_amdgcn_readlane((int)m2, 63) >> 8;
        ct = (uint32_t)__builtin_amdgcn_readlane((int)t1, 63);
        const uint32_t k0 = q & capm;
        const bool lowest = k0 == 0u;  // first rank of a recorded wave: no record below
        pm = lowest ? kEmpty : pm;
        const uint32_t p2 = ((m2 << 8) | pm) & 0xFFFFu;  // the record one rank below each of the two
        const uint32_t x2 = m2 ^ p2;
        // bit 7 of each of the two bytes: that byte of the argument is not zero
        auto nonzero7 = [](uint32_t v) -> uint32_t { return ((v & 0x7F7Fu) + 0x7F7Fu) | v; };
        const uint32_t end2 = m2 & 0x8080u;                                   // is an END (no record: 0)
        const uint32_t differ2 = nonzero7(x2 & 0x3F3Fu) & end2;               // END, other region one rank below
        const uint32_t near2 = ~nonzero7((x2 & 0xBFBFu) ^ 0x8080u) & end2;    // END, START of its region one rank below
        bool p0 = (near2 & 0x80u) != 0u, p1 = (near2 & 0x8000u) != 0u;
        uint32_t st0 = pt, st1 = t0;  // clock of the START
        // (a position without a record holds the largest clock, and so do all above it in its wave)
        n_nonmono += count(!lowest && t0 < pt) + count(t1 < t0);
        // as END, or as the START of the odd position; the mark of an END sits one bit above its flag
        uint32_t flags = (near2 >> 1) | ((near2 >> 9) & kPaired);
        claims |= (p0 ? 1u : 0u) << j;
        if (j == 0 && p0 && lane == 0u && pbase > 0) meta[pbase - 1] = (uint8_t)(pm | kPaired);
        if (__builtin_amdgcn_ballot_w64(differ2 != 0u)) {
          const uint32_t m0 = m2 & 0xFFu, m1 = m2 >> 8;
          const bool deep0 = (differ2 & 0x80u) && k0 > 1, deep1 = (differ2 & 0x8000u) && k0 > 0;
          bool have0 = false, have1 = false;
          uint32_t sm0 = 0, sm1 = 0, sq0 = 0, sq1 = 0;
          if (deep0) walk_back(q, m0, have0, sm0, sq0, st0);
          if (deep1) walk_back(q + 1, m1, have1, sm1, sq1, st1);
          const bool far0 = have0 && !(sm0 & kEnd), far1 = have1 && !(sm1 & kEnd);
          if (far0) meta[sq0] = (uint8_t)(sm0 | kPaired);
          if (far1) meta[sq1] = (uint8_t)(sm1 | kPaired);
          flags |= (far0 ? kPaired : 0u) | (far1 ? kPaired << 8 : 0u);
          marked = marked || far0 || far1;
          p0 = p0 || far0; p1 = p1 || far1;
        }
        mq[j >> 1] |= flags << (16 * (j & 1));
        const uint32_t w = q >> cl2;
        if (p0 || p1) account_pair(w, (p1 ? m2 >> 8 : m2) & kRegion, p1 ? t1 - st1 : t0 - st0);
        const bool both = p0 && p1;
        if (__builtin_amdgcn_ballot_w64(both)) {
          if (both) account_pair(w, m2 & kRegion, t0 - st0);
        }
      }
      // the START claimed by the even position of the lane above (lane 63: of lane 0 in the next round)
      const uint32_t claims0 = (uint32_t)__builtin_amdgcn_readlane((int)claims, 0);
#pragma unroll
      for (int j = 0; j < kNR / 2; ++j) {
        const uint32_t next_round = j + 1 < kNR / 2 ? (claims0 >> (j + 1)) & 1u : 0u;
        const uint32_t got = (uint32_t)__builtin_amdgcn_update_dpp((int)next_round, (int)((claims >> j) & 1u), 0x130, 0xF, 0xF,
                                                                   false);  // wave_shl:1
        set_paired(2 * j + 1, got);
      }
      // ENDs, and ENDs that are paired (the flag sits one bit below): counted on the packed bytes
      uint32_t n_ends = 0, n_pairs = 0;
#pragma unroll
      for (int x = 0; x < kNR / 4; ++x) {
        n_ends += __popc(mq[x] & 0x80808080u);
        n_pairs += __popc(mq[x] & (mq[x] << 1) & 0x80808080u);
      }
      n_pairs = wave_scan_add(n_ends | (n_pairs << 16));  // both at most 1024 per wave
      const bool any_marked = __builtin_amdgcn_ballot_w64(marked) != 0;
      if (lane == 0u) {
        if (any_marked) tmp[T_MARKS] = 1u;
        if (n_nonmono) atomicAdd(&tmp[T_NONMONO], n_nonmono);
      }
      if (lane == 63u) {
        atomicAdd(&tmp[T_PAIRS], n_pairs >> 16);
        atomicAdd(&tmp[T_ENDS], n_pairs & 0xFFFFu);
      }
      if (tid == 0) tmp[T_STARTS] = n_occupied;  // records; orphans = records - ENDs - pairs, ENDs - pairs
    } else {
      // ---- B, workgroup with holes: the definition, one thread per (wave, region) -----------------
      for (uint32_t e = tid; e < W * R; e += BLOCK) {
        const uint32_t w = e / R, r = e - w * R, V = sVF[w].x;
        bool have_prev = false;
        uint32_t prev_m = 0, prev_t = 0, n_pairs = 0, n_starts = 0, n_ends = 0;
        for (uint32_t k = 0; k < V; ++k) {
          const uint32_t mm = meta[w * cap + k];
          if ((mm & kRegion) != r) continue;
          const uint32_t ts = clk[clk_word(w * cap + k)];
          if (mm & kEnd) {
            ++n_ends;
            if (have_prev && !(prev_m & kEnd)) { ++n_pairs; account_pair(w, r, ts - prev_t); }
          } else {
            ++n_starts;
          }
          have_prev = true; prev_m = mm; prev_t = ts;
        }
        if (n_pairs) atomicAdd(&tmp[T_PAIRS], n_pairs);
        if (n_starts + n_ends) atomicAdd(&tmp[T_STARTS], n_starts + n_ends);
        if (n_ends) atomicAdd(&tmp[T_ENDS], n_ends);
      }
      for (uint32_t w = tid; w < W; w += BLOCK) {
        const uint32_t V = sVF[w].x;
        bool have_prev = false;
        uint32_t prev_t = 0, n = 0;
        for (uint32_t k = 0; k < V; ++k) {
          if ((meta[w * cap + k] & kRegion) == kEmpty) continue;
          const uint32_t ts = clk[clk_word(w * cap + k)];
          n += (have_prev && ts < prev_t) ? 1u : 0u;
          have_prev = true; prev_t = ts;
        }
        if (n) atomicAdd(&tmp[T_NONMONO], n);
      }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kNR; ++i) asm volatile("" : "+v"(t[i]));  // (opaque across the barrier, see below)
#pragma unroll
    for (int i = 0; i < kNR / 4; ++i) asm volatile("" : "+v"(mq[i]));
    eligible = !misc[0] && wg_invalid == 0u && tmp[T_NONMONO] == 0u;

    if (eligible && stop_after != kStepPaired) {
      // ---- C: order the paired records of all waves by clock ---------------------------------------
      // marks left by ENDs of other hardware waves (only the last position can have one) and by walks
      set_paired(kNR - 1, ((uint32_t)meta[qe + 128u * (kNR / 2 - 1) + 1u] >> 6) & 1u);
      if (tmp[T_MARKS]) {
#pragma unroll
        for (int j = 0; j < kNR / 2; ++j)
          mq[j >> 1] |= ((uint32_t)*reinterpret_cast<const uint16_t*>(meta + qe + 128u * j) & 0x4040u) << (16 * (j & 1));
      }
      const uint32_t scale = misc[1];
      // Straight-line code from here to the sorted sequence: the LDS operations of a lane's 16 records
      // are issued together and no array is assigned inside a branch.
      uint32_t ca[kNR];  // cell | arrival slot << 16; then: first place of the cell; then: place in the sorted sequence
      uint32_t t_max = 0;
#pragma unroll
      for (int i = 0; i < kNR; ++i) {
        const bool ev = (meta_of(i) & kPaired) != 0u;
        t_max = ev && t[i] > t_max ? t[i] : t_max;
        uint32_t c = __umulhi(t[i], scale);
        c = c < NCELL - 1 ? c : NCELL - 1;
        const uint32_t sh = (c & 1u) << 4;
        // a record that is no event adds nothing, so that all 16 atomics are in flight together
        const uint32_t old = atomicAdd(&cells[c >> 1], ev ? 1u << sh : 0u);
        ca[i] = c | (((old >> sh) & 0xFFFFu) << 16);
      }
      if (__builtin_amdgcn_ballot_w64(t_max > misc[2]) && lane == 0u) tmp[T_WIDE] = 1u;  // a clock past the span
      __syncthreads();
      if (stop_after == kStepCounted) break;
      // (the registers that cross this barrier are made opaque: values derived from them for the next
      // phase would otherwise be computed before it and held in registers across it)
#pragma unroll
      for (int i = 0; i < kNR; ++i) asm volatile("" : "+v"(t[i]), "+v"(ca[i]));
#pragma unroll
      for (int i = 0; i < kNR / 4; ++i) asm volatile("" : "+v"(mq[i]));
      {  // exclusive prefix sum over the cell counters, 16 cells (8 words) per thread
        u32x4 a = reinterpret_cast<u32x4*>(cells)[2 * tid], b = reinterpret_cast<u32x4*>(cells)[2 * tid + 1];
        uint32_t wv[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
        uint32_t run = 0, fullest = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const uint32_t lo = wv[i] & 0xFFFFu, hi = wv[i] >> 16;
          fullest = lo > fullest ? lo : fullest;
          fullest = hi > fullest ? hi : fullest;
          wv[i] = run | ((run + lo) << 16);
          run += lo + hi;
        }
        const uint32_t incl = wave_scan_add(run);
        if (lane == 63) wtot[hw] = incl;
        {  // fullest cell of the workgroup
          uint32_t f = fullest, o;
          o = scan_src<0>(f); f = o > f ? o : f; o = scan_src<1>(f); f = o > f ? o : f;
          o = scan_src<2>(f); f = o > f ? o : f; o = scan_src<3>(f); f = o > f ? o : f;
          o = scan_src<4>(f); f = o > f ? o : f; o = scan_src<5>(f); f = o > f ? o : f;
          if (lane == 63) atomicMax(&tmp[T_MAXCELL], f);
        }
        __syncthreads();
        uint32_t base = incl - run;
        {  // + the totals of the waves below: lane h of the first row takes wave h's
          uint32_t below = (lane & 15u) < hw ? wtot[lane & 15u] : 0u;
          below += scan_src<0>(below); below += scan_src<1>(below); below += scan_src<2>(below); below += scan_src<3>(below);
          base += (uint32_t)__builtin_amdgcn_readlane((int)below, 15);
        }
        const uint32_t both = base * 0x00010001u;
        a = u32x4{wv[0] + both, wv[1] + both, wv[2] + both, wv[3] + both};
        b = u32x4{wv[4] + both, wv[5] + both, wv[6] + both, wv[7] + both};
        reinterpret_cast<u32x4*>(cells)[2 * tid] = a;
        reinterpret_cast<u32x4*>(cells)[2 * tid + 1] = b;
        if (tid == BLOCK - 1) { cells[NCELL / 2] = base + run; tmp[T_EVENTS] = base + run; }
      }
      __syncthreads();
      if (stop_after == kStepCellSums) break;
      // (the registers that cross this barrier are made opaque: values derived from them for the next
      // phase would otherwise be computed before it and held in registers across it)
#pragma unroll
      for (int i = 0; i < kNR; ++i) asm volatile("" : "+v"(t[i]), "+v"(ca[i]));
#pragma unroll
      for (int i = 0; i < kNR / 4; ++i) asm volatile("" : "+v"(mq[i]));
      auto cell_start = [&](uint32_t c) -> uint32_t { return (cells[c >> 1] >> ((c & 1u) << 4)) & 0xFFFFu; };
      // sorted sequence entry besides the clock: region << 1 | END
      auto info_of = [&](int i) -> uint32_t { return ((meta_of(i) & 0x1Fu) << 1) | (meta_of(i) >> 7); };
      // When clock and region fit one word and no cell holds more than kMaxCellWindow records, the records stay
      // in arrival order inside their cell here and every lane of the sweep sorts a window of the sequence
      // in registers; otherwise the records are ranked inside their cell first.
      const bool window_sort = R <= 16u && misc[2] < (1u << 26) && !tmp[T_WIDE] && tmp[T_MAXCELL] <= kMaxCellWindow;
      if (window_sort) {
#pragma unroll
        for (int i = 0; i < kNR; ++i) {
          const bool ev = (meta_of(i) & kPaired) != 0u;
          const uint32_t g = cell_start(ca[i] & 0xFFFFu) + (ca[i] >> 16);
          // the word the sweep sorts: clock << 6 | region << 1 | END (no branch: the others all write one unused word)
          clk[ev ? clk_word(g) : kSpareWord] = (t[i] << 6) | info_of(i);
        }
        __syncthreads();
        if (stop_after >= kStepPlaced && stop_after <= kStepSorted) break;
      } else {
      // provisional place: cell start + arrival slot (plain index here, the padded layout comes with the
      // final places)
      uint32_t nm[kNR];  // records in the cell (0: this record is no event) | arrival slot << 16
#pragma unroll
      for (int i = 0; i < kNR; ++i) {
        const uint32_t ev = 0u - ((meta_of(i) >> 6) & 1u);  // all ones for an event
        const uint32_t c = ca[i] & 0xFFFFu, mine = ca[i] >> 16;
        const uint32_t s0 = cell_start(c), s1 = cell_start(c + 1);
        clk[ev ? s0 + mine : kSpareWord] = t[i];  // no branch: the others all write one unused word
        ca[i] = s0;
        nm[i] = ((s1 - s0) | (mine << 16)) & ev;
      }
      __syncthreads();
      if (stop_after == kStepPlaced) break;
      // rank among the records of the same cell: by clock, then by arrival slot
#pragma unroll
      for (int i = 0; i < kNR; ++i) {
        const uint32_t n = nm[i] & 0xFFFFu, s0 = ca[i], mine = nm[i] >> 16, t0 = t[i];
        uint32_t before = 0;
        for (uint32_t it = 0; __builtin_amdgcn_ballot_w64(it < n); ++it) {
          if (it < n) {
            const uint32_t tm = clk[s0 + it];
            before += (uint32_t)(tm < t0) | ((uint32_t)(tm == t0) & (uint32_t)(it < mine));  // the record's own entry gives 0
          }
        }
        ca[i] = s0 + before;
      }
      __syncthreads();
      if (stop_after == kStepRanked) break;
#pragma unroll
      for (int i = 0; i < kNR; ++i) {
        const bool ev = (meta_of(i) & kPaired) != 0u;
        clk[ev ? clk_word(ca[i]) : kSpareWord] = t[i];
        meta[ev ? ca[i] : NPOS] = (uint8_t)info_of(i);
      }
      __syncthreads();
      if (stop_after == kStepSorted) break;
      }

      // ---- D: region-pair overlap, 16 consecutive records of the sorted sequence per lane ----------
      {
        const uint32_t n_events = tmp[T_EVENTS];
        const uint32_t g0 = tid * kNR;
        const uint32_t region_bits = 0xFFFFFFFFu >> (32u - R);  // places past the end carry a bit above the regions
        uint32_t pl[PLANES], inc[PLANES];
#pragma unroll
        for (int k = 0; k < PLANES; ++k) pl[k] = 0u;
        // From each lane's net change (pl) to the state before its stretch (pl again): an inclusive scan
        // over the lanes, the waves' totals through LDS and one barrier, a scan over those.  `first_clock`
        // is the clock of the lane's first record, left for the last lane of the wave below.
        auto state_before = [&](uint32_t first_clock) {
#pragma unroll
          for (int k = 0; k < PLANES; ++k) inc[k] = pl[k];
          {
            uint32_t o[PLANES];
#pragma unroll
            for (int k = 0; k < PLANES; ++k) o[k] = scan_src<0>(inc[k]);
            planes_add<PLANES>(inc, o);
#pragma unroll
            for (int k = 0; k < PLANES; ++k) o[k] = scan_src<1>(inc[k]);
            planes_add<PLANES>(inc, o);
#pragma unroll
            for (int k = 0; k < PLANES; ++k) o[k] = scan_src<2>(inc[k]);
            planes_add<PLANES>(inc, o);
#pragma unroll
            for (int k = 0; k < PLANES; ++k) o[k] = scan_src<3>(inc[k]);
            planes_add<PLANES>(inc, o);
#pragma unroll
            for (int k = 0; k < PLANES; ++k) o[k] = scan_src<4>(inc[k]);
            planes_add<PLANES>(inc, o);
#pragma unroll
            for (int k = 0; k < PLANES; ++k) o[k] = scan_src<5>(inc[k]);
            planes_add<PLANES>(inc, o);
          }
          if (lane == 63) {
#pragma unroll
            for (int k = 0; k < PLANES; ++k) ptot[hw * 8 + k] = inc[k];
          }
          if (lane == 0) wtot[hw] = first_clock;
          __syncthreads();
#pragma unroll
          for (int k = 0; k < PLANES; ++k) pl[k] = wave_shr1(inc[k], 0u);
          if (hw > 0) {  // lane h of a row takes wave h's net change; a scan over the row, then the entry of wave hw - 1
            uint32_t wsum[PLANES], o[PLANES];
#pragma unroll
            for (int k = 0; k < PLANES; ++k) wsum[k] = ptot[(lane & 15u) * 8 + k];
#pragma unroll
            for (int k = 0; k < PLANES; ++k) o[k] = scan_src<0>(wsum[k]);
            planes_add<PLANES>(wsum, o);
#pragma unroll
            for (int k = 0; k < PLANES; ++k) o[k] = scan_src<1>(wsum[k]);
            planes_add<PLANES>(wsum, o);
#pragma unroll
            for (int k = 0; k < PLANES; ++k) o[k] = scan_src<2>(wsum[k]);
            planes_add<PLANES>(wsum, o);
#pragma unroll
            for (int k = 0; k < PLANES; ++k) o[k] = scan_src<3>(wsum[k]);
            planes_add<PLANES>(wsum, o);
#pragma unroll
            for (int k = 0; k < PLANES; ++k) o[k] = (uint32_t)__builtin_amdgcn_readlane((int)wsum[k], (int)(hw - 1u));
            planes_add<PLANES>(pl, o);
          }
        };
        // One record of the sequence for the general way of adding up: a region that switches on or off
        // adds -t / +t to its sums with every region open at that instant (LDS atomics).
        auto switch_record = [&](uint32_t x, uint32_t dm, uint32_t tt) {
          uint32_t act_before = pl[0];
#pragma unroll
          for (int k = 1; k < PLANES; ++k) act_before |= pl[k];
          planes_step<PLANES>(pl, x, dm);
          uint32_t act_after = pl[0];
#pragma unroll
          for (int k = 1; k < PLANES; ++k) act_after |= pl[k];
          const uint32_t act = dm ? act_after : act_before;  // active regions other than this one
          if (x & ~act) {  // the region was off before this START / is off after this END
            // modulo 2^32: the totals of one workgroup lie below its span, which is below 2^32
            const uint32_t a = __ffs(x) - 1;
            uint32_t* row = oacc32 + a * (R | 1u);
            const uint32_t val = dm ? tt : 0u - tt;
            atomicAdd(&row[a], val);
            uint32_t set = act & region_bits;
            while (set) {
              const uint32_t bb = __ffs(set) - 1;
              set &= set - 1;
              atomicAdd(&row[bb], val);
            }
          }
        };
        if (window_sort) {
          // ---- the order is finished in registers; one word per record from here on ------------------
          uint32_t key[kNR];
          const uint32_t fake = (misc[2] << 6) | 0x3Fu;
          if (tmp[T_MAXCELL] <= 9u) sorted_own<NPOS>(clk, tid, n_events, fake, key);
          else sorted_pairs<NPOS>(clk, tid, n_events, fake, key);
#pragma unroll
          for (int i = 0; i < kNR; ++i) planes_step<PLANES>(pl, key_region_bit(key[i]), key_end_mask(key[i]));
          state_before(key_clock(key[0]));
#pragma unroll
          for (int i = 0; i < kNR; ++i) asm volatile("" : "+v"(key[i]));  // (opaque across the barrier, as above)
          // ---- the sorted sequence as segments: the set of active regions after record k and the ticks
          // until record k + 1.  O[a][b] = sum over segments of ticks * active(a) * active(b) is a 16 x K by
          // K x 16 matrix product: the matrix cores take it 64 segments at a time (i8 operands: the ticks in
          // 7-bit limbs, one product per limb), and no accumulator atomics are left in the sweep.
          // clock of the record after the lane's 16: the first one of the lane above
          const uint32_t t_above = hw + 1 < BLOCK / 64 ? wtot[hw + 1 < BLOCK / 64 ? hw + 1 : hw] : misc[2];
          const uint32_t t_next = (uint32_t)__builtin_amdgcn_update_dpp((int)t_above, (int)key_clock(key[0]), 0x130, 0xF, 0xF, false);  // wave_shl:1
          // (places past the end of the sequence carry the workgroup's last clock: stretches of length 0
          // behind a last one in which no region is open)
          uint32_t len[kNR];
          uint32_t any_len = 0;
#pragma unroll
          for (int i = 0; i < kNR; ++i) {
            len[i] = (i + 1 < kNR ? key_clock(key[i + 1]) : t_next) - key_clock(key[i]);
            any_len |= len[i];
          }
          {  // OR over the wave
            uint32_t f = any_len;
            f |= scan_src<0>(f); f |= scan_src<1>(f); f |= scan_src<2>(f);
            f |= scan_src<3>(f); f |= scan_src<4>(f); f |= scan_src<5>(f);
            any_len = (uint32_t)__builtin_amdgcn_readlane((int)f, 63);
          }
          if (any_len < (1u << 21)) {  // else: a gap of more than three limbs, the general way takes this wave
            const uint32_t n_limbs = any_len < (1u << 7) ? 1u : (any_len < (1u << 14) ? 2u : 3u);
            // The lane's own 16 places of the sequence are free now (every neighbour read them before the last
            // barrier): they take the active sets and two limbs, the 16 metadata bytes the third limb.
            u32x4* own = reinterpret_cast<u32x4*>(clk + clk_word(g0));
            {
              uint32_t l0[4] = {0u, 0u, 0u, 0u};
#pragma unroll
              for (int i = 0; i < kNR; ++i) l0[i >> 2] |= (len[i] & 0x7Fu) << (8 * (i & 3));
              own[2] = u32x4{l0[0], l0[1], l0[2], l0[3]};
            }
            if (n_limbs > 1u) {
              uint32_t l1[4] = {0u, 0u, 0u, 0u};
#pragma unroll
              for (int i = 0; i < kNR; ++i) l1[i >> 2] |= ((len[i] >> 7) & 0x7Fu) << (8 * (i & 3));
              own[3] = u32x4{l1[0], l1[1], l1[2], l1[3]};
            }
            if (n_limbs > 2u) {
              uint32_t l2[4] = {0u, 0u, 0u, 0u};
#pragma unroll
              for (int i = 0; i < kNR; ++i) l2[i >> 2] |= ((len[i] >> 14) & 0x7Fu) << (8 * (i & 3));
              reinterpret_cast<u32x4*>(meta)[tid] = u32x4{l2[0], l2[1], l2[2], l2[3]};
            }
            uint32_t mk[kNR / 2];  // active sets after records 2x and 2x + 1, 16 bits each
            uint32_t act_even = 0u;
#pragma unroll
            for (int i = 0; i < kNR; ++i) {
              planes_step<PLANES>(pl, key_region_bit(key[i]), key_end_mask(key[i]));
              uint32_t act = pl[0];
#pragma unroll
              for (int k = 1; k < PLANES; ++k) act |= pl[k];
              if (i & 1) mk[i >> 1] = __builtin_amdgcn_perm(act, act_even, 0x05040100u);  // the low halves of the two
              else act_even = act;
            }
            own[0] = u32x4{mk[0], mk[1], mk[2], mk[3]};
            own[1] = u32x4{mk[4], mk[5], mk[6], mk[7]};
            products = (tid & ~63u) * kNR < n_events ? n_limbs : 0u;  // this wave holds records
          } else {
#pragma unroll
            for (int i = 0; i < kNR; ++i)
              switch_record(key_region_bit(key[i]) & region_bits, key_end_mask(key[i]), key_clock(key[i]));
          }
        } else {
          // ---- the general way: the sequence is already in order, clocks up to 32 bits, up to 32 regions --
          uint32_t st[kNR], sx[kNR];  // clock, region bit (0: no record)
          uint32_t ends = 0;           // bit i: record i is an END
          const u32x4 mv = reinterpret_cast<const u32x4*>(meta)[tid];
          const uint32_t mw[4] = {mv.x, mv.y, mv.z, mv.w};
          const u32x4* tv = reinterpret_cast<const u32x4*>(clk + clk_word(g0));
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const u32x4 v = tv[i];
            st[4 * i] = v.x; st[4 * i + 1] = v.y; st[4 * i + 2] = v.z; st[4 * i + 3] = v.w;
          }
#pragma unroll
          for (int i = 0; i < kNR; ++i) {
            const uint32_t info = (mw[i >> 2] >> (8 * (i & 3))) & 0xFFu;
            sx[i] = g0 + i < n_events ? 1u << (info >> 1) : 0u;
            ends |= (info & 1u) << i;
          }
          auto end_mask = [&](int i) -> uint32_t { return (uint32_t)((int32_t)(ends << (31 - i)) >> 31); };  // all ones for an END
#pragma unroll
          for (int i = 0; i < kNR; ++i) planes_step<PLANES>(pl, sx[i], end_mask(i));
          state_before(st[0]);
#pragma unroll
          for (int i = 0; i < kNR; ++i) switch_record(sx[i], end_mask(i), st[i]);
        }
      }
    }
    } while (0);
    // The first records of the next workgroup travel while the matrix cores work.
    request_units(wg_ahead, tid, std::integral_constant<int, 0>{}, std::integral_constant<int, kEarly>{});
    if (products) {  // wave-uniform
      const uint32_t n_limbs = products;
      __builtin_amdgcn_wave_barrier();
      typedef int i32x4 __attribute__((ext_vector_type(4)));
      i32x4 acc[3];
#pragma unroll
      for (int l = 0; l < 3; ++l) acc[l] = i32x4{0, 0, 0, 0};
      const uint32_t j = lane & 15u;  // operand row / column: region j
      const uint32_t up = 15u - j;      // shift that takes bit j of a 16-bit set to its top
      for (uint32_t n = 0; n < 16; ++n) {  // 64 segments: those of lanes 4n .. 4n + 3
        const uint32_t src = (tid & ~63u) + 4u * n + (lane >> 4);
        const u32x4* from = reinterpret_cast<const u32x4*>(clk + clk_word(src * kNR));
        const u32x4 s0 = from[0], s1 = from[1];
        const uint32_t w8[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
        // One byte per segment, all ones if region j is open in it: the byte permute's selectors 8..11
        // replicate the top bits of the four halves of its two operands.  As an i8 operand such a byte
        // is -1, so the products below come out negated.
        i32x4 ones;
#pragma unroll
        for (int y = 0; y < 4; ++y)
          ones[y] = (int)__builtin_amdgcn_perm(w8[2 * y + 1] << up, w8[2 * y] << up, 0x0B0A0908u);
        const i32x4 bits = ones;
        const u32x4 l0 = from[2];
        acc[0] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ones & i32x4{(int)l0.x, (int)l0.y, (int)l0.z, (int)l0.w}, bits,
                                                       acc[0], 0, 0, 0);
        if (n_limbs > 1u) {
          const u32x4 l1 = from[3];
          acc[1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ones & i32x4{(int)l1.x, (int)l1.y, (int)l1.z, (int)l1.w}, bits,
                                                         acc[1], 0, 0, 0);
        }
        if (n_limbs > 2u) {
          const u32x4 l2 = reinterpret_cast<const u32x4*>(meta)[src];
          acc[2] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ones & i32x4{(int)l2.x, (int)l2.y, (int)l2.z, (int)l2.w}, bits,
                                                         acc[2], 0, 0, 0);
        }
      }
      // element v of a lane: row 4 * (lane / 16) + v, column lane % 16.  The product is symmetric and the
      // fold below adds the two halves of a pair: the upper triangle takes the whole sum.
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const uint32_t a = 4u * (lane >> 4) + v, b = j;
        const uint32_t total = 0u - ((uint32_t)acc[0][v] + ((uint32_t)acc[1][v] << 7) + ((uint32_t)acc[2][v] << 14));
        if (a <= b && b < R && total) atomicAdd(&oacc32[a * (R | 1u) + b], total);
      }
    }
    __syncthreads();
    request_header(wg_ahead, tid);
    if (stop_after) continue;

    // ---- E: per-(workgroup, wave, region) output, fold into running totals ------------------------
    for (uint32_t e = tid; e < W * R; e += BLOCK) {
      unsigned long long pk = 0;
      uint32_t mx = 0, mn = 0xFFFFFFFFu;
      for (uint32_t c = 0; c < n_copies; ++c) {
        const uint32_t ec = e * n_copies + c;
        pk += pw_pack[ec];
        mx = pw_max[ec] > mx ? pw_max[ec] : mx;
        mn = pw_min[ec] < mn ? pw_min[ec] : mn;
        pw_pack[ec] = 0; pw_max[ec] = 0; pw_min[ec] = 0xFFFFFFFFu;
      }
      const uint32_t n = (uint32_t)(pk >> 46);
      const unsigned long long s = pk & ((1ull << 46) - 1);
      uint64_t* dst = p.out + SL.per + ((size_t)wg * W * R + e) * 2;
      dst[0] = s;
      dst[1] = (uint64_t)n | ((uint64_t)mx << 32);
      if (n) {
        const uint32_t r = e % R;
        atomicAdd(&reg_sum[r], s);
        atomicMax(&reg_max[r], mx);
        atomicMin(&reg_min[r], mn);
      }
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
      ctr[H_ORPHAN_START] += tmp[T_STARTS] - tmp[T_ENDS] - tmp[T_PAIRS];  // T_STARTS counts the records
      ctr[H_ORPHAN_END] += tmp[T_ENDS] - tmp[T_PAIRS];
      ctr[H_SPAN_OVF] += misc[0];
      ctr[H_OVERLAP_WGS] += eligible ? 1u : 0u;
    }
    // No barrier here: the arrays this tail reads and resets are next written in B, two barriers on, and
    // what the head of the next workgroup writes first (temporaries, header words) is touched here only by
    // thread 0, whose own wave writes them there.
  }
  __syncthreads();

  // ---- flush this decoder workgroup's totals --------------------------------------------------
  unsigned long long* out = reinterpret_cast<unsigned long long*>(p.out);
  for (uint32_t i = tid_k; i < R * 64; i += BLOCK) {
    const uint32_t h = hist[(i >> 6) * kHistStride + (i & 63u)];
    if (h) atomicAdd(&out[SL.hist + i], (unsigned long long)h);
  }
  for (uint32_t i = tid_k; i < R * R; i += BLOCK)
    if (oacc[i]) atomicAdd(&out[SL.F + i], oacc[i]);  // staged in the F area until finalize
  for (uint32_t r = tid_k; r < R; r += BLOCK) {
    if (reg_min[r] != 0xFFFFFFFFu || reg_max[r] || reg_sum[r]) {
      atomicAdd(&out[SL.sum + r], reg_sum[r]);
      atomicMax(&out[SL.max + r], (unsigned long long)reg_max[r]);
      atomicMin(&out[SL.min + r], (unsigned long long)reg_min[r]);
    }
  }
  if (tid_k < H_STATUS && ctr[tid_k]) atomicAdd(&out[tid_k], ctr[tid_k]);
}

// Launch shape of one kernel instantiation for one LDS size, queried once per device.
struct LaunchCache { int dev = -1; uint32_t max_grid = 0; };

template <int BLOCK, int PLANES>
kp_status launch_main(const DecodeParams& p, hipStream_t s) {
  auto kern = kp_reduce_main<BLOCK, PLANES>;
  static thread_local LaunchCache cache;
  int dev = 0;
  KP_HIP_TRY(hipGetDevice(&dev));
  if (cache.dev != dev) {
    int per_cu = 0, cus = 0;
    KP_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, BLOCK, 0));
    if (per_cu < 1) return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "decoder kernel does not fit one CU (LDS %u B)", Lds<BLOCK>::total);
    KP_HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    cache.dev = dev; cache.max_grid = (uint32_t)per_cu * (uint32_t)cus;
  }
  uint32_t grid = cache.max_grid;
  if (grid > p.n_wg) grid = p.n_wg;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(BLOCK), 0, s, p);
  KP_HIP_TRY(hipGetLastError());
  return KP_OK;
}

template <int BLOCK>
kp_status launch_planes(const DecodeParams& p, hipStream_t s) {
  // counters of open waves per region run up to the number of waves
  return p.W < 16 ? launch_main<BLOCK, 4>(p, s) : launch_main<BLOCK, 5>(p, s);
}

kp_status reduce_impl(const void* raw, size_t n, const kp_trace_hdr& h, void* out_stats, uint32_t stop_after,
                      hipStream_t s, hipEvent_t main_begin = nullptr, hipEvent_t main_end = nullptr) {
  if (h.magic != KP_TRACE_MAGIC || h.version != KP_TRACE_VERSION)
    return kp::fail(KP_ERR_BAD_TRACE, "trace header: bad magic/version (%08x, %u)", h.magic, h.version);
  if (h.waves_per_wg < 1 || h.waves_per_wg > KP_MAX_WAVES || h.n_regions < 1 || !kp::is_pow2(h.cap_wave))
    return kp::fail(KP_ERR_BAD_TRACE, "trace header: waves=%u regions=%u cap_wave=%u", h.waves_per_wg, h.n_regions, h.cap_wave);
  if ((size_t)h.n_wg * h.waves_per_wg * h.cap_wave != n)
    return kp::fail(KP_ERR_BAD_TRACE, "trace header describes %zu record slots, caller passed %zu",
                    (size_t)h.n_wg * h.waves_per_wg * h.cap_wave, n);
  if ((h.flags & ~(KP_FLAG_FLUSH | KP_FLAG_REALTIME | KP_FLAG_HW_IDS)) != 0) return kp::fail(KP_ERR_BAD_TRACE, "trace header: unknown flags %x", h.flags);
  if (h.n_regions > KP_MAX_TAG_REGIONS)
    return kp::fail(KP_ERR_BAD_TRACE, "trace header: n_regions=%u, the tag holds %d", h.n_regions, KP_MAX_TAG_REGIONS);
  if (h.cap_wave < 2) return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "cap_wave must be at least 2");
  if (h.cap_wave > (1u << 20)) return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "cap_wave=%u exceeds the range of seq", h.cap_wave);
  const uint32_t nrec = h.waves_per_wg * h.cap_wave;
  // geometries the LDS-resident kernel is not built for go to the multi-pass kernel
  const bool wide = h.n_regions > KP_MAX_REGIONS || nrec > kMaxRecPerWg;
  if (wide) {
    const kp_status st = wide_supported(h);
    if (st != KP_OK) return st;
  }
  if (wide && stop_after)
    return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "single steps exist for the LDS-resident decoder only (n_regions <= %d, %u records per workgroup)",
                    KP_MAX_REGIONS, kMaxRecPerWg);
  if (((uintptr_t)raw & 15u) || ((uintptr_t)out_stats & 15u))
    return kp::fail(KP_ERR_INVALID_ARG, "raw and out_stats must be 16-byte aligned");

  const uint32_t W = h.waves_per_wg, R = h.n_regions, cap = h.cap_wave;
  const int block = nrec > 4096 ? 1024 : (nrec > 1024 ? 256 : 64);  // 16 positions per lane
  uint32_t ncopy = 4;  // as many copies of the per-(wave, region) sums as their LDS array has room for
  while (ncopy > 1 && ncopy * W * R > kMaxPerWave) ncopy >>= 1;

  uint64_t* out = static_cast<uint64_t*>(out_stats);
  const uint8_t* base = static_cast<const uint8_t*>(raw);
  const StatsLayout SL = stats_layout(h.n_wg, W, R);
  int init_blocks = (int)((SL.per + 255) / 256);
  if (init_blocks > 64) init_blocks = 64;
  hipLaunchKernelGGL(kp_reduce_init, dim3(init_blocks), dim3(256), 0, s,
                     reinterpret_cast<const uint32_t*>(base), out, h.n_wg, W, R, cap, h.flags);
  KP_HIP_TRY(hipGetLastError());

  if (main_begin) KP_HIP_TRY(hipEventRecord(main_begin, s));
  if (h.n_wg > 0 && wide) {
    const kp_status st = launch_wide(reinterpret_cast<const uint32_t*>(base + sizeof(kp_trace_hdr)),
                                     base + sizeof(kp_trace_hdr) + sizeof(kp_wg_hdr) * (size_t)h.n_wg, out, h, s);
    if (st != KP_OK) return st;
  } else if (h.n_wg > 0) {
    DecodeParams p;
    p.wg_hdrs = reinterpret_cast<const uint32_t*>(base + sizeof(kp_trace_hdr));
    p.records = reinterpret_cast<const u32x4*>(base + sizeof(kp_trace_hdr) + sizeof(kp_wg_hdr) * (size_t)h.n_wg);
    p.out = out;
    p.n_wg = h.n_wg; p.W = W; p.R = R; p.cap = cap;
    p.cap_log2 = 0; while ((1u << p.cap_log2) < cap) ++p.cap_log2;
    p.rec_cost = h.rec_cost; p.flush = h.flags & KP_FLAG_FLUSH;
    p.nrec = nrec; p.ncopy = ncopy; p.stop_after = stop_after;
    const kp_status st = block == 1024 ? launch_planes<1024>(p, s)
                       : block == 256  ? launch_planes<256>(p, s)
                                       : launch_planes<64>(p, s);
    if (st != KP_OK) return st;
  }
  if (main_end) KP_HIP_TRY(hipEventRecord(main_end, s));
  hipLaunchKernelGGL(kp_reduce_finalize, dim3(1), dim3(256), 0, s, out, h.n_wg, W, R);
  KP_HIP_TRY(hipGetLastError());
  return KP_OK;
}

}  // namespace

extern "C" kp_status kp_trace_reduce_hdr(const void* raw, size_t n, const kp_trace_hdr* hdr_host,
                                         void* out_stats, void* stream) {
  kp::clear_error();
  if (!raw || !hdr_host || !out_stats) return kp::fail(KP_ERR_INVALID_ARG, "NULL argument");
  return reduce_impl(raw, n, *hdr_host, out_stats, 0u, static_cast<hipStream_t>(stream));
}

extern "C" kp_status kp_trace_reduce_hdr_events(const void* raw, size_t n, const kp_trace_hdr* hdr_host,
                                                void* out_stats, void* stream, void* main_begin, void* main_end) {
  kp::clear_error();
  if (!raw || !hdr_host || !out_stats) return kp::fail(KP_ERR_INVALID_ARG, "NULL argument");
  return reduce_impl(raw, n, *hdr_host, out_stats, 0u, static_cast<hipStream_t>(stream),
                     static_cast<hipEvent_t>(main_begin), static_cast<hipEvent_t>(main_end));
}

extern "C" kp_status kp_trace_reduce_steps(const void* raw, size_t n, const kp_trace_hdr* hdr_host,
                                           void* out_stats, int last_step, void* stream) {
  kp::clear_error();
  if (!raw || !hdr_host || !out_stats) return kp::fail(KP_ERR_INVALID_ARG, "NULL argument");
  if (last_step < kStepOrdered || last_step > kStepSwept)
    return kp::fail(KP_ERR_INVALID_ARG, "last_step must be %d..%d", kStepOrdered, kStepSwept);
  return reduce_impl(raw, n, *hdr_host, out_stats, (uint32_t)last_step, static_cast<hipStream_t>(stream));
}

extern "C" kp_status kp_trace_reduce(const void* raw, size_t n, void* out_stats, void* stream) {
  kp::clear_error();
  if (!raw || !out_stats) return kp::fail(KP_ERR_INVALID_ARG, "NULL argument");
  kp_trace_hdr h;
  hipStream_t s = static_cast<hipStream_t>(stream);
  KP_HIP_TRY(hipMemcpyAsync(&h, raw, sizeof h, hipMemcpyDeviceToHost, s));
  KP_HIP_TRY(hipStreamSynchronize(s));
  return reduce_impl(raw, n, h, out_stats, 0u, s);
}

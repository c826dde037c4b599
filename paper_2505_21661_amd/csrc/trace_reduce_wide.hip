// Statistics decoder for wide geometries: more than 32 regions (the tag holds 128) or more records
// per workgroup than the LDS-resident decoder stages at once.
//
// Same replay as there (Sec. 4.2: per-wave rings whose tail survives; Sec. 4.3: records are stored
// unpaired and aligned at replay, the constant record cost is subtracted), same statistics block, in
// several passes over a recorded workgroup's records, which stay in HBM:
//   0  every slot is checked once (fields, slot against seq).  Only a workgroup with a record outside
//      the slot of its seq needs more: those records go on a list, and which slot wins each rank is
//      then found a range of ranks at a time from the slots the ranks belong in and the list (the
//      later slot wins: atomic max into a rank -> slot table); a workgroup with more such records
//      than the list holds scans all its slots for every range instead;
//   1  pairing, a range of ranks of every wave at a time: the records of the range are put into LDS in
//      rank order and one thread per (wave, region) walks them, which is the definition of the pairing
//      (an END is paired iff the nearest earlier record of its wave and region is a START).  The
//      thread keeps the region's last record and its sums in registers from range to range; a paired
//      START and END each set their bit in a bitmap of the workgroup's ranks;
//   2  overlap, a window of time at a time: every wave offers its next range of ranks, the window
//      ends at the earliest last clock among the waves that have more to offer, the marked records
//      inside the window are sorted by clock (bitonic, in LDS) and swept.  Each hardware wave sweeps a
//      slab of the sorted events with one lane per region (two regions per lane): a first pass gives
//      the slab's net change of the number of waves that have each region open, a prefix over the
//      slabs the state at the slab's start.  The time two regions are both open is the sum over the
//      ends of their common stretches minus the sum over the beginnings; a common stretch of a and b
//      begins when one of them opens while the other is open and ends when one closes while the other
//      is open, so every event that opens or closes a region adds its clock, signed, to the sums of
//      that region with every open region (modulo 2^64: the total is exact).
// Nothing but the inputs and the statistics block is touched in HBM.
#include "kp_reduce.h"
#include "kp_stage.h"

namespace {

using namespace kp_reduce;

constexpr int kBlock = 1024;
constexpr uint32_t kWavesHw = kBlock / 64;
constexpr uint32_t kK = 2048;               // records in LDS at a time: 2 per thread
constexpr uint32_t kList = 2048;            // records outside the slot of their seq that a workgroup can list
constexpr uint32_t kSlab = kK / kWavesHw;   // sorted events per hardware wave
constexpr uint32_t kSeqMask = 0xFFFFFu;
constexpr uint32_t kHistStride = 65;        // histogram rows 65 words apart: equal bins of different regions, different banks
constexpr uint32_t kRegStride = 128;        // per-slab tables: one entry per region the tag can name
constexpr uint64_t kNoKey = ~0ull;
constexpr uint32_t kMaxLds = 160 * 1024;

// per-workgroup temporaries (u32 words in LDS)
enum { T_FIELDVALID = 0, T_DISORDER, T_OCCUPIED, T_WINNER_DISORDER, T_NONMONO, T_PAIRS, T_ORPHAN_START, T_ORPHAN_END, T_WINDOW_END,
       T_ADVANCED, T_LISTED, T_COUNT };

struct WideLds {  // byte offsets
  uint32_t keys, table, list, bitmap, otri, hist, reg_sum, reg_max, reg_min, n_open, slab_delta, ctr, tmp, vf, pos, adv, total;
};
inline uint32_t up16(uint32_t x) { return (x + 15u) & ~15u; }
WideLds wide_lds(uint32_t R, uint32_t nrec) {
  WideLds l;
  l.keys = 0;
  l.table = l.keys + kK * 8;
  l.list = l.table + kK * 4;
  l.bitmap = l.list + kList * 4;
  l.otri = up16(l.bitmap + ((nrec + 31) / 32) * 4);
  l.hist = l.otri + R * (R + 1) / 2 * 8;
  l.reg_sum = up16(l.hist + R * kHistStride * 4);
  l.reg_max = l.reg_sum + R * 8;
  l.reg_min = l.reg_max + R * 4;
  l.n_open = up16(l.reg_min + R * 4);
  l.slab_delta = l.n_open + kRegStride * 4;
  l.ctr = l.slab_delta + kWavesHw * kRegStride * 4;
  l.tmp = l.ctr + 16 * 8;
  l.vf = l.tmp + 16 * 4;
  static_assert(T_COUNT <= 16, "temporaries");
  l.pos = l.vf + 32 * 8;
  l.adv = l.pos + 16 * 4;
  l.total = l.adv + 16 * 4;
  return l;
}

struct WideParams {
  const uint32_t* wg_hdrs;  // 32 words per recorded workgroup
  const uint2* records;     // {tag, payload}
  uint64_t* out;
  uint32_t n_wg, W, R, cap, cap_log2, rec_cost, flush, nrec;
  uint32_t range_log2;      // ranks of one wave in LDS at a time: kK >> ceil(log2 W)
  WideLds lds;
};

__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
  return v;
}

__global__ __launch_bounds__(kBlock) void kp_reduce_wide(WideParams p) {
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned long long* keys = reinterpret_cast<unsigned long long*>(smem + p.lds.keys);
  uint32_t* table = reinterpret_cast<uint32_t*>(smem + p.lds.table);    // rank -> winning slot + 1, for the ranks in LDS
  uint32_t* list = reinterpret_cast<uint32_t*>(smem + p.lds.list);      // wave << 20 | slot of the records outside the slot of their seq
  uint32_t* bitmap = reinterpret_cast<uint32_t*>(smem + p.lds.bitmap);  // bit wave * cap + rank: the record is a paired START or END
  unsigned long long* otri = reinterpret_cast<unsigned long long*>(smem + p.lds.otri);  // pair (a <= b) at b (b + 1) / 2 + a
  uint32_t* hist = reinterpret_cast<uint32_t*>(smem + p.lds.hist);
  unsigned long long* reg_sum = reinterpret_cast<unsigned long long*>(smem + p.lds.reg_sum);
  uint32_t* reg_max = reinterpret_cast<uint32_t*>(smem + p.lds.reg_max);
  uint32_t* reg_min = reinterpret_cast<uint32_t*>(smem + p.lds.reg_min);
  int32_t* n_open = reinterpret_cast<int32_t*>(smem + p.lds.n_open);          // waves that have the region open, at the window's start
  int32_t* slab_delta = reinterpret_cast<int32_t*>(smem + p.lds.slab_delta);  // [hardware wave][region]: net change over its slab
  unsigned long long* ctr = reinterpret_cast<unsigned long long*>(smem + p.lds.ctr);
  uint32_t* tmp = reinterpret_cast<uint32_t*>(smem + p.lds.tmp);
  uint2* sVF = reinterpret_cast<uint2*>(smem + p.lds.vf);               // per wave: records held, first surviving seq
  uint32_t* pos = reinterpret_cast<uint32_t*>(smem + p.lds.pos);        // per wave: first rank of the range in LDS
  uint32_t* adv = reinterpret_cast<uint32_t*>(smem + p.lds.adv);        // per wave: ranks the window took

  const uint32_t tid = threadIdx.x, lane = tid & 63u, hw = tid >> 6;
  const uint32_t W = p.W, R = p.R, cap = p.cap, capm = cap - 1u, cl2 = p.cap_log2, nrec = p.nrec;
  const uint32_t rsh = p.range_log2, C = 1u << rsh;
  const StatsLayout SL = stats_layout(p.n_wg, W, R);
  if (p.out[H_STATUS] != 0) return;  // device header did not match the launch geometry

  for (uint32_t i = tid; i < R * kHistStride; i += kBlock) hist[i] = 0;
  for (uint32_t i = tid; i < R * (R + 1) / 2; i += kBlock) otri[i] = 0;
  for (uint32_t i = tid; i < R; i += kBlock) { reg_sum[i] = 0; reg_max[i] = 0; reg_min[i] = 0xFFFFFFFFu; }
  if (tid < 16) ctr[tid] = 0;
  __syncthreads();

  // The (wave, region) walks of this thread: entry e = wave * R + region.  Consecutive entries go to
  // different hardware waves: a walk's lane is busy at one record in R while the other lanes of its
  // hardware wave wait, so the walks that are busy at the same time should not share one.
  uint32_t ee[2], ew[2], er[2];
  bool ehas[2];
#pragma unroll
  for (int x = 0; x < 2; ++x) {
    ee[x] = hw + kWavesHw * (lane + 64u * x);
    ehas[x] = ee[x] < W * R;
    ew[x] = ehas[x] ? ee[x] / R : 0u;
    er[x] = ee[x] - ew[x] * R;
  }

  for (uint32_t wg = blockIdx.x; wg < p.n_wg; wg += gridDim.x) {
    const uint32_t* wh = p.wg_hdrs + (size_t)32 * wg;
    const uint2* recs = p.records + (size_t)wg * nrec;
    __syncthreads();  // every wave is done with the workgroup before

    // ---- workgroup header ------------------------------------------------------------------------
    if (tid <= KP_MAX_WAVES) {  // (entries from W up: no records)
      const uint32_t T = tid < W ? wh[8 + tid] : 0u;
      const uint32_t V = T < cap ? T : cap;
      sVF[tid] = make_uint2(V, p.flush ? 0u : T - V);
      if (tid < W) {
        atomicAdd(&ctr[H_DROPPED], (unsigned long long)(T - V));
        atomicAdd(&ctr[H_SLOTS_VALID], (unsigned long long)V);
      }
    }
    if (tid < T_COUNT) tmp[tid] = 0;
    if (tid < kRegStride) n_open[tid] = 0;
    for (uint32_t i = tid; i < (nrec + 31u) / 32u; i += kBlock) bitmap[i] = 0;
    __syncthreads();
    uint32_t held = 0, max_v = 0;
    for (uint32_t w = 0; w < W; ++w) {
      const uint32_t V = sVF[w].x;
      held += V;
      max_v = V > max_v ? V : max_v;
    }
    const bool span_overflow = (((uint64_t)wh[4] | ((uint64_t)wh[5] << 32)) - ((uint64_t)wh[2] | ((uint64_t)wh[3] << 32))) >> 32 != 0;

    // A record that passes the checks of its fields: its rank, else all ones.
    auto rank_of = [&](uint2 rec, uint32_t w, uint32_t s) -> uint32_t {
      const uint2 vf = sVF[w];
      const uint32_t k = (rec.x - vf.y) & kSeqMask;  // the low 20 bits of tag - first are those of seq - first
      const bool good = s < vf.x && k < vf.x && ((rec.x >> 20) & 0xFu) == w && ((rec.x >> 24) & 0x7Fu) < R;
      return good ? k : 0xFFFFFFFFu;
    };

    // ---- pass 0: every slot once -------------------------------------------------------------------
    {
      uint32_t c_field = 0, c_dis = 0;
      for (uint32_t i = tid; i < nrec; i += kBlock) {
        const uint2 rec = recs[i];
        const uint32_t s = i & capm;
        const bool good = rank_of(rec, i >> cl2, s) != 0xFFFFFFFFu;
        c_field += good ? 1u : 0u;
        if (good && ((rec.x ^ s) & capm) != 0u) {
          ++c_dis;
          const uint32_t at = atomicAdd(&tmp[T_LISTED], 1u);
          if (at < kList) list[at] = ((i >> cl2) << 20) | s;
        }
      }
      c_field = wave_sum(c_field);
      c_dis = wave_sum(c_dis);
      if (lane == 0) {
        if (c_field) atomicAdd(&tmp[T_FIELDVALID], c_field);
        if (c_dis) atomicAdd(&tmp[T_DISORDER], c_dis);
      }
    }
    __syncthreads();
    // Records that all sit in the slot of their own seq have distinct seq modulo the ring size, hence
    // distinct ranks, and rank k of a wave is in slot (first + k) mod cap.
    const bool displaced = tmp[T_DISORDER] != 0u;
    const uint32_t n_listed = tmp[T_LISTED] <= kList ? tmp[T_LISTED] : 0xFFFFFFFFu;  // all ones: the list is not complete
    uint32_t n_occupied = tmp[T_FIELDVALID], n_disorder = 0;

    // The ranks pos[w] .. pos[w] + C of every wave: which slot holds each (the later slot wins).
    auto build_table = [&]() {
      __syncthreads();  // pos[] is written, the table's last readers are done
      table[tid] = 0; table[tid + kBlock] = 0;
      __syncthreads();
      auto offer = [&](uint32_t w, uint32_t s) {
        const uint32_t k = rank_of(recs[(size_t)w * cap + s], w, s);
        if (k == 0xFFFFFFFFu) return;
        const uint32_t d = k - pos[w];
        if (d < C) atomicMax(&table[(w << rsh) + d], s + 1u);
      };
      if (n_listed != 0xFFFFFFFFu) {
        // a record in the slot of its seq: rank k of a wave is in slot (first + k) mod cap; the others: listed
#pragma unroll
        for (int x = 0; x < 2; ++x) {
          const uint32_t idx = tid + x * kBlock, w = idx >> rsh;
          if (w >= W) continue;
          const uint2 vf = sVF[w];
          const uint32_t k = pos[w] + (idx & (C - 1u));
          if (k < vf.x) offer(w, (vf.y + k) & capm);
        }
        for (uint32_t i = tid; i < n_listed; i += kBlock) offer(list[i] >> 20, list[i] & 0xFFFFFu);
      } else {
        for (uint32_t i = tid; i < nrec; i += kBlock) offer(i >> cl2, i & capm);
      }
      __syncthreads();
    };
    // The record at place idx of the ranks in LDS, (wave idx >> rsh, rank pos + (idx & (C - 1))); false: none.
    auto fetch = [&](uint32_t idx, uint2& rec) -> bool {
      const uint32_t w = idx >> rsh, j = idx & (C - 1u);
      if (w >= W) return false;
      const uint2 vf = sVF[w];
      const uint32_t k = pos[w] + j;
      if (k >= vf.x) return false;
      if (displaced) {
        const uint32_t t = table[idx];
        if (t == 0u) return false;
        rec = recs[(size_t)w * cap + (t - 1u)];
        return true;
      }
      const uint32_t s = (vf.y + k) & capm;
      rec = recs[(size_t)w * cap + s];
      return rank_of(rec, w, s) == k;
    };

    if (displaced) {
      uint32_t occ = 0, dis = 0;
      for (uint32_t k0 = 0; k0 < max_v; k0 += C) {
        if (tid < 16) pos[tid] = k0;
        build_table();
#pragma unroll
        for (int x = 0; x < 2; ++x) {
          const uint32_t idx = tid + x * kBlock, t = table[idx];
          if (t) {
            const uint32_t s = t - 1u;
            ++occ;
            dis += (s != (recs[(size_t)(idx >> rsh) * cap + s].x & capm)) ? 1u : 0u;
          }
        }
      }
      occ = wave_sum(occ);
      dis = wave_sum(dis);
      if (lane == 0) { atomicAdd(&tmp[T_OCCUPIED], occ); atomicAdd(&tmp[T_WINNER_DISORDER], dis); }
      __syncthreads();
      n_occupied = tmp[T_OCCUPIED];
      n_disorder = tmp[T_WINNER_DISORDER];
    }
    const uint32_t wg_invalid = held - n_occupied;  // slots that hold a record and did not make it into the ordered sequence

    // ---- pass 1: pairing, durations, per-(wave, region) statistics, monotonicity ---------------------
    {
      bool have_prev[2] = {false, false}, prev_end[2] = {false, false};
      uint32_t prev_ts[2] = {0, 0}, prev_k[2] = {0, 0};
      uint32_t n[2] = {0, 0}, mx[2] = {0, 0}, mn[2] = {0xFFFFFFFFu, 0xFFFFFFFFu}, orphan_s[2] = {0, 0}, orphan_e[2] = {0, 0};
      unsigned long long sum[2] = {0, 0};
      bool have_any[2] = {false, false};  // (region 0's walk of a wave also checks the wave's clocks)
      uint32_t last_ts[2] = {0, 0}, nonmono = 0;
      for (uint32_t k0 = 0; k0 < max_v; k0 += C) {
        __syncthreads();  // the walks over the previous range are done
        if (tid < 16) pos[tid] = k0;
        if (displaced) build_table(); else __syncthreads();
#pragma unroll
        for (int x = 0; x < 2; ++x) {
          const uint32_t idx = tid + x * kBlock;
          uint2 rec = make_uint2(0u, 0u);
          const bool ok = fetch(idx, rec);
          // clock | 1 << 8 | END << 7 | region
          keys[idx] = ok ? ((unsigned long long)rec.y << 32) | 0x100u | (rec.x >> 24) : 0ull;
        }
        __syncthreads();
#pragma unroll
        for (int x = 0; x < 2; ++x) {
          if (!ehas[x]) continue;
          const uint32_t w = ew[x], V = sVF[w].x, mine = 0x100u | er[x];
          const uint32_t nj = V > k0 ? (V - k0 < C ? V - k0 : C) : 0u;
          const uint4* ent = reinterpret_cast<const uint4*>(keys + (w << rsh));  // two entries per load
          // four entries per step, so that their loads are in flight together (places past the wave's last
          // record hold no record; the range is a multiple of four long)
          for (uint32_t j4 = 0; j4 < nj; j4 += 4u) {
            const uint4 e01 = ent[j4 / 2u], e23 = ent[j4 / 2u + 1u];
            const uint32_t ms[4] = {e01.x, e01.z, e23.x, e23.z}, tss[4] = {e01.y, e01.w, e23.y, e23.w};
#pragma unroll
            for (uint32_t u = 0; u < 4u; ++u) {
            const uint32_t j = j4 + u, m = ms[u], ts = tss[u];
            if (!(m & 0x100u)) continue;  // no record at this rank
            if (er[x] == 0u) {
              nonmono += (have_any[x] && ts < last_ts[x]) ? 1u : 0u;
              last_ts[x] = ts; have_any[x] = true;
            }
            if ((m & 0x17Fu) != mine) continue;
            const bool is_end = (m & 0x80u) != 0u;
            if (!is_end) {
              orphan_s[x] += (have_prev[x] && !prev_end[x]) ? 1u : 0u;  // START START
            } else if (have_prev[x] && !prev_end[x]) {
              const uint32_t d_raw = ts - prev_ts[x];
              const uint32_t d = d_raw > p.rec_cost ? d_raw - p.rec_cost : 0u;
              ++n[x]; sum[x] += d;
              mx[x] = d > mx[x] ? d : mx[x];
              mn[x] = d < mn[x] ? d : mn[x];
              atomicAdd(&hist[er[x] * kHistStride + (31 - __clz(d | 1u))], 1u);
              const uint32_t b0 = w * cap + prev_k[x], b1 = w * cap + k0 + j;
              atomicOr(&bitmap[b0 >> 5], 1u << (b0 & 31u));
              atomicOr(&bitmap[b1 >> 5], 1u << (b1 & 31u));
            } else {
              ++orphan_e[x];
            }
            have_prev[x] = true; prev_end[x] = is_end; prev_ts[x] = ts; prev_k[x] = k0 + j;
            }
          }
        }
      }
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        if (!ehas[x]) continue;
        orphan_s[x] += (have_prev[x] && !prev_end[x]) ? 1u : 0u;  // START at the end of the sequence
        uint64_t* dst = p.out + SL.per + ((size_t)wg * W * R + ee[x]) * 2;
        dst[0] = sum[x];
        dst[1] = (uint64_t)n[x] | ((uint64_t)mx[x] << 32);
        if (n[x]) {
          atomicAdd(&reg_sum[er[x]], sum[x]);
          atomicMax(&reg_max[er[x]], mx[x]);
          atomicMin(&reg_min[er[x]], mn[x]);
          atomicAdd(&tmp[T_PAIRS], n[x]);
        }
        if (orphan_s[x]) atomicAdd(&tmp[T_ORPHAN_START], orphan_s[x]);
        if (orphan_e[x]) atomicAdd(&tmp[T_ORPHAN_END], orphan_e[x]);
      }
      if (nonmono) atomicAdd(&tmp[T_NONMONO], nonmono);
    }
    __syncthreads();
    const bool eligible = !span_overflow && wg_invalid == 0u && tmp[T_NONMONO] == 0u;
    if (tid == 0) {
      ctr[H_INVALID] += wg_invalid;
      ctr[H_DISORDER] += n_disorder;
      ctr[H_NONMONO] += tmp[T_NONMONO];
      ctr[H_PAIRS] += tmp[T_PAIRS];
      ctr[H_ORPHAN_START] += tmp[T_ORPHAN_START];
      ctr[H_ORPHAN_END] += tmp[T_ORPHAN_END];
      ctr[H_SPAN_OVF] += span_overflow ? 1u : 0u;
      ctr[H_OVERLAP_WGS] += eligible ? 1u : 0u;
    }
    if (!eligible) continue;  // (the same in every thread)

    // ---- pass 2: region-pair overlap -----------------------------------------------------------------
    // Every rank below a wave's record count holds a record here and the clocks of a wave do not decrease.
    if (tid < 16) pos[tid] = 0;
    for (uint32_t round = 0; round <= nrec; ++round) {  // (every window takes at least one record: the bound is never reached)
      __syncthreads();
      bool more = false;
      for (uint32_t w = 0; w < W; ++w) more = more || pos[w] < sVF[w].x;
      if (!more) break;
      __syncthreads();
      if (tid == 0) { tmp[T_WINDOW_END] = 0xFFFFFFFFu; tmp[T_ADVANCED] = 0; }
      if (tid < 16) adv[tid] = 0;
      if (displaced) build_table(); else __syncthreads();
      // clock << 9 | not marked << 8 | region << 1 | END
      unsigned long long mine[2];
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        const uint32_t idx = tid + x * kBlock, w = idx >> rsh, j = idx & (C - 1u);
        uint2 rec = make_uint2(0u, 0u);
        const bool ok = fetch(idx, rec);
        mine[x] = kNoKey;
        if (ok) {
          const uint32_t k = pos[w] + j, b = w * cap + k;
          const uint32_t marked = (bitmap[b >> 5] >> (b & 31u)) & 1u;
          mine[x] = ((unsigned long long)rec.y << 9) | ((marked ^ 1u) << 8) | (((rec.x >> 24) & 0x7Fu) << 1) | (rec.x >> 31);
          // a wave with records beyond this range: the window cannot reach past the range's last clock
          if (j == C - 1u && k + 1u < sVF[w].x) atomicMin(&tmp[T_WINDOW_END], rec.y);
        }
        keys[idx] = mine[x];
      }
      __syncthreads();
      const uint32_t window_end = tmp[T_WINDOW_END];
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        const uint32_t idx = tid + x * kBlock, w = idx >> rsh, j = idx & (C - 1u);
        const unsigned long long next = j == C - 1u ? kNoKey : keys[idx + 1u];
        const bool inside = mine[x] != kNoKey && (uint32_t)(mine[x] >> 9) <= window_end;
        const bool next_inside = next != kNoKey && (uint32_t)(next >> 9) <= window_end;
        if (inside && !next_inside) { adv[w] = j + 1u; tmp[T_ADVANCED] = 1u; }  // the records inside are the first ones of the range
        mine[x] = inside ? mine[x] : kNoKey;  // (records that are no events stay: every wave's run stays in clock order)
      }
      __syncthreads();
      keys[tid] = mine[0]; keys[tid + kBlock] = mine[1];
      __syncthreads();
      if (tmp[T_ADVANCED] == 0u) break;  // (cannot happen, see above)
      // The runs of the waves (C places each, in clock order; places without a record at the end) are merged
      // by clock, pairs of runs of `size / 2` at a time: the first step compares place i of the lower run
      // with place size/2 - 1 - i of the upper one, the others are the half-cleaners of a bitonic merge.
      for (uint32_t size = 2u * C; size <= kK; size <<= 1) {
        const uint32_t half = size >> 1;
        {
          const uint32_t blk = (tid / half) * size, i = tid & (half - 1u), lo = blk + i, hi = blk + size - 1u - i;
          const unsigned long long a = keys[lo], b = keys[hi];
          if ((a >> 9) > (b >> 9)) { keys[lo] = b; keys[hi] = a; }
          __syncthreads();
        }
        for (uint32_t stride = half >> 1; stride > 0; stride >>= 1) {
          const uint32_t lo = ((tid & ~(stride - 1u)) << 1) | (tid & (stride - 1u)), hi = lo | stride;
          const unsigned long long a = keys[lo], b = keys[hi];
          if ((a >> 9) > (b >> 9)) { keys[lo] = b; keys[hi] = a; }
          __syncthreads();
        }
      }
      // slab of this hardware wave, two places per lane: lane l holds places l and 64 + l
      const unsigned long long place0 = keys[hw * kSlab + lane], place1 = keys[hw * kSlab + 64u + lane];
      const uint32_t low0 = (uint32_t)place0, high0 = (uint32_t)(place0 >> 32), low1 = (uint32_t)place1, high1 = (uint32_t)(place1 >> 32);
      // net change per region over the slab
      slab_delta[hw * kRegStride + lane] = 0;
      slab_delta[hw * kRegStride + 64u + lane] = 0;  // (LDS operations of one wave take effect in order)
      if (place0 != kNoKey && !(low0 & 0x100u)) atomicAdd(&slab_delta[hw * kRegStride + ((low0 >> 1) & 0x7Fu)], (low0 & 1u) ? -1 : 1);
      if (place1 != kNoKey && !(low1 & 0x100u)) atomicAdd(&slab_delta[hw * kRegStride + ((low1 >> 1) & 0x7Fu)], (low1 & 1u) ? -1 : 1);
      __syncthreads();
      {
        int32_t c_lo = n_open[lane], c_hi = n_open[64u + lane];  // waves that have region lane, lane + 64 open
        for (uint32_t h = 0; h < hw; ++h) {
          c_lo += slab_delta[h * kRegStride + lane];
          c_hi += slab_delta[h * kRegStride + 64u + lane];
        }
        // Which events open or close their region: the number of waves that have the region open right
        // before the event is the number at the slab's start plus the STARTs minus the ENDs of the region
        // at earlier places of the slab.  The lanes whose event has the same region come from one ballot per
        // bit of the region number.
        const bool ev0 = place0 != kNoKey && !(low0 & 0x100u), ev1 = place1 != kNoKey && !(low1 & 0x100u);
        const uint32_t r0 = (low0 >> 1) & 0x7Fu, r1 = (low1 >> 1) & 0x7Fu;
        const bool end0 = (low0 & 1u) != 0u, end1 = (low1 & 1u) != 0u;
        uint64_t same00 = __builtin_amdgcn_ballot_w64(ev0);  // places 0..63 with the region of this lane's place there
        uint64_t same01 = same00;                              // places 0..63 with the region of this lane's place 64 + lane
        uint64_t same11 = __builtin_amdgcn_ballot_w64(ev1);  // places 64..127 with that region
#pragma unroll
        for (uint32_t b = 0; b < 7u; ++b) {
          const uint64_t set0 = __builtin_amdgcn_ballot_w64(ev0 && ((r0 >> b) & 1u));
          const uint64_t set1 = __builtin_amdgcn_ballot_w64(ev1 && ((r1 >> b) & 1u));
          same00 &= ((r0 >> b) & 1u) ? set0 : ~set0;
          same01 &= ((r1 >> b) & 1u) ? set0 : ~set0;
          same11 &= ((r1 >> b) & 1u) ? set1 : ~set1;
        }
        const uint64_t ends0 = __builtin_amdgcn_ballot_w64(ev0 && end0), ends1 = __builtin_amdgcn_ballot_w64(ev1 && end1);
        const uint64_t below = (1ull << lane) - 1ull;
        auto net = [](uint64_t places, uint64_t ends) -> int32_t {  // STARTs minus ENDs among `places`
          return (int32_t)__popcll(places & ~ends) - (int32_t)__popcll(places & ends);
        };
        // the counts at the slab's start sit in the lane of the region
        const int32_t at0_lo = __shfl(c_lo, (int)(r0 & 63u), 64), at0_hi = __shfl(c_hi, (int)(r0 & 63u), 64);
        const int32_t at1_lo = __shfl(c_lo, (int)(r1 & 63u), 64), at1_hi = __shfl(c_hi, (int)(r1 & 63u), 64);
        const int32_t before0 = (r0 < 64u ? at0_lo : at0_hi) + net(same00 & below, ends0);
        const int32_t before1 = (r1 < 64u ? at1_lo : at1_hi) + net(same01, ends0) + net(same11 & below, ends1);
        // the region opens (no wave had it open) or closes (the last wave that had it open)
        const uint64_t switch0 = __builtin_amdgcn_ballot_w64(ev0 && before0 == (end0 ? 1 : 0));
        const uint64_t switch1 = __builtin_amdgcn_ballot_w64(ev1 && before1 == (end1 ? 1 : 0));
        // Only these events change the set of open regions; they are taken one after the other, each
        // lane holding whether its two regions (lane, lane + 64) are open.
        bool open_lo = c_lo > 0, open_hi = c_hi > 0;
        auto take = [&](uint64_t todo, uint32_t low_v, uint32_t high_v) {
          while (todo) {
            const int src = (int)__builtin_ctzll(todo);
            todo &= todo - 1ull;
            const uint32_t low = (uint32_t)__builtin_amdgcn_readlane((int)low_v, src);
            const uint32_t high = (uint32_t)__builtin_amdgcn_readlane((int)high_v, src);
            const uint32_t r = (low >> 1) & 0x7Fu, t = (low >> 9) | (high << 23);
            const bool is_end = (low & 1u) != 0u;
            const unsigned long long val = is_end ? (unsigned long long)t : 0ull - (unsigned long long)t;
            const uint32_t b0 = lane, b1 = lane + 64u;
            if (b0 < R && (b0 == r || open_lo)) {
              const uint32_t a = b0 < r ? b0 : r, b = b0 < r ? r : b0;
              atomicAdd(&otri[b * (b + 1u) / 2u + a], val);
            }
            if (b1 < R && (b1 == r || open_hi)) {
              const uint32_t a = b1 < r ? b1 : r, b = b1 < r ? r : b1;
              atomicAdd(&otri[b * (b + 1u) / 2u + a], val);
            }
            if (b0 == r) open_lo = !is_end;
            if (b1 == r) open_hi = !is_end;
          }
        };
        take(switch0, low0, high0);
        take(switch1, low1, high1);
      }
      __syncthreads();
      if (tid < kRegStride) {
        int32_t s = 0;
        for (uint32_t h = 0; h < kWavesHw; ++h) s += slab_delta[h * kRegStride + tid];
        n_open[tid] += s;
      }
      if (tid < W) pos[tid] += adv[tid];
    }
  }
  __syncthreads();

  // ---- flush this decoder workgroup's totals ----------------------------------------------------
  unsigned long long* out = reinterpret_cast<unsigned long long*>(p.out);
  for (uint32_t i = tid; i < R * 64; i += kBlock) {
    const uint32_t h = hist[(i >> 6) * kHistStride + (i & 63u)];
    if (h) atomicAdd(&out[SL.hist + i], (unsigned long long)h);
  }
  for (uint32_t i = tid; i < R * R; i += kBlock) {  // staged in the F area until finalize; entry (a, b) with a <= b holds the pair's sum
    const uint32_t a = i / R, b = i - a * R;
    if (a <= b && otri[b * (b + 1u) / 2u + a]) atomicAdd(&out[SL.F + i], otri[b * (b + 1u) / 2u + a]);
  }
  for (uint32_t r = tid; r < R; r += kBlock) {
    if (reg_min[r] != 0xFFFFFFFFu || reg_max[r] || reg_sum[r]) {
      atomicAdd(&out[SL.sum + r], reg_sum[r]);
      atomicMax(&out[SL.max + r], (unsigned long long)reg_max[r]);
      atomicMin(&out[SL.min + r], (unsigned long long)reg_min[r]);
    }
  }
  if (tid < H_STATUS && ctr[tid]) atomicAdd(&out[tid], ctr[tid]);
}

}  // namespace

namespace kp_reduce {

kp_status wide_supported(const kp_trace_hdr& h) {
  const uint32_t nrec = h.waves_per_wg * h.cap_wave;
  const uint32_t need = wide_lds(h.n_regions, nrec).total;
  if (need > kMaxLds)
    return kp::fail(KP_ERR_UNSUPPORTED_SHAPE,
                    "%u record slots per workgroup with %u regions: the decoder needs %u B of LDS (limit %u)", nrec,
                    h.n_regions, need, kMaxLds);
  return KP_OK;
}

kp_status launch_wide(const uint32_t* wg_hdrs, const void* records, uint64_t* out, const kp_trace_hdr& h,
                      hipStream_t s) {
  const kp_status ok = wide_supported(h);
  if (ok != KP_OK) return ok;
  WideParams p;
  p.wg_hdrs = wg_hdrs;
  p.records = static_cast<const uint2*>(records);
  p.out = out;
  p.n_wg = h.n_wg; p.W = h.waves_per_wg; p.R = h.n_regions; p.cap = h.cap_wave;
  p.cap_log2 = 0; while ((1u << p.cap_log2) < p.cap) ++p.cap_log2;
  p.rec_cost = h.rec_cost; p.flush = h.flags & KP_FLAG_FLUSH;
  p.nrec = p.W * p.cap;
  uint32_t wl2 = 0; while ((1u << wl2) < p.W) ++wl2;
  p.range_log2 = 11u - wl2;  // kK = 2^11 places
  p.lds = wide_lds(p.R, p.nrec);
  static thread_local kp_stage::LaunchCache cache;
  uint32_t grid = 0;
  const kp_status st = kp_stage::resident_grid(kp_reduce_wide, kBlock, p.lds.total, &cache, &grid);
  if (st != KP_OK) return st;
  if (grid > p.n_wg) grid = p.n_wg;
  hipLaunchKernelGGL(kp_reduce_wide, dim3(grid), dim3(kBlock), p.lds.total, s, p);
  KP_HIP_TRY(hipGetLastError());
  return KP_OK;
}

}  // namespace kp_reduce

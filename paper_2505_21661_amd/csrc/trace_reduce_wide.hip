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
//   1  pairing (an END is paired iff the nearest earlier record of its wave and region is a START):
//      hardware wave w walks recorded wave w, 64 ranks at a time, one per lane; the lanes that hold a
//      lane's region come from one ballot per bit of the region number, the last record of every region
//      in the ranks before from a table in LDS.  Durations go to the histogram and the region's extrema
//      in LDS and to the (workgroup, wave, region) row in HBM with atomics; a paired START and END each
//      set their bit in a bitmap of the workgroup's ranks;
//   2  overlap, a window of time at a time: every wave offers its next range of ranks, the window
//      ends at the earliest last clock among the waves that have more to offer, the marked records
//      inside the window are sorted by clock (bitonic, in LDS) and swept.  Each hardware wave sweeps a
//      slab of the sorted events, two events per lane: LDS atomics give the slab's net change of the
//      number of waves that have each region open, a prefix over the slabs the numbers at the slab's
//      start, ballots over the events of a region the number right before each event.  The time two
//      regions are both open is the sum over the ends of their common stretches minus the sum over the
//      beginnings; a common stretch of a and b begins when one of them opens while the other is open
//      and ends when one closes while the other is open, so every event that opens or closes a region
//      adds its clock, signed, to the sums of that region with every open region (modulo 2^64: the
//      total is exact).
// Nothing but the inputs and the statistics block is touched in HBM.
#include "kp_reduce.h"
#include "kp_stage.h"

namespace {

using namespace kp_reduce;

constexpr int kBlock = 1024;
constexpr uint32_t kWavesHw = kBlock / 64;
constexpr uint32_t kK = 2048;               // records in LDS at a time: 2 per thread
constexpr uint32_t kListMin = 512, kListMax = 8192;  // records outside the slot of their seq that a workgroup can list: what LDS has room for
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
  uint32_t keys, table, bitmap, otri, hist, reg_sum, reg_max, reg_min, n_open, slab_delta, ctr, tmp, vf, pos, adv, seen, rows, list, total;
  uint32_t rows_in_lds, list_cap;
};
inline uint32_t up16(uint32_t x) { return (x + 15u) & ~15u; }
WideLds wide_lds(uint32_t W, uint32_t R, uint32_t nrec) {
  WideLds l;
  l.keys = 0;
  l.table = l.keys + kK * 8;
  l.bitmap = l.table + kK * 4;
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
  l.seen = l.adv + 16 * 4;
  l.rows = l.seen + kWavesHw * 16;
  // what is left goes to the (wave, region) rows of the workgroup in flight, if they fit next to the
  // smallest list, and then to the list
  const uint32_t rows_bytes = W * R * 16;
  l.rows_in_lds = l.rows + rows_bytes + kListMin * 8 <= kMaxLds ? 1u : 0u;
  l.list = l.rows + (l.rows_in_lds ? rows_bytes : 0u);
  l.list_cap = kListMin;
  while (l.list_cap < kListMax && l.list + l.list_cap * 2 * 8 <= kMaxLds) l.list_cap *= 2;
  l.total = l.list + l.list_cap * 8;
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
  // the records outside the slot of their seq: (wave << 20 | rank) << 20 | slot, sorted
  unsigned long long* list = reinterpret_cast<unsigned long long*>(smem + p.lds.list);
  uint32_t* rows_lds = reinterpret_cast<uint32_t*>(smem + p.lds.rows);  // {u64 sum; u32 n; u32 max} per (wave, region), if p.lds.rows_in_lds
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
  uint32_t* seen_all = reinterpret_cast<uint32_t*>(smem + p.lds.seen);  // per hardware wave: the regions in its slab, one bit each

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
    for (uint32_t e = tid; e < W * R; e += kBlock) {
      keys[e] = 0ull;  // no last record of (wave, region) yet
      // pass 1 adds every pair to its row with atomics: in LDS, or in the statistics block itself
      if (p.lds.rows_in_lds) {
        reinterpret_cast<uint4*>(rows_lds)[e] = make_uint4(0u, 0u, 0u, 0u);
      } else {
        uint64_t* row = p.out + SL.per + ((size_t)wg * W * R + e) * 2;
        row[0] = 0ull; row[1] = 0ull;
      }
    }
    __threadfence();
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
          if (at < p.lds.list_cap) list[at] = ((unsigned long long)(((i >> cl2) << 20) | rank_of(rec, i >> cl2, s)) << 20) | s;
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
    // A workgroup with such records: which slot holds rank k (the later slot wins) comes from the sorted
    // list of those records, next to the slot the rank belongs in; a workgroup with more of them than the
    // list holds scans all its slots into a rank -> slot table, a range of ranks at a time.
    const bool listed = displaced && tmp[T_LISTED] <= p.lds.list_cap, tabled = displaced && !listed;
    const uint32_t n_listed = listed ? tmp[T_LISTED] : 0u;
    if (listed) {
      // sorted (bitonic) over the smallest power of two of places that holds it
      uint32_t n_sort = kListMin;
      while (n_sort < n_listed) n_sort <<= 1;
      for (uint32_t i = tid; i < n_sort; i += kBlock) {
        if (i >= n_listed) list[i] = kNoKey;
      }
      __syncthreads();
      for (uint32_t size = 2; size <= n_sort; size <<= 1) {
        for (uint32_t stride = size >> 1; stride > 0; stride >>= 1) {
          for (uint32_t i = tid; i < n_sort / 2u; i += kBlock) {
            const uint32_t lo = ((i & ~(stride - 1u)) << 1) | (i & (stride - 1u)), hi = lo | stride;
            const bool up = (lo & size) == 0u;
            const unsigned long long x = list[lo], y = list[hi];
            if ((x > y) == up) { list[lo] = y; list[hi] = x; }
          }
          __syncthreads();
        }
      }
    }
    // first place of the sorted list whose (wave << 20 | rank) is not below `prefix`
    auto list_lower_bound = [&](uint32_t prefix) -> uint32_t {
      uint32_t lo = 0, hi = n_listed;
      while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if ((uint32_t)(list[mid] >> 20) < prefix) lo = mid + 1u; else hi = mid;
      }
      return lo;
    };

    // The ranks pos[w] .. pos[w] + C of every wave: which slot holds each (the later slot wins).
    auto build_table = [&]() {
      __syncthreads();  // pos[] is written, the table's last readers are done
      table[tid] = 0; table[tid + kBlock] = 0;
      __syncthreads();
      for (uint32_t i = tid; i < nrec; i += kBlock) {
        const uint32_t w = i >> cl2, s = i & capm;
        const uint32_t k = rank_of(recs[i], w, s);
        if (k == 0xFFFFFFFFu) continue;
        const uint32_t d = k - pos[w];
        if (d < C) atomicMax(&table[(w << rsh) + d], s + 1u);
      }
      __syncthreads();
    };
    // The record at place idx of the ranks in LDS, (wave idx >> rsh, rank pos + (idx & (C - 1))); false: none.
    // (With a list: for workgroups in which no two records have the same rank, as pass 2 requires.)
    auto fetch = [&](uint32_t idx, uint2& rec) -> bool {
      const uint32_t w = idx >> rsh, j = idx & (C - 1u);
      if (w >= W) return false;
      const uint2 vf = sVF[w];
      const uint32_t k = pos[w] + j;
      if (k >= vf.x) return false;
      if (tabled) {
        const uint32_t t = table[idx];
        if (t == 0u) return false;
        rec = recs[(size_t)w * cap + (t - 1u)];
        return true;
      }
      const uint32_t s = (vf.y + k) & capm;
      rec = recs[(size_t)w * cap + s];
      if (rank_of(rec, w, s) == k) return true;
      if (!listed) return false;
      const uint32_t at = list_lower_bound((w << 20) | k);
      if (at >= n_listed || (uint32_t)(list[at] >> 20) != ((w << 20) | k)) return false;
      rec = recs[(size_t)w * cap + ((uint32_t)list[at] & 0xFFFFFu)];
      return true;
    };

    uint32_t n_occupied = 0, n_disorder = 0;
    if (tabled) {
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
    }

    // ---- pass 1: pairing, durations, per-(wave, region) statistics, monotonicity ---------------------
    // Hardware wave w takes recorded wave w, 64 consecutive ranks at a time, one per lane.  The nearest
    // earlier record of a lane's (wave, region) is the highest lower lane with the same region (the lanes
    // with a lane's region: one ballot per bit of the region number) or, when there is none, the last
    // record of that region in the ranks before, which the wave keeps in a table of its own.
    {
      uint2* last = reinterpret_cast<uint2*>(keys) + hw * R;  // per region: {clock, 1 << 31 | END << 30 | rank} of its last record
      uint32_t n_pairs = 0, orphan_s = 0, orphan_e = 0, nonmono = 0, occupied = 0, moved = 0;  // (the same in all lanes)
      bool carry_has = false;
      uint32_t carry_ts = 0;  // clock of the wave's last record so far
      const uint64_t below = (1ull << lane) - 1ull;
      uint64_t* rows = p.out + SL.per + ((size_t)wg * W + hw) * R * 2;
      uint32_t* rows_here = rows_lds + hw * R * 4u;
      auto group = [&](uint32_t k, bool ok, uint2 rec) {  // this lane: rank k, its record if ok
        const uint32_t r = (rec.x >> 24) & 0x7Fu, ts = rec.y;
        const bool is_end = (rec.x >> 31) != 0u;
        const uint64_t there = __builtin_amdgcn_ballot_w64(ok);
        if (there == 0ull) return;
        {  // clocks must not decrease from one record of the wave to the next
          const uint64_t lower = there & below;
          const uint32_t before = (uint32_t)__shfl((int)ts, lower ? 63 - (int)__builtin_clzll(lower) : 0, 64);
          const bool has = lower != 0ull || carry_has;
          nonmono += (uint32_t)__popcll(__builtin_amdgcn_ballot_w64(ok && has && ts < (lower ? before : carry_ts)));
          carry_ts = (uint32_t)__builtin_amdgcn_readlane((int)ts, 63 - (int)__builtin_clzll(there));
          carry_has = true;
        }
        uint64_t same = there;
#pragma unroll
        for (uint32_t b = 0; b < 7u; ++b) {
          const uint64_t set = __builtin_amdgcn_ballot_w64(ok && ((r >> b) & 1u));
          same &= ((r >> b) & 1u) ? set : ~set;
        }
        const uint64_t lower = same & below;
        const int src = lower ? 63 - (int)__builtin_clzll(lower) : 0;
        uint32_t pred_ts = (uint32_t)__shfl((int)ts, src, 64);
        uint32_t pred_info = (uint32_t)__shfl((int)(0x80000000u | ((uint32_t)is_end << 30) | k), src, 64);
        if (ok && lower == 0ull) { const uint2 c = last[r]; pred_ts = c.x; pred_info = c.y; }
        if (ok && (same >> lane) >> 1 == 0ull) last[r] = make_uint2(ts, 0x80000000u | ((uint32_t)is_end << 30) | k);  // the region's last record here
        const bool pred_start = ok && (pred_info >> 30) == 2u;  // there is one and it is a START
        const bool pair = pred_start && is_end;
        orphan_s += (uint32_t)__popcll(__builtin_amdgcn_ballot_w64(pred_start && !is_end));  // START START
        orphan_e += (uint32_t)__popcll(__builtin_amdgcn_ballot_w64(ok && is_end && !pred_start));
        const uint64_t pairs = __builtin_amdgcn_ballot_w64(pair);
        n_pairs += (uint32_t)__popcll(pairs);
        if (pair) {
          const uint32_t d_raw = ts - pred_ts;
          const uint32_t d = d_raw > p.rec_cost ? d_raw - p.rec_cost : 0u;
          atomicAdd(&hist[r * kHistStride + (31 - __clz(d | 1u))], 1u);
          atomicAdd(&reg_sum[r], (unsigned long long)d);
          atomicMax(&reg_max[r], d);
          atomicMin(&reg_min[r], d);
          const uint32_t b0 = hw * cap + (pred_info & kSeqMask), b1 = hw * cap + k;
          atomicOr(&bitmap[b0 >> 5], 1u << (b0 & 31u));
          atomicOr(&bitmap[b1 >> 5], 1u << (b1 & 31u));
          // row {u64 sum; u32 n; u32 max}, cleared above
          if (p.lds.rows_in_lds) {
            uint32_t* row = rows_here + 4u * r;
            atomicAdd(reinterpret_cast<unsigned long long*>(row), (unsigned long long)d);
            atomicAdd(row + 2, 1u);
            atomicMax(row + 3, d);
          } else {
            uint64_t* row = rows + 2u * r;
            atomicAdd(reinterpret_cast<unsigned long long*>(row), (unsigned long long)d);
            atomicAdd(reinterpret_cast<uint32_t*>(row) + 2, 1u);
            atomicMax(reinterpret_cast<uint32_t*>(row) + 3, d);
          }
        }
      };
      const uint32_t V = hw < W ? sVF[hw < W ? hw : 0u].x : 0u;
      if (!tabled) {
        // rank k belongs in slot (first + k) mod cap; nothing is shared with the other waves
        const uint32_t first = sVF[hw < W ? hw : 0u].y;
        uint32_t cursor = 0, cursor_end = 0;  // this wave's stretch of the sorted list
        if (listed && hw < W) { cursor = list_lower_bound(hw << 20); cursor_end = list_lower_bound((hw + 1u) << 20); }
        for (uint32_t k0 = 0; k0 < V; k0 += 256u) {
          uint2 rec[4];
          bool ok[4];
          uint32_t slot[4];
#pragma unroll
          for (int g = 0; g < 4; ++g) {  // (the loads are in flight together)
            const uint32_t k = k0 + 64u * g + lane;
            slot[g] = (first + k) & capm;
            rec[g] = recs[(size_t)hw * cap + (k < V ? slot[g] : 0u)];
            ok[g] = k < V && rank_of(rec[g], hw, slot[g]) == k;
          }
          if (cursor < cursor_end && ((uint32_t)(list[cursor] >> 20) & kSeqMask) < k0 + 256u) {
            // listed records whose rank is among these: a later slot displaces an earlier one
            bool moved_here[4] = {false, false, false, false};
            while (cursor < cursor_end) {
              const unsigned long long key = list[cursor];
              const uint32_t rank = (uint32_t)(key >> 20) & kSeqMask, s = (uint32_t)key & 0xFFFFFu;
              if (rank >= k0 + 256u) break;
              ++cursor;
#pragma unroll
              for (int g = 0; g < 4; ++g) {
                if (rank == k0 + 64u * g + lane && (!ok[g] || s > slot[g])) { slot[g] = s; ok[g] = true; moved_here[g] = true; }
              }
            }
#pragma unroll
            for (int g = 0; g < 4; ++g) {
              if (moved_here[g]) rec[g] = recs[(size_t)hw * cap + slot[g]];
            }
          }
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            occupied += (uint32_t)__popcll(__builtin_amdgcn_ballot_w64(ok[g]));
            moved += (uint32_t)__popcll(__builtin_amdgcn_ballot_w64(ok[g] && ((rec[g].x ^ slot[g]) & capm) != 0u));
            group(k0 + 64u * g + lane, ok[g], rec[g]);
          }
        }
      } else {
        for (uint32_t k0 = 0; k0 < max_v; k0 += C) {
          if (tid < 16) pos[tid] = k0;
          build_table();
          for (uint32_t j0 = 0; j0 < C && k0 + j0 < V; j0 += 128u) {
            uint2 rec[2];
            bool ok[2];
#pragma unroll
            for (int g = 0; g < 2; ++g) {
              const uint32_t j = j0 + 64u * g + lane, t = table[(hw << rsh) + j];
              ok[g] = t != 0u;
              rec[g] = recs[(size_t)hw * cap + (ok[g] ? t - 1u : 0u)];
            }
#pragma unroll
            for (int g = 0; g < 2; ++g) group(k0 + j0 + 64u * g + lane, ok[g], rec[g]);
          }
        }
      }
      if (lane == 0 && hw < W) {
        if (n_pairs) atomicAdd(&tmp[T_PAIRS], n_pairs);
        if (orphan_s) atomicAdd(&tmp[T_ORPHAN_START], orphan_s);
        if (orphan_e) atomicAdd(&tmp[T_ORPHAN_END], orphan_e);
        if (nonmono) atomicAdd(&tmp[T_NONMONO], nonmono);
        if (occupied) atomicAdd(&tmp[T_OCCUPIED], occupied);
        if (moved) atomicAdd(&tmp[T_WINNER_DISORDER], moved);
      }
      __syncthreads();
      // a region whose last record is a START: that START has no END
      uint32_t open_ended = 0;
      for (uint32_t e = tid; e < W * R; e += kBlock) {
        open_ended += (reinterpret_cast<const uint2*>(keys)[e].y >> 30) == 2u ? 1u : 0u;
        if (p.lds.rows_in_lds) {
          uint64_t* row = p.out + SL.per + ((size_t)wg * W * R + e) * 2;
          row[0] = reinterpret_cast<const uint64_t*>(rows_lds)[2u * e];
          row[1] = reinterpret_cast<const uint64_t*>(rows_lds)[2u * e + 1u];
        }
      }
      open_ended = wave_sum(open_ended);
      if (lane == 0 && open_ended) atomicAdd(&tmp[T_ORPHAN_START], open_ended);
      n_occupied = tmp[T_OCCUPIED];
      n_disorder = tmp[T_WINNER_DISORDER];
    }
    const uint32_t wg_invalid = held - n_occupied;  // slots that hold a record and did not make it into the ordered sequence
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
      if (tabled) build_table(); else __syncthreads();
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
        // Each of these events adds its clock, signed, to the sums of its region with every region that is
        // open at that moment (and with itself: the time the region is open at all).  Region by region,
        // over the regions that are open at the slab's start or occur in it: whether region b is open
        // right before an event is again the count at the start plus the STARTs minus the ENDs of b at the
        // places before it.
        const bool sw0 = (switch0 >> lane) & 1ull, sw1 = (switch1 >> lane) & 1ull;
        const uint32_t t0 = (low0 >> 9) | (high0 << 23), t1 = (low1 >> 9) | (high1 << 23);
        const unsigned long long val0 = end0 ? (unsigned long long)t0 : 0ull - (unsigned long long)t0;
        const unsigned long long val1 = end1 ? (unsigned long long)t1 : 0ull - (unsigned long long)t1;
        uint32_t* seen = seen_all + hw * 4u;  // bit r: region r occurs in the slab
        if (lane < 4u) seen[lane] = 0u;       // (LDS operations of one wave take effect in order)
        if (ev0) atomicOr(&seen[r0 >> 5], 1u << (r0 & 31u));
        if (ev1) atomicOr(&seen[r1 >> 5], 1u << (r1 & 31u));
        const uint64_t starts0 = __builtin_amdgcn_ballot_w64(ev0 && !end0), starts1 = __builtin_amdgcn_ballot_w64(ev1 && !end1);
        auto with_region = [&](uint32_t b) {  // (b is the same in all lanes)
          const int32_t lo_c = __builtin_amdgcn_readlane(c_lo, (int)(b & 63u)), hi_c = __builtin_amdgcn_readlane(c_hi, (int)(b & 63u));
          const int32_t base = b < 64u ? lo_c : hi_c;
          const uint64_t is_b0 = __builtin_amdgcn_ballot_w64(ev0 && r0 == b), is_b1 = __builtin_amdgcn_ballot_w64(ev1 && r1 == b);
          const uint64_t s0 = is_b0 & starts0, e0 = is_b0 & ends0, s1 = is_b1 & starts1, e1 = is_b1 & ends1;
          const int32_t all0 = (int32_t)__popcll(s0) - (int32_t)__popcll(e0);
          const int32_t cnt0 = base + (int32_t)__popcll(s0 & below) - (int32_t)__popcll(e0 & below);
          const int32_t cnt1 = base + all0 + (int32_t)__popcll(s1 & below) - (int32_t)__popcll(e1 & below);
          if (sw0 && (r0 == b || cnt0 > 0)) {
            const uint32_t lo_r = r0 < b ? r0 : b, hi_r = r0 < b ? b : r0;
            atomicAdd(&otri[hi_r * (hi_r + 1u) / 2u + lo_r], val0);
          }
          if (sw1 && (r1 == b || cnt1 > 0)) {
            const uint32_t lo_r = r1 < b ? r1 : b, hi_r = r1 < b ? b : r1;
            atomicAdd(&otri[hi_r * (hi_r + 1u) / 2u + lo_r], val1);
          }
        };
        const uint32_t seen0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)seen[0]), seen1 = (uint32_t)__builtin_amdgcn_readfirstlane((int)seen[1]);
        const uint32_t seen2 = (uint32_t)__builtin_amdgcn_readfirstlane((int)seen[2]), seen3 = (uint32_t)__builtin_amdgcn_readfirstlane((int)seen[3]);
        for (uint64_t todo = __builtin_amdgcn_ballot_w64(c_lo > 0) | seen0 | ((uint64_t)seen1 << 32); todo; todo &= todo - 1ull)
          with_region((uint32_t)__builtin_ctzll(todo));
        for (uint64_t todo = __builtin_amdgcn_ballot_w64(c_hi > 0) | seen2 | ((uint64_t)seen3 << 32); todo; todo &= todo - 1ull)
          with_region(64u + (uint32_t)__builtin_ctzll(todo));
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
  const uint32_t need = wide_lds(h.waves_per_wg, h.n_regions, nrec).total;
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
  p.lds = wide_lds(p.W, p.R, p.nrec);
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

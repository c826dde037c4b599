// Staging of one recorded workgroup in LDS, shared by the replay kernels that walk the records of
// each wave in order (timeline rows, asynchronous waits).
//
// The paper stores START/END records unpaired, per warp, in a ring whose tail survives, and aligns
// them at trace replay (Sec. 4.2 "SM-level Data Layout", "Shared Memory Circular Buffer"; Sec. 4.3).
// Here every record goes to position wave * cap_wave + rank, rank = seq - first surviving seq, as a
// (clock, metadata) pair, which undoes ring rotation and out-of-order flushes in O(1) per record.
// A sequence number that occurs twice must leave the later slot in place; that is detected by
// counting the occupied ranks and repaired by a serial pass.
#pragma once
#include "kp_common.h"

namespace kp_stage {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr uint32_t kSeqMask = 0xFFFFFu;
// staged metadata: bits 6:0 region, 7 END, 8 valid, 31:16 generation of the staging pass
constexpr uint32_t kMRegion = 0x7Fu, kMEnd = 0x80u, kMValid = 0x100u;
constexpr uint32_t kLiveMask = 0xFFFF0000u | kMValid;
constexpr uint32_t kMaxRecPerWg = 16384;
constexpr uint32_t kMaxLds = 160 * 1024;

struct Trace {
  const uint32_t* wg_hdrs;  // 32 words per recorded workgroup
  const u32x4* records;     // two records per 16-byte load
  uint32_t n_wg, W, R, cap, cap_log2, rec_cost, flush, nrec;
};

// LDS of the staging step: byte offsets from the start of dynamic shared memory.
struct Lds { uint32_t rec, tmp, v, first, end; };
__host__ __device__ inline uint32_t align16(uint32_t x) { return (x + 15u) & ~15u; }
__host__ __device__ inline Lds lds_layout(uint32_t nrec) {
  Lds l;
  uint32_t o = 0;
  l.rec = o; o = align16(o + nrec * 8);
  l.tmp = o; o = align16(o + 4 * 4);     // [0] records accepted, [1] ranks occupied, [2] accepted outside their seq's slot
  l.v = o; o = align16(o + 16 * 4);      // records held per wave
  l.first = o; o = align16(o + 16 * 4);  // first surviving seq per wave
  l.end = o;
  return l;
}

__device__ inline uint32_t wave_sum(uint32_t v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
  return v;
}

// Lane l receives the value of lane l-1; lane 0 receives `lane0` (DPP wave shift right by one).
__device__ __forceinline__ uint32_t wave_shr1(uint32_t v, uint32_t lane0) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)lane0, (int)v, 0x138, 0xF, 0xF, false);
}

// Inclusive prefix sum over the 64 lanes: four shifts inside each row of 16, then the last lane of
// row 0/2 into row 1/3 and the last lane of the lower half into the upper half.
__device__ __forceinline__ uint32_t wave_scan_add(uint32_t v) {
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xF, 0xF, false);  // row_shr:1
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xF, 0xF, false);  // row_shr:2
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xF, 0xF, false);  // row_shr:4
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xF, 0xF, false);  // row_shr:8
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xA, 0xF, false);  // row_bcast:15
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xC, 0xF, false);  // row_bcast:31
  return v;
}

// The metadata tag of the records staged in pass `iter` of a persistent workgroup.  A staged word
// counts only if it carries the generation of its pass, so the staging area is cleared on the
// first pass and when the 16-bit generation wraps, not for every recorded workgroup.
__device__ __forceinline__ uint32_t live_tag_of(uint32_t iter) { return ((1u + iter % 0xFFFFu) << 16) | kMValid; }
__device__ __forceinline__ bool is_live(uint32_t m, uint32_t live_tag) { return (m & kLiveMask) == live_tag; }

// Stages recorded workgroup `wg`.  Every thread of the block calls it; it ends with a barrier, after
// which rec[w * cap + k] holds the record of rank k of wave w (live iff its metadata carries
// live_tag) and sV[w] the number of ranks of wave w.  The caller must put a barrier between its last
// read of the staging area and the next call.
template <int BLOCK>
__device__ __forceinline__ void stage_workgroup(const Trace& p, unsigned char* smem, const Lds& L, uint32_t wg,
                                                uint32_t iter) {
  uint2* rec = reinterpret_cast<uint2*>(smem + L.rec);
  uint32_t* recw = reinterpret_cast<uint32_t*>(smem + L.rec);  // word 2p = clock, 2p+1 = metadata
  uint32_t* tmp = reinterpret_cast<uint32_t*>(smem + L.tmp);
  uint32_t* sV = reinterpret_cast<uint32_t*>(smem + L.v);
  uint32_t* sFirst = reinterpret_cast<uint32_t*>(smem + L.first);
  const uint32_t tid = threadIdx.x, lane = tid & 63u;
  const uint32_t W = p.W, R = p.R, cap = p.cap, nrec = p.nrec, capm = cap - 1, cl2 = p.cap_log2;
  const uint32_t* wh = p.wg_hdrs + (size_t)32 * wg;
  const uint32_t live_tag = live_tag_of(iter);

  if (tid < W) {
    const uint32_t T = wh[8 + tid];
    const uint32_t V = T < cap ? T : cap;
    sV[tid] = V;
    sFirst[tid] = p.flush ? 0u : T - V;
  }
  if (tid >= 64 && tid < 67) tmp[tid - 64] = 0;
  if ((live_tag >> 16) == 1u) {
    u32x4* z = reinterpret_cast<u32x4*>(rec);
    for (uint32_t i = tid; i < nrec / 2; i += BLOCK) z[i] = u32x4{0u, 0u, 0u, 0u};
  }
  __syncthreads();
  // ---- load and scatter by rank ---------------------------------------------------------------
  {
    const u32x4* recs = p.records + (size_t)wg * (nrec / 2);
    const uint32_t n16 = nrec / 2;  // 16-byte units, two records each
    uint32_t c_field = 0, c_dis = 0;
    for (uint32_t i0 = tid; i0 < n16; i0 += 4 * BLOCK) {
      u32x4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const uint32_t i = i0 + u * BLOCK;
        v[u] = __builtin_nontemporal_load(recs + (i < n16 ? i : i0));
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const uint32_t i = i0 + u * BLOCK;
        const bool live = i < n16;
        const uint32_t f0 = 2 * (live ? i : i0);
        const uint32_t w = f0 >> cl2;
        const uint32_t V = live ? sV[w] : 0u, first = sFirst[w];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const uint32_t tag = h ? v[u].z : v[u].x, pay = h ? v[u].w : v[u].y;
          const uint32_t s = (f0 + h) & capm;
          const uint32_t k = ((tag & kSeqMask) - first) & kSeqMask;
          const uint32_t region = (tag >> 24) & 0x7Fu;
          const bool good = s < V && k < V && ((tag >> 20) & 0xFu) == w && region < R;
          c_field += good ? 1u : 0u;
          c_dis += (good && s != (tag & capm)) ? 1u : 0u;
          if (good) rec[(w << cl2) + k] = make_uint2(pay, region | ((tag >> 31) ? kMEnd : 0u) | live_tag);
        }
      }
    }
    c_field = wave_sum(c_field);
    if (lane == 0 && c_field) atomicAdd(&tmp[0], c_field);
    if (__builtin_amdgcn_ballot_w64(c_dis != 0u) && lane == 0) tmp[2] = 1u;
  }
  __syncthreads();
  // ---- a duplicated seq leaves fewer occupied ranks than accepted records ------------------------
  // Records that all sit in the slot of their own seq have distinct seq modulo the ring size, hence
  // distinct ranks: only a workgroup with a record elsewhere needs the count.
  if (tmp[2] == 0u) return;
  {
    uint32_t occ = 0;
    for (uint32_t q = tid; q < nrec; q += BLOCK) occ += is_live(recw[2 * q + 1], live_tag) ? 1u : 0u;
    occ = wave_sum(occ);
    if (lane == 0 && occ) atomicAdd(&tmp[1], occ);
  }
  __syncthreads();
  if (tmp[1] != tmp[0]) {
    // Rare: some seq occurs twice.  The later slot must win, so redo this workgroup's scatter in
    // slot order, one thread per wave.
    __syncthreads();
    for (uint32_t i = tid; i < nrec; i += BLOCK) recw[2 * i + 1] = 0;
    __syncthreads();
    if (tid < W) {
      const uint32_t w = tid, V = sV[w], first = sFirst[w];
      const uint32_t* seg = reinterpret_cast<const uint32_t*>(p.records) + ((size_t)wg * nrec + (size_t)w * cap) * 2;
      for (uint32_t s = 0; s < V; ++s) {
        const uint32_t tag = seg[2 * s];
        const uint32_t k = ((tag & kSeqMask) - first) & kSeqMask, region = (tag >> 24) & 0x7Fu;
        if (k >= V || ((tag >> 20) & 0xFu) != w || region >= R) continue;
        rec[w * cap + k] = make_uint2(seg[2 * s + 1], region | ((tag >> 31) ? kMEnd : 0u) | live_tag);
      }
    }
    __syncthreads();
  }
}

// Host-side checks common to the replay entry points; fills `t` from a validated header.
inline kp_status trace_from_header(const void* raw, size_t n, const kp_trace_hdr& h, const void* out, Trace* t) {
  if (h.magic != KP_TRACE_MAGIC || h.version != KP_TRACE_VERSION)
    return kp::fail(KP_ERR_BAD_TRACE, "trace header: bad magic/version (%08x, %u)", h.magic, h.version);
  if (h.waves_per_wg < 1 || h.waves_per_wg > KP_MAX_WAVES || h.n_regions < 1 || h.n_regions > 128 ||
      !kp::is_pow2(h.cap_wave) || h.cap_wave < 2)
    return kp::fail(KP_ERR_BAD_TRACE, "trace header: waves=%u regions=%u cap_wave=%u", h.waves_per_wg, h.n_regions, h.cap_wave);
  if ((size_t)h.n_wg * h.waves_per_wg * h.cap_wave != n)
    return kp::fail(KP_ERR_BAD_TRACE, "trace header describes %zu record slots, caller passed %zu",
                    (size_t)h.n_wg * h.waves_per_wg * h.cap_wave, n);
  if ((h.flags & ~(KP_FLAG_FLUSH | KP_FLAG_REALTIME | KP_FLAG_HW_IDS)) != 0) return kp::fail(KP_ERR_BAD_TRACE, "trace header: unknown flags %x", h.flags);
  const uint32_t nrec = h.waves_per_wg * h.cap_wave;
  if (nrec > kMaxRecPerWg)
    return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "%u records per workgroup exceed the LDS staging limit %u", nrec, kMaxRecPerWg);
  if (((uintptr_t)raw & 15u) || ((uintptr_t)out & 15u))
    return kp::fail(KP_ERR_INVALID_ARG, "raw and the output block must be 16-byte aligned");
  const uint8_t* base = static_cast<const uint8_t*>(raw);
  t->wg_hdrs = reinterpret_cast<const uint32_t*>(base + sizeof(kp_trace_hdr));
  t->records = reinterpret_cast<const u32x4*>(base + sizeof(kp_trace_hdr) + sizeof(kp_wg_hdr) * (size_t)h.n_wg);
  t->n_wg = h.n_wg; t->W = h.waves_per_wg; t->R = h.n_regions; t->cap = h.cap_wave;
  t->cap_log2 = 0; while ((1u << t->cap_log2) < h.cap_wave) ++t->cap_log2;
  t->rec_cost = h.rec_cost; t->flush = h.flags & KP_FLAG_FLUSH; t->nrec = nrec;
  return KP_OK;
}

// One hardware wave per recorded wave, and enough threads to stage the records quickly.
inline int block_threads(uint32_t W, uint32_t nrec) {
  return (W > 8 || nrec >= 8192) ? 1024 : ((W > 4 || nrec >= 2048) ? 512 : 256);
}

// Grid of a persistent kernel: as many workgroups as stay resident, at most one per recorded workgroup.
struct LaunchCache { int dev = -1; uint32_t lds = 0; uint32_t max_grid = 0; };
template <typename Kernel>
kp_status resident_grid(Kernel kern, int block, uint32_t lds_bytes, LaunchCache* cache, uint32_t* grid) {
  int dev = 0;
  KP_HIP_TRY(hipGetDevice(&dev));
  if (cache->dev != dev || cache->lds != lds_bytes) {
    KP_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes));
    int per_cu = 0, cus = 0;
    KP_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, block, lds_bytes));
    if (per_cu < 1) return kp::fail(KP_ERR_UNSUPPORTED_SHAPE, "replay kernel does not fit one CU (LDS %u B)", lds_bytes);
    KP_HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    cache->dev = dev; cache->lds = lds_bytes; cache->max_grid = (uint32_t)per_cu * (uint32_t)cus;
  }
  *grid = cache->max_grid;
  return KP_OK;
}

}  // namespace kp_stage

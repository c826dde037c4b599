// Device-side record path: ring init, record, flush (Sec. 3.1 InitOp / ReadCounterOp /
// StoreCounterOp / FinalizeOp semantics; Sec. 4.2 record layout and circular buffer).
//
// Every wave owns a private sub-ring of cap_wave 8-byte slots inside the workgroup's LDS ring
// (Sec. 4.2 "SM-level Data Layout": non-overlapping slots per profiling space), so recording
// needs no atomics.  The record counter and all tag fields are wave-uniform and live in scalar
// registers; the slot index is counter & (cap_wave-1) (Sec. 4.2: a cheap modular op with a
// precomputed capacity).  A record site only samples s_memtime; the 8-byte store of a record
// (one lane writes) is deferred to the next record site, so no site ever waits for the clock
// value it has just requested (the paper's split into ReadCounterOp and StoreCounterOp,
// Sec. 3.1).  A region's measured length therefore includes the constant cost of storing its
// own START record, which the decoder's rec_cost subtracts.  Kernels whose sites are a fixed sequence go
// one step further (chained sites, below): inside the loop they store only the clocks, one 4-byte entry
// per site, and the records are made from those when the trace is copied out.
//
// Circular strategy: the sub-ring is overwritten cyclically and copied to HBM once, at exit.
// Flush strategy: whenever a sub-ring fills up, its wave copies it to the next chunk of its HBM
// segment; records that no longer fit are counted as dropped (total_written - cap_wave).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "kperf.h"

namespace kp {

constexpr uint32_t kPhaseStart = 0u, kPhaseEnd = 1u;
constexpr uint32_t kNoPending = 0xFFFFFFFFu;
constexpr uint32_t kNoRegion = 0xFFu;

struct Ring {
  uint32_t* sub;       // LDS: this wave's sub-ring (2 dwords per slot)
  uint32_t sub_lds;    // the same as a 32-bit LDS byte address
  uint32_t cnt;        // records written by this wave so far
  uint32_t lds_mask;   // LDS sub-ring capacity - 1
  uint32_t tag_wave;   // wave index << 20
  uint32_t t0_lo;      // low 32 bits of the workgroup's t_begin
  uint32_t mask;       // enabled regions (none in a wave that does not write its group's stream)
  uint32_t stream;     // record stream of this wave: wave index >> group_log2
  uint32_t leader;     // 1 in the wave that writes the stream (the first wave of its group)
  uint32_t collab;     // generic sites only: 1 = all 64 lanes store a record to the same address (Sec. 4.2)
  uint32_t pend_tag;   // up to two records that share the last clock sample and are not in LDS yet
  uint32_t pend_tag2;  //   (an END and the START that follows it); kNoPending: none
  uint32_t stored;     // records already written to the LDS sub-ring
  uint64_t pend_t;     // its raw 64-bit clock; untouched until the store so nothing waits on s_memtime
  uint32_t cw;         // lean sites: tag_wave + records written so far (stands in for cnt); chained sites: sites so far
  uint32_t cmask;      // chained sites only: entries of the clock ring - 1
  uint64_t dq_t[4];    // chained sites only: raw clocks of up to four sites that are not in the clock ring yet
  uint64_t t_begin;    // workgroup start: s_memtime
  uint64_t rt_begin;   // workgroup start: s_memrealtime (constant rate)
  // flush strategy only
  uint32_t flush;      // 0 circular, 1 flush
  uint32_t cap_hbm;    // slots of this wave's HBM segment
  uint32_t* seg;       // HBM: this wave's segment
};

struct TraceGeom {
  uint32_t n_wg, waves, n_regions, cap_wave, flags;
};

__device__ __forceinline__ uint32_t wave_uniform(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }

// Workgroup prologue.  `ring_lds` holds streams * cap_lds slots.  `scratch_lds` (16 bytes) is only used
// inside this call to hand thread 0's clock samples to every wave and may be reused afterwards.
// Granularity (Sec. 3.1, the Granularity option; Sec. 4.2: one profiling space per warp group): with
// group_log2 = g the 2^g consecutive waves of a group share one record stream, which the first wave of
// the group writes on behalf of all; `streams` = waves per workgroup >> g.  Only the generic record
// sites (boundary / record) honour it.  GROUPS = false ignores group_log2 (taken as 0) and leaves the
// region mask as the caller gave it, so that a constant mask stays a constant in the record sites.
template <bool GROUPS = false>
__device__ __forceinline__ Ring ring_init(uint32_t* ring_lds, uint64_t* scratch_lds, uint32_t cap_lds,
                                          uint32_t region_mask, uint32_t flush, uint32_t cap_hbm,
                                          void* trace_buf, uint32_t n_wg, uint32_t streams, uint32_t wg,
                                          uint32_t group_log2 = 0) {
  const uint32_t hw_wave = wave_uniform(threadIdx.x >> 6);
  const uint32_t wave = GROUPS ? hw_wave >> group_log2 : hw_wave;  // the stream index stands where the wave index stood
  if (threadIdx.x == 0) {
    scratch_lds[0] = __builtin_readcyclecounter();
    scratch_lds[1] = __builtin_amdgcn_s_memrealtime();
  }
  __syncthreads();
  Ring r;
  {
    const uint64_t a = scratch_lds[0], b = scratch_lds[1];
    r.t_begin = ((uint64_t)wave_uniform((uint32_t)(a >> 32)) << 32) | wave_uniform((uint32_t)a);
    r.rt_begin = ((uint64_t)wave_uniform((uint32_t)(b >> 32)) << 32) | wave_uniform((uint32_t)b);
  }
  __syncthreads();  // scratch_lds may be overwritten from here on
  r.sub = ring_lds + (size_t)wave * cap_lds * 2;
  // the low 32 bits of a flat pointer into LDS are its LDS byte address
  r.sub_lds = wave_uniform((uint32_t)(uintptr_t)ring_lds) + wave * cap_lds * 8;
  r.cnt = 0;
  r.lds_mask = cap_lds - 1;
  r.tag_wave = wave << 20;
  r.t0_lo = (uint32_t)r.t_begin;
  r.stream = wave;
  r.leader = 1u;
  r.collab = 0u;
  r.mask = region_mask;
  if constexpr (GROUPS) {
    r.leader = (hw_wave & ((1u << group_log2) - 1u)) == 0u ? 1u : 0u;
    r.mask = r.leader ? region_mask : 0u;
  }
  r.pend_tag = kNoPending;
  r.pend_tag2 = kNoPending;
  r.stored = 0;
  r.pend_t = 0;
  r.flush = flush;
  r.cap_hbm = cap_hbm;
  r.seg = reinterpret_cast<uint32_t*>(static_cast<unsigned char*>(trace_buf) + sizeof(kp_trace_hdr) +
                                      sizeof(kp_wg_hdr) * (size_t)n_wg) +
          ((size_t)wg * streams + wave) * cap_hbm * 2;
  return r;
}

// Copy `n` slots of a wave's LDS sub-ring to HBM, 16 bytes per lane (n even or the tail lane copies 8).
__device__ __forceinline__ void wave_copy_slots(const uint32_t* src, uint32_t* dst, uint32_t n) {
  const uint32_t lane = threadIdx.x & 63u;
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
  for (uint32_t i = lane * 2; i < n; i += 128) {
    if (i + 1 < n) {
      *reinterpret_cast<u32x4*>(dst + 2 * i) = *reinterpret_cast<const u32x4*>(src + 2 * i);
    } else {
      *reinterpret_cast<u32x2*>(dst + 2 * i) = *reinterpret_cast<const u32x2*>(src + 2 * i);
    }
  }
}

// Put one record into the wave's LDS sub-ring; in the flush strategy a sub-ring that has just
// filled up is copied to the next chunk of the wave's HBM segment if it still fits.
// The store is seven instructions with no branch: narrow EXEC to lane 0, move the three scalar
// values into VGPRs, one ds_write2_b32, restore EXEC.
__device__ __forceinline__ void store_one(Ring& r, uint32_t tag, uint32_t ts) {
  const uint32_t addr = r.sub_lds + ((tag & r.lds_mask) << 3);  // seq sits in the low tag bits
  uint32_t va, v0, v1;
  if (r.collab) {
    // The paper's store for AMD (Sec. 4.2): every lane writes the same record to the same address,
    // so the execution mask stays as it is.
    asm volatile(
        "v_mov_b32 %0, %3\n\t"
        "v_mov_b32 %1, %4\n\t"
        "v_mov_b32 %2, %5\n\t"
        "ds_write2_b32 %0, %1, %2 offset1:1"
        : "=&v"(va), "=&v"(v0), "=&v"(v1)
        : "s"(addr), "s"(tag), "s"(ts)
        : "memory");
  } else {
    uint64_t saved_exec;
    asm volatile(
        "s_mov_b64 %0, exec\n\t"
        "s_mov_b64 exec, 1\n\t"
        "v_mov_b32 %1, %4\n\t"
        "v_mov_b32 %2, %5\n\t"
        "v_mov_b32 %3, %6\n\t"
        "ds_write2_b32 %1, %2, %3 offset1:1\n\t"
        "s_mov_b64 exec, %0"
        : "=&s"(saved_exec), "=&v"(va), "=&v"(v0), "=&v"(v1)
        : "s"(addr), "s"(tag), "s"(ts)
        : "memory");
  }
  r.stored += 1;
  if (r.flush && (r.stored & r.lds_mask) == 0u) {
    if (r.stored <= r.cap_hbm)
      wave_copy_slots(r.sub, r.seg + (size_t)(r.stored - (r.lds_mask + 1u)) * 2, r.lds_mask + 1u);
  }
}

// The clock is sampled with s_memtime, whose 64-bit result arrives in its SGPR pair some 200
// cycles later and is counted in lgkmcnt together with LDS traffic.  The sample is issued from
// inline assembly so that the compiler's wait-count bookkeeping does not see it: LDS operations
// complete in order, so with one more operation outstanding than the compiler knows of, each of
// its partial waits "lgkmcnt(n)" still guarantees what it was meant to (it may at most wait for
// one LDS operation more), instead of every LDS wait after a sample turning into a wait for the
// clock.  The registers must not be read before the value has landed, so the only consumer is
// clock_delta(): one assembly statement that waits for everything counted in lgkmcnt and then
// subtracts.  It also names the whole pair as an input, which keeps both halves allocated up to
// there (a dead half could be reused right after the sample was issued, and that write-after-write
// hazard stalls the wave at the sample).
// REALTIME selects the metric (the paper's ReadCounterOp carries a MetricType, Sec. 3.1): the shader
// clock (s_memtime, the default) or the constant-rate 100 MHz clock (s_memrealtime).
template <bool REALTIME = false>
__device__ __forceinline__ uint64_t sample_clock() {
  uint64_t t;
  if constexpr (REALTIME) asm volatile("s_memrealtime %0" : "=s"(t));
  else asm volatile("s_memtime %0" : "=s"(t));
  return t;
}
// low 32 bits of (t - t0) for a value returned by sample_clock()
__device__ __forceinline__ uint32_t clock_delta(uint64_t t, uint32_t t0_lo) {
  uint32_t d;
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_sub_u32 %0, %1, %2" : "=s"(d) : "s"((uint32_t)t), "s"(t0_lo), "s"(t) : "scc");
  return d;
}

__device__ __forceinline__ void store_pending(Ring& r) {
  const uint32_t ts = clock_delta(r.pend_t, r.t0_lo);
  if (r.pend_tag != kNoPending) store_one(r, r.pend_tag, ts);
  if (r.pend_tag2 != kNoPending) store_one(r, r.pend_tag2, ts);
  r.pend_tag = kNoPending;
  r.pend_tag2 = kNoPending;
}

// One record site with ONE clock sample: the END of region `end_region` and/or the START of
// region `start_region` (kNoRegion for neither); both are compile-time constants at every site.
// Split as in the paper's ReadCounterOp / StoreCounterOp (Sec. 3.1).  The site first retires the
// records of the previous site (their clock value returned long ago), then samples s_memtime and
// leaves the 64-bit result untouched: lgkmcnt is shared between s_memtime and LDS, so any use
// of a fresh value stalls the wave for the full s_memtime round trip (~200 cycles on gfx950).
// Back-to-back END/START therefore share one sample instead of paying that stall.
template <bool REALTIME = false>
__device__ __forceinline__ void boundary(Ring& r, uint32_t end_region, uint32_t start_region) {
  __builtin_amdgcn_sched_barrier(0);
  store_pending(r);  // also when nothing is pending: the previous sample must have landed before the next
  // the sample goes straight into the register pair its consumer names: no copy of a value in flight
  r.pend_t = sample_clock<REALTIME>();
  const bool on_e = end_region != kNoRegion && ((r.mask >> (end_region & 31u)) & 1u) != 0u;     // scalar
  const bool on_s = start_region != kNoRegion && ((r.mask >> (start_region & 31u)) & 1u) != 0u;
  r.pend_tag = on_e ? ((1u << 31) | (end_region << 24) | r.tag_wave | (r.cnt & 0xFFFFFu)) : kNoPending;
  r.cnt += on_e ? 1u : 0u;
  r.pend_tag2 = on_s ? ((start_region << 24) | r.tag_wave | (r.cnt & 0xFFFFFu)) : kNoPending;
  r.cnt += on_s ? 1u : 0u;
  __builtin_amdgcn_sched_barrier(0);
}

// The same site for the common case "every region enabled, circular strategy", without a branch.
// Every instruction here is paid once per wave and site (a wave issues roughly one instruction
// every four to five cycles and all waves of a workgroup reach their sites together), so the site
// is kept to about twenty instructions:
//   - the two tags of a site are (running counter | compile-time constant); the counter already
//     carries the wave field, which holds as long as a wave writes fewer than 2^20 records (the
//     host only selects these sites when that is certain),
//   - a site always leaves exactly two records pending, so the next site retires two records under
//     one EXEC switch.  The first site of a kernel (START only) and the last (END only) leave the
//     same record twice: both copies go to the same slot with the same contents.  What the very
//     first site retires is the placeholder set up by lean_begin(): it lands in slot 0, which the
//     record with sequence number 0 overwrites one site later.
__device__ __forceinline__ void lean_begin(Ring& r) {
  r.cw = r.tag_wave;
  r.pend_tag = 0u;
  r.pend_tag2 = 0u;
  r.pend_t = r.t_begin;
}

__device__ __forceinline__ void boundary_fast(Ring& r, uint32_t end_region, uint32_t start_region) {
  __builtin_amdgcn_sched_barrier(0);
  {
    const uint32_t ts = clock_delta(r.pend_t, r.t0_lo);
    uint64_t saved_exec;
    uint32_t a0, a1, va, vb, vc, vd, ve;
    asm volatile(
        "s_and_b32 %1, %8, %11\n\t"          // slot = tag & (capacity - 1): seq sits in the low tag bits
        "s_lshl3_add_u32 %1, %1, %12\n\t"    // LDS byte address = sub-ring base + 8 * slot
        "s_and_b32 %2, %10, %11\n\t"
        "s_lshl3_add_u32 %2, %2, %12\n\t"
        "s_mov_b64 %0, exec\n\t"
        "s_mov_b64 exec, 1\n\t"
        "v_mov_b32 %3, %1\n\t"
        "v_mov_b32 %4, %8\n\t"
        "v_mov_b32 %5, %9\n\t"
        "ds_write2_b32 %3, %4, %5 offset1:1\n\t"
        "v_mov_b32 %6, %2\n\t"
        "v_mov_b32 %7, %10\n\t"
        "ds_write2_b32 %6, %7, %5 offset1:1\n\t"
        "s_mov_b64 exec, %0"
        : "=&s"(saved_exec), "=&s"(a0), "=&s"(a1), "=&v"(va), "=&v"(vb), "=&v"(vc), "=&v"(vd), "=&v"(ve)
        : "s"(r.pend_tag), "s"(ts), "s"(r.pend_tag2), "s"(r.lds_mask), "s"(r.sub_lds)
        : "memory", "scc");
  }
  r.pend_t = sample_clock();
  if (end_region != kNoRegion && start_region != kNoRegion) {
    r.pend_tag = r.cw | ((1u << 31) | (end_region << 24));
    r.pend_tag2 = (r.cw + 1u) | (start_region << 24);
    r.cw += 2u;
  } else {
    const uint32_t k = end_region != kNoRegion ? ((1u << 31) | (end_region << 24)) : (start_region << 24);
    r.pend_tag = r.cw | k;
    r.pend_tag2 = r.pend_tag;
    r.cw += 1u;
  }
  __builtin_amdgcn_sched_barrier(0);
}

// Before ring_finish() in a kernel that used the lean sites: hand the record count back.
__device__ __forceinline__ void lean_end(Ring& r) { r.cnt = r.cw - r.tag_wave; }

// A second form, for kernels whose record sites are a fixed sequence known when the kernel is compiled
// (site i closes region e(i) and/or opens region s(i), whatever the data): which records site i writes is
// then a function of i and the region mask alone, so the loop keeps nothing but the clocks.  A site is the
// clock read into one of four scalar register pairs (site_chain<K>, one instruction; no wait, no LDS
// traffic, so it can stand in the middle of pipelined LDS traffic), and chain_commit<N>(), placed where
// the kernel has waited for its LDS traffic anyway, puts the low clock words of sites 0..N-1 of the batch
// into lanes 0..N-1 of one transient vector register and stores them with a single ds_write_b32 into a
// ring of 4-byte entries, one per site: about 14 instructions per commit plus one per site, no vector
// register held across the loop.  The records themselves -- tags, sequence numbers, clock minus workgroup
// start -- are made from that ring when the workgroup copies its trace out (ring_finish with a CHAIN
// functor: end_region(i, n) and start_region(i, n) of site i out of n, kNoRegion for none), exactly those
// the generic sites would have left in the ring: the region mask decides which exist, a wave that does not
// lead its group writes none, and slot = sequence number modulo capacity.
// The clock ring has 2 * capacity entries (the LDS the record ring would take), so it covers the newest
// `capacity` records as long as the enabled records average one per two sites or more, which holds in the
// kernels here for every mask that enables a region.  Whoever uses a clock value has to wait for
// everything counted in lgkmcnt, LDS reads and writes in flight included (scalar-memory results come back
// out of order); the commit is the only place that does.
// Measured: attention kernel (three sites per KV tile) 10 % with the records written at the sites (51
// instructions per tile and wave, whether they took six LDS instructions or two) against 3 %; large GEMM
// with four sites per K step 6-8 % with the sites buffered in vector registers against 3 %.
// Every pair that a site samples into must be read by a later commit on every path: a pair whose value is
// never read is free for the compiler to reuse at once, and the clock would then land in whatever lives there.
// MAY_CROSS: the kinds of instruction the scheduler may move across the site (a sched_barrier mask; 0: none).
// A kernel whose regions are defined by its matrix instructions can let vector, scalar and LDS-read
// instructions cross (0x106) and keep the matrix and memory instructions on their side of the clock read.
template <int K, bool REALTIME = false, int MAY_CROSS = 0>
__device__ __forceinline__ void site_chain(Ring& r) {
  static_assert(K >= 0 && K < 4, "four sites per batch at most");
  __builtin_amdgcn_sched_barrier(MAY_CROSS);
  r.dq_t[K] = sample_clock<REALTIME>();
  __builtin_amdgcn_sched_barrier(MAY_CROSS);
}

template <int N>
__device__ __forceinline__ void chain_commit(Ring& r) {
  static_assert(N >= 1 && N <= 4, "four sites per batch at most");
  // (no scheduling fence: the commit's instructions may sit between the MFMAs around it)
  uint32_t vt = 0u;
#pragma unroll
  for (int k = 0; k < N; ++k) {
    // the wait names the register pair as its output, so nothing can read the pair ahead of it
    uint64_t t = r.dq_t[k];
    if (k == 0) asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(t));
    else asm volatile("" : "+s"(t));
    asm volatile("v_writelane_b32 %0, %1, %2" : "+v"(vt) : "s"((uint32_t)t), "n"(k));
  }
  const uint32_t lane = __builtin_amdgcn_mbcnt_lo(~0u, 0u);  // (the lane index in lanes 0..31, enough for four)
  const uint32_t addr = r.sub_lds + (((r.cw + lane) & r.cmask) << 2);
  uint64_t saved_exec;
  asm volatile(
      "s_mov_b64 %0, exec\n\t"
      "s_mov_b64 exec, %3\n\t"
      "ds_write_b32 %1, %2\n\t"
      "s_mov_b64 exec, %0"
      : "=&s"(saved_exec)
      : "v"(addr), "v"(vt), "n"((1 << N) - 1)
      : "memory");
  r.cw += (uint32_t)N;
}

// r.cw counts sites in this form.  A wave that does not write its group's stream stores its clocks to
// `spare_lds` instead, the LDS byte address of four bytes nobody reads (needed with wave groups only): an
// instruction sequence that is the same for every wave costs less than two more scalar instructions per commit
// (measured on the GEMM with four sites per K step: 3 % against 6 %).
__device__ __forceinline__ void chain_begin(Ring& r, uint32_t spare_lds = 0u) {
  r.cw = 0u;
  r.cmask = 2u * r.lds_mask + 1u;
  if (!r.leader) {  // (uniform)
    r.sub_lds = spare_lds;
    r.cmask = 0u;
  }
}

struct NoChain {};

// Inclusive sum over the lanes of a wave in six data-parallel-primitive adds (shifts inside rows of 16,
// then the last lane of a row into the rows above); every lane must be active.
__device__ __forceinline__ uint32_t wave_inclusive_sum(uint32_t v) {
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xF, 0xF, false);  // row_shr:1
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xF, 0xF, false);  // row_shr:2
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xF, 0xF, false);  // row_shr:4
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xF, 0xF, false);  // row_shr:8
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xA, 0xF, false);  // row_bcast:15
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xC, 0xF, false);  // row_bcast:31
  return v;
}

// The trace segment of this wave from the ring of site clocks, straight to HBM (slot = sequence number
// modulo capacity, as the record sites would have placed them; slots that were never written are
// cleared).  Every lane of the wave takes part.  CHAIN also gives total(n, mask), the records n sites
// leave under a region mask, and kDense, which says that every site but the first and the last both closes and
// opens a region (such a sequence also states kRegions, the number of its regions).
//
// With every region enabled in a dense sequence the record of a slot follows from the slot alone: the
// newest sequence number q in that slot, then site (q + 1) / 2 (behind kLead leading sites without records),
// its END for odd q and its START for even q.
template <class CHAIN>
__device__ __forceinline__ void chain_copy_out_dense(const Ring& r, uint32_t cap_lds, CHAIN chain, uint32_t total) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  const uint32_t lane = threadIdx.x & 63u, n_sites = r.cw;
  for (uint32_t i = lane * 2; i < cap_lds; i += 128) {  // the capacity is a power of two >= 2
    uint32_t w[4];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const uint32_t slot = i + (uint32_t)h;
      uint32_t tag = 0u, ts = 0u;
      if (slot < total) {
        const uint32_t q = total - 1u - ((total - 1u - slot) & r.lds_mask);
        const uint32_t site = ((q + 1u) >> 1) + CHAIN::kLead, end = q & 1u;
        const uint32_t region = end ? chain.end_region(site, n_sites) : chain.start_region(site, n_sites);
        tag = (end << 31) | (region << 24) | r.tag_wave | (q & 0xFFFFFu);
        ts = r.sub[site & r.cmask] - r.t0_lo;
      }
      w[2 * h] = tag; w[2 * h + 1] = ts;
    }
    *reinterpret_cast<u32x4*>(r.seg + 2 * (size_t)i) = u32x4{w[0], w[1], w[2], w[3]};
  }
}

// In general the sites are walked from the last one back, 64 at a time, until the newest `cap_lds` records
// are out: a prefix sum over the lanes says how many records lie behind those of a lane's site.
template <class CHAIN>
__device__ __forceinline__ void chain_copy_out(Ring& r, uint32_t cap_lds, CHAIN chain) {
  typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
  const uint32_t lane = threadIdx.x & 63u, n_sites = r.cw;
  const uint32_t total = chain.total(n_sites, r.mask);
  r.cnt = total;
  if constexpr (CHAIN::kDense) {
    constexpr uint32_t kAll = (1u << CHAIN::kRegions) - 1u;
    if ((r.mask & kAll) == kAll) {  // (uniform)
      chain_copy_out_dense(r, cap_lds, chain, total);
      return;
    }
  }
  for (uint32_t slot = total + lane; slot < cap_lds; slot += 64u)
    *reinterpret_cast<u32x2*>(r.seg + 2 * (size_t)slot) = u32x2{0u, 0u};
  uint32_t covered = 0u;  // records newer than the sites still to come
  for (uint32_t base = n_sites; base > 0u && covered < cap_lds && n_sites - base <= r.cmask; base = base > 64u ? base - 64u : 0u) {
    const bool in = lane < base && n_sites - base + lane <= r.cmask;  // (its clock is still in the ring)
    const uint32_t i = in ? base - 1u - lane : 0u;
    // the regions site i closes and opens, kNoRegion where it does not or the mask says no
    uint32_t e = in ? chain.end_region(i, n_sites) : kNoRegion;
    uint32_t s = in ? chain.start_region(i, n_sites) : kNoRegion;
    if (e != kNoRegion && ((r.mask >> (e & 31u)) & 1u) == 0u) e = kNoRegion;
    if (s != kNoRegion && ((r.mask >> (s & 31u)) & 1u) == 0u) s = kNoRegion;
    const uint32_t n = (e != kNoRegion ? 1u : 0u) + (s != kNoRegion ? 1u : 0u);
    const uint32_t incl = wave_inclusive_sum(n);
    uint32_t newer = covered + incl - n;  // records behind this site's
    const uint32_t ts = r.sub[i & r.cmask] - r.t0_lo;
    if (s != kNoRegion) {  // the START is the later of a site's two records
      if (newer < cap_lds) {
        const uint32_t q = total - 1u - newer;
        *reinterpret_cast<u32x2*>(r.seg + 2 * (size_t)(q & r.lds_mask)) = u32x2{(s << 24) | r.tag_wave | (q & 0xFFFFFu), ts};
      }
      newer += 1u;
    }
    if (e != kNoRegion && newer < cap_lds) {
      const uint32_t q = total - 1u - newer;
      *reinterpret_cast<u32x2*>(r.seg + 2 * (size_t)(q & r.lds_mask)) = u32x2{(1u << 31) | (e << 24) | r.tag_wave | (q & 0xFFFFFu), ts};
    }
    covered += (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
  }
}

// MODE 1: generic (region mask, either strategy, either store); MODE 3: generic, on the constant-rate
// clock; MODE 2: every region enabled, circular strategy, records written to LDS at the next site.
// (Chained sites are placed with site_chain / chain_commit by the kernel itself.)
template <int MODE>
__device__ __forceinline__ void site(Ring& r, uint32_t end_region, uint32_t start_region) {
  static_assert(MODE == 1 || MODE == 2 || MODE == 3, "chained sites are placed with site_chain<K>()");
  if constexpr (MODE == 2) boundary_fast(r, end_region, start_region);
  else boundary<MODE == 3>(r, end_region, start_region);
}
template <int MODE>
__device__ __forceinline__ void sites_begin(Ring& r) {
  if constexpr (MODE == 2) lean_begin(r);
}
template <int MODE>
__device__ __forceinline__ void sites_end(Ring& r) {
  if constexpr (MODE == 2) lean_end(r);
}

template <bool REALTIME = false>
__device__ __forceinline__ void record(Ring& r, uint32_t region, uint32_t phase) {
  boundary<REALTIME>(r, phase == kPhaseEnd ? region : kNoRegion, phase == kPhaseStart ? region : kNoRegion);
}

// After ring_init(): record the constant-rate clock from here on.  Payloads, t_begin and t_end of
// the trace are then in 100 MHz ticks; use record<true>() / ring_finish<true>() with it.
__device__ __forceinline__ void ring_use_realtime(Ring& r) { r.t0_lo = (uint32_t)r.rt_begin; }

// Workgroup epilogue: copy what is still in LDS to HBM and write the headers.
template <bool REALTIME = false, class CHAIN = NoChain>
__device__ __forceinline__ void ring_finish(Ring& r, uint32_t cap_lds, void* trace_buf, TraceGeom g, uint32_t wg,
                                            uint32_t rec_cost, CHAIN chain = CHAIN{}) {
  __syncthreads();  // t_end must not precede any wave's last record
  const uint64_t t_end = __builtin_readcyclecounter();
  const uint64_t rt_end = __builtin_amdgcn_s_memrealtime();
  unsigned char* base = static_cast<unsigned char*>(trace_buf);
  const uint32_t lane = threadIdx.x & 63u;
  kp_wg_hdr* wh = reinterpret_cast<kp_wg_hdr*>(base + sizeof(kp_trace_hdr)) + wg;
  if (r.leader) {  // the wave that wrote the stream also copies it out
    if constexpr (!std::is_same<CHAIN, NoChain>::value) {
      chain_copy_out(r, cap_lds, chain);
    } else {
    store_pending(r);
    if (r.flush) {
      const uint32_t tail = r.cnt & r.lds_mask;           // records not yet copied
      const uint32_t done = r.cnt - tail;
      if (tail && done < r.cap_hbm) {
        const uint32_t room = r.cap_hbm - done;
        wave_copy_slots(r.sub, r.seg + (size_t)done * 2, tail < room ? tail : room);
      }
    } else {
      wave_copy_slots(r.sub, r.seg, cap_lds);  // whole sub-ring; the decoder ignores slots >= total
    }
    }
    if (lane == 0) {
      wh->total_written[r.stream] = r.cnt;
      if (g.flags & KP_FLAG_HW_IDS)
        wh->wave_hw_id[r.stream] = (uint16_t)__builtin_amdgcn_s_getreg((4 << 0) | (0 << 6) | (11 << 11));  // HW_ID, low 12 bits
    }
  }
  if (threadIdx.x == 0) {
    wh->wg_id = wg;
    wh->hw_id = __builtin_amdgcn_s_getreg((4 << 0) | (0 << 6) | (11 << 11));  // HW_ID, low 12 bits
    // the header's span is in the unit of the payloads; `reserved` holds the same span on the other clock
    wh->t_begin = REALTIME ? r.rt_begin : r.t_begin;
    wh->t_end = REALTIME ? rt_end : t_end;
    wh->reserved = REALTIME ? t_end - r.t_begin : rt_end - r.rt_begin;
    for (uint32_t w = g.waves; w < KP_MAX_WAVES; ++w) wh->total_written[w] = 0;
    for (uint32_t w = (g.flags & KP_FLAG_HW_IDS) ? g.waves : 0u; w < KP_MAX_WAVES; ++w) wh->wave_hw_id[w] = 0;
    if (wg == 0) {
      kp_trace_hdr* h = reinterpret_cast<kp_trace_hdr*>(base);
      h->magic = KP_TRACE_MAGIC; h->version = KP_TRACE_VERSION;
      h->n_wg = g.n_wg; h->waves_per_wg = g.waves; h->n_regions = g.n_regions;
      h->cap_wave = g.cap_wave; h->rec_cost = rec_cost; h->flags = g.flags;
      for (int i = 0; i < 8; ++i) h->pad[i] = 0;
    }
  }
}

}  // namespace kp

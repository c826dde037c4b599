/*
 * libkperf -- region-level intra-kernel timing on MI355X (gfx950): C ABI.
 *
 * The library implements the data-parallel hot path of the region-based timing
 * tool of "KPerfIR" (arXiv 2505.21661, Sec. 4): kernels record START/END clock
 * events of marked code regions per wavefront into an LDS ring (Sec. 4.2),
 * copy the ring to a caller-provided trace buffer in HBM before returning
 * (Sec. 4.2 "Global Program Trace"), and a GPU decoder pairs the events into
 * durations and overlap statistics (Sec. 4.3 "Trace Replay", moved onto the
 * GPU).
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller unless the
 *     parameter comment says "host".  The library keeps no device allocation.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Work is enqueued asynchronously; results are valid once the caller has
 *     synchronised the stream.  Exception: kp_trace_reduce (see there).
 *   - Return value: KP_OK or a negative kp_status.  Nothing throws or aborts;
 *     kp_last_error() gives a human-readable reason for the calling thread.
 */
#ifndef KPERF_H
#define KPERF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int kp_status;
enum {
  KP_OK = 0,
  KP_ERR_INVALID_ARG = -1,       /* NULL pointer, negative size, bad flag                      */
  KP_ERR_UNSUPPORTED_SHAPE = -2, /* shape/geometry outside what the kernels are built for      */
  KP_ERR_TRACE_TOO_SMALL = -3,   /* trace_cap not usable (see each call)                       */
  KP_ERR_BAD_TRACE = -4,         /* trace header magic/version/geometry does not match `n`     */
  KP_ERR_HIP = -5                /* a HIP runtime call failed; message holds hipGetErrorString */
};

/* ---- raw trace format (Sec. 4.2: 8-byte records, per-wave slot runs, metadata) ------------
 *
 *   [ kp_trace_hdr : 64 B ][ kp_wg_hdr : 128 B x n_wg ][ records : n_wg x waves x cap_wave x 8 B ]
 *
 * A record is a 4-byte tag followed by a 4-byte payload (Sec. 4.2 "Warp-level Region Data
 * Structure").  The paper fixes one START/END flag bit and leaves the other 31 tag bits to
 * the backend; this library uses
 *   tag[31]    phase: 0 = START, 1 = END
 *   tag[30:24] region id
 *   tag[23:20] wave index inside the workgroup
 *   tag[19:0]  seq: the wave's record counter (mod 2^20) when the record was written
 *   payload    low 32 bits of (s_memtime - t_begin of the workgroup)
 * The segment of (workgroup g, wave w) is the cap_wave slots starting at record index
 * (g*waves + w)*cap_wave.  Circular strategy: a record lives in slot seq mod cap_wave and
 * only the newest cap_wave records of a wave survive (Sec. 4.2 "Shared Memory Circular
 * Buffer").  Flush strategy: slot = seq, records beyond cap_wave are dropped and counted.
 */
#define KP_TRACE_MAGIC 0x4652504Bu /* bytes 'K','P','R','F' */
#define KP_TRACE_VERSION 1u
#define KP_FLAG_FLUSH 1u            /* kp_trace_hdr.flags bit 0: 0 circular, 1 flush */
#define KP_FLAG_REALTIME 2u         /* bit 1: payloads, t_begin and t_end are ticks of the constant-rate 100 MHz clock */
#define KP_FLAG_HW_IDS 4u           /* bit 2: kp_wg_hdr.wave_hw_id[] holds the hardware id of every record stream's wave */
#define KP_MAX_WAVES 16
#define KP_MAX_REGIONS 32           /* regions of the recording kernels and of the decoder's fast path */
#define KP_MAX_TAG_REGIONS 128      /* regions the tag's 7-bit field can name: the decoders' limit */
#define KP_HIST_BINS 64

typedef struct kp_trace_hdr {
  uint32_t magic, version;
  uint32_t n_wg;          /* recorded workgroups                                   */
  uint32_t waves_per_wg;  /* 1..KP_MAX_WAVES                                        */
  uint32_t n_regions;     /* region ids are 0..n_regions-1                          */
  uint32_t cap_wave;      /* slots per wave segment, power of two                   */
  uint32_t rec_cost;      /* ticks subtracted (saturating) from every duration      */
  uint32_t flags;         /* KP_FLAG_*                                              */
  uint32_t pad[8];
} kp_trace_hdr;            /* 64 bytes */

typedef struct kp_wg_hdr {
  uint32_t wg_id;                         /* linear workgroup index                        */
  uint32_t hw_id;                         /* low bits of the hardware id register          */
  uint64_t t_begin;                       /* 64-bit clock at ring init                     */
  uint64_t t_end;                         /* 64-bit clock at flush                         */
  uint64_t reserved;
  uint32_t total_written[KP_MAX_WAVES];   /* records each wave tried to write              */
  uint16_t wave_hw_id[KP_MAX_WAVES];      /* KP_FLAG_HW_IDS: low 12 bits of the hardware id register of the wave
                                             that wrote the stream (wave slot, SIMD, pipe, CU; Sec. 4.2), else 0 */
} kp_wg_hdr;               /* 128 bytes */

/* ---- statistics block written by the decoder ------------------------------------------------
 *
 *   kp_stats_hdr (128 B)
 *   u64 hist[R][64]      log2 duration histogram: bin 0 holds d in {0,1}, bin b holds 2^b <= d < 2^(b+1)
 *   u64 cnt[R], sum[R], min[R], max[R]      (min = UINT64_MAX where cnt = 0)
 *   u64 U[R]             ticks during which region a is active in at least one wave of a workgroup
 *   u64 O[R][R]          ticks during which a and b are both active (O[a][a] = U[a], symmetric)
 *   f64 F[R][R]          O[a][b] / U[a]  (0 where U[a] = 0)
 *   { u64 sum; u32 n; u32 max } per[n_wg][waves][R]
 * with R = n_regions.  All sums are exact integers.
 */
typedef struct kp_stats_hdr {
  uint64_t n_slots_valid;       /* slots that hold a record                                    */
  uint64_t n_pairs;             /* START immediately followed by END of the same (wave,region) */
  uint64_t n_orphan_start;
  uint64_t n_orphan_end;
  uint64_t n_invalid;           /* bad wave/region/seq fields, or displaced by a duplicate seq */
  uint64_t n_dropped;           /* records that did not fit (overwritten or never stored)      */
  uint64_t n_disorder;          /* records found in a slot other than seq mod cap_wave         */
  uint64_t n_span_overflow_wgs; /* workgroups whose t_end - t_begin >= 2^32                    */
  uint64_t n_nonmonotonic;      /* adjacent records of a wave whose clock decreases            */
  uint64_t n_overlap_wgs;       /* workgroups that contributed to U and O                      */
  uint64_t status;              /* 0, or a nonzero code when the device header did not match   */
  uint64_t n_wg, waves_per_wg, n_regions, cap_wave;
  uint64_t reserved;
} kp_stats_hdr;             /* 128 bytes */

typedef struct kp_wave_region_stat {
  uint64_t sum;
  uint32_t n;
  uint32_t max;
} kp_wave_region_stat;      /* 16 bytes */

/* Reason for the most recent failure on the calling thread ("" if none).  Static storage. */
const char* kp_last_error(void);

/* Bytes of a trace buffer for n_wg workgroups of waves_per_wg waves sharing cap_per_wg record
 * slots (cap_per_wg / waves_per_wg slots per wave).  0 on invalid arguments. */
size_t kp_trace_bytes(int n_wg, int waves_per_wg, int cap_per_wg);

/* Bytes of the statistics block.  0 on invalid arguments. */
size_t kp_stats_bytes(int n_wg, int waves_per_wg, int n_regions);

/*
 * Decode, pair and reduce a raw trace (Sec. 4.3: records are stored unpaired and are aligned
 * at replay; the constant record overhead rec_cost is subtracted).
 *
 *   raw        device, the whole trace buffer (headers + records), 16-byte aligned
 *   n          number of record slots = n_wg * waves_per_wg * cap_wave; must match the header
 *   out_stats  device, kp_stats_bytes(...) bytes, 16-byte aligned; fully overwritten
 *
 * kp_trace_reduce reads the 64-byte trace header back from the device to learn the geometry:
 * it synchronises `stream` once before it enqueues the kernels.  kp_trace_reduce_hdr takes
 * the geometry from a HOST copy of the header instead and never synchronises; if the device
 * header disagrees, no statistics are produced and kp_stats_hdr.status is set to 1.
 *
 * Limits: waves_per_wg <= 16, n_regions <= 128, cap_wave a power of two, 2 <= cap_wave <= 2^20.
 * A trace with n_regions <= 32 and waves_per_wg * cap_wave <= 16384 is decoded by a kernel that
 * keeps one workgroup's records in LDS; any other one by a kernel that makes several passes over
 * the records in device memory and keeps one bit per record slot of a workgroup in LDS, next to
 * accumulators whose size grows with n_regions: waves_per_wg * cap_wave <= 2^19 for up to 64
 * regions, <= 2^17 for 128 (KP_ERR_UNSUPPORTED_SHAPE beyond; kp_last_error names the bytes).
 * Header/`n` mismatch, unknown flags, n_regions > 128: KP_ERR_BAD_TRACE.
 */
kp_status kp_trace_reduce(const void* raw, size_t n, void* out_stats, void* stream);
kp_status kp_trace_reduce_hdr(const void* raw, size_t n, const kp_trace_hdr* hdr_host,
                              void* out_stats, void* stream);

/*
 * Timing aid: kp_trace_reduce_hdr that also records two events of the caller's (hipEvent_t handles,
 * created with timing enabled; either may be NULL) on `stream`: main_begin after the kernel that
 * clears the block, right before the kernel that does the replay of Sec. 4.3, main_end right after it,
 * before the kernel that derives O and F from the sums.  Their distance is that one kernel's run time.
 */
kp_status kp_trace_reduce_hdr_events(const void* raw, size_t n, const kp_trace_hdr* hdr_host,
                                     void* out_stats, void* stream, void* main_begin, void* main_end);

/*
 * Timing aid for the decoder: kp_trace_reduce_hdr cut short.  Every recorded workgroup leaves the
 * kernel after step `last_step` of the replay (Sec. 4.3): 1 records ordered by sequence number,
 * 2 paired, durations and histogram accumulated; then the paired records of all waves are sorted
 * by clock: 3 counted into time cells, 4 prefix sum over the cells, 5 placed by cell, 6 ranked
 * inside their cell, 7 sorted sequence written; 8 region-pair overlap swept.  The differences
 * between the run times of consecutive steps are the cost of each step.  out_stats is written but
 * its contents are unspecified.  Only for traces that the LDS-resident kernel takes (n_regions <= 32,
 * waves_per_wg * cap_wave <= 16384); KP_ERR_UNSUPPORTED_SHAPE otherwise.
 */
kp_status kp_trace_reduce_steps(const void* raw, size_t n, const kp_trace_hdr* hdr_host,
                                void* out_stats, int last_step, void* stream);

/*
 * Timeline rows of the same replay.  The paper decodes the profile buffer into one activity
 * struct per timed region instance for timeline front ends such as Chrome Trace (Sec. 3.2) and
 * associates loop iterations with the records (Sec. 3.3 "Iteration-based Timing").  One row per
 * paired START/END, paired exactly as kp_trace_reduce pairs them:
 *   start   payload of the START record: clock ticks since the workgroup began
 *   dur     (u32)(end - start) minus the trace header's rec_cost, not below 0
 *   iter    number of earlier pairs of the same (workgroup, wave, region) among the surviving
 *           records: the loop iteration when the region is recorded once per iteration and the
 *           ring did not wrap
 *   region  region id
 * Output block (device, kp_pairs_bytes(...) bytes, 16-byte aligned):
 *   u32 count[n_wg * waves_per_wg], padded with zeros to a multiple of 4 entries, then
 *   kp_pair_row rows[n_wg * waves_per_wg][cap_wave / 2]; the rows of a wave are ordered by their END
 *   records and only the first count[wg * waves_per_wg + wave] of them are written.
 * Arguments, synchronisation and errors as for kp_trace_reduce / kp_trace_reduce_hdr; a device header
 * that disagrees with hdr_host gives undefined rows.  Limits: n_regions <= 128, and one workgroup's
 * records are staged in LDS: waves_per_wg * cap_wave <= 16384 (KP_ERR_UNSUPPORTED_SHAPE beyond; this
 * kernel has no multi-pass form).
 */
typedef struct {
  uint32_t start;
  uint32_t dur;
  uint32_t iter;
  uint32_t region;
} kp_pair_row;

size_t kp_pairs_bytes(int n_wg, int waves_per_wg, int cap_per_wg);
kp_status kp_trace_pairs(const void* raw, size_t n, void* out_pairs, void* stream);
kp_status kp_trace_pairs_hdr(const void* raw, size_t n, const kp_trace_hdr* hdr_host,
                             void* out_pairs, void* stream);

/* ---- waits behind asynchronous operations ---------------------------------------------------
 *
 * Sec. 4.3 (trace replay, asynchronous instructions): the records around an asynchronous operation
 * are placed as START before its launch (clock CLK0), END right before the barrier that waits for
 * it (CLK1) and START right after that barrier (CLK2); T_wait = CLK2 - CLK1 needs no correction
 * because the records' own cost cancels, and it holds only while what is left of the operation at
 * the barrier outlasts one record (T_MMA - T_exe > T_a + T_b).
 * In the rank order of one (workgroup, wave) -- the order kp_trace_reduce uses -- every END of a
 * region a whose successor is a START (of any region) is one wait of region a:
 *   gap    = (u32)(CLK2 - CLK1)
 *   uncovered if gap <= rec_cost (the trace header's cost of one record)
 *   whole  = (u32)(CLK2 - CLK0) minus rec_cost, not below 0, when the END is paired with a START at
 *            CLK0 (the nearest earlier record of region a in the wave)
 * Output block (device, kp_waits_bytes(...) bytes, 16-byte aligned, fully written), u64 words:
 *   16 header words {n_waits, n_uncovered, n_async, 0 x5, n_wg, waves_per_wg, n_regions, cap_wave,
 *                    rec_cost, 0 x3}
 *   hist[n_regions][64]   gaps by floor(log2 gap), gaps 0 and 1 in bin 0
 *   cnt, sum, min, max    of the gaps per region (min is all ones when cnt is 0)
 *   uncovered, async_cnt, async_sum   per region (async_sum adds up `whole`)
 *   per[n_wg][waves_per_wg][n_regions] of 16 bytes {u64 sum, u32 n, u32 max} of the gaps
 * Arguments, synchronisation, limits (n_regions <= 128) and errors as for kp_trace_pairs /
 * kp_trace_pairs_hdr; KP_ERR_UNSUPPORTED_SHAPE also when waves, cap_wave and n_regions together
 * exceed the kernel's LDS budget.  One wave may hold at most 2^18 waits.
 */
size_t kp_waits_bytes(int n_wg, int waves_per_wg, int n_regions);
kp_status kp_trace_waits(const void* raw, size_t n, void* out_waits, void* stream);
kp_status kp_trace_waits_hdr(const void* raw, size_t n, const kp_trace_hdr* hdr_host,
                             void* out_waits, void* stream);

/* ---- stage latencies per loop iteration ----------------------------------------------------
 *
 * The paper's critical-path analysis and its overlap models (Sec. 3.3 "Critical-path Analysis";
 * Sec. 5.2 "Performance Modeling for GPU Overlapping", Table 4) work on the latency of every stage
 * (region) in every loop iteration.  A stage that the waves of a workgroup execute together lasts
 * as long as its slowest wave: kp_pairs_stages folds the timeline rows that kp_trace_pairs wrote
 * for the waves of a workgroup into one entry per (workgroup, region, iteration),
 *   max_dur    max over the rows of dur
 *   min_start  min over the rows of start
 *   max_end    max over the rows of (u32)(start + dur)
 *   n_waves    number of rows folded in (one per wave that ran this iteration of the region)
 * An entry without rows reads {0, 0xFFFFFFFF, 0, 0}.
 *   pairs        device, the block kp_trace_pairs / kp_trace_pairs_hdr wrote for (n_wg, waves_per_wg,
 *                cap_per_wg); every count must be <= cap_wave / 2; read only
 *   n_regions    rows whose region is not below it are left out and counted (n_bad_region)
 *   max_iter     iterations kept per region; rows with iter >= max_iter are left out and counted
 *   out_stages   device, kp_stages_bytes(n_wg, n_regions, max_iter) bytes, 16-byte aligned, fully
 *                written: 4 u64 {n_rows folded, n_clipped, n_bad_region, 0}, then
 *                kp_stage_row table[n_wg][n_regions][max_iter]
 * Asynchronous on `stream`.  KP_ERR_INVALID_ARG for NULL or misaligned pointers and bad sizes;
 * KP_ERR_UNSUPPORTED_SHAPE when n_regions * (max_iter + 1) * 16 exceeds 64 KiB (the table of one
 * workgroup lives in LDS).
 */
typedef struct {
  uint32_t max_dur;
  uint32_t min_start;
  uint32_t max_end;
  uint32_t n_waves;
} kp_stage_row;

size_t kp_stages_bytes(int n_wg, int n_regions, int max_iter);
kp_status kp_pairs_stages(const void* pairs, int n_wg, int waves_per_wg, int cap_per_wg, int n_regions,
                          int max_iter, void* out_stages, void* stream);

/* ---- critical path over the stage table ------------------------------------------------------
 *
 * The paper reads the critical path of a kernel whose warp groups work on different stages off its
 * timeline: a chain of stages, each of which could only start when the one before it had finished
 * (Sec. 3.3 "Critical-path Analysis"; Sec. 5.2), and models the latency of such a kernel as the sum
 * of the latencies of the stages on that path (Table 4, WS model).  kp_stages_critical takes the
 * chain of every recorded workgroup from its stage table (entries with n_waves = 0 are no stages):
 *   the stages are ordered by (max_end, region * max_iter + iteration);
 *   the path ends in the last stage of that order;
 *   the stage before a stage X of the path is the latest stage of that order, earlier than X, with
 *   max_end <= X.min_start (the one X waited for); without one, X is the first stage of the path.
 * Clocks are compared as plain 32-bit unsigned numbers.
 *   stages      device, the block kp_pairs_stages wrote for (n_wg, n_regions, max_iter); read only
 *   out_paths   device, kp_critical_bytes(n_wg, n_regions) bytes, 16-byte aligned, fully written:
 *               8 u64 {n_wg, n_regions, max_iter, workgroups with a path, stages on all paths, sum of
 *               their latencies (max_dur), sum of all bubbles, 0}; per region 2 u64 {stages on paths,
 *               their latencies}; kp_path_row rows[n_wg]
 * Asynchronous on `stream`.  KP_ERR_INVALID_ARG for NULL or misaligned pointers and bad sizes;
 * KP_ERR_UNSUPPORTED_SHAPE when n_regions * max_iter exceeds 4096 (the stages of one workgroup are
 * sorted in LDS).
 */
typedef struct {
  uint32_t n_stages;     /* stages on the path                                                        */
  uint32_t last_stage;   /* region << 16 | iteration of the stage that ends last; all ones: no stage  */
  uint32_t first_start;  /* min_start of the first stage of the path                                  */
  uint32_t last_end;     /* max_end of the last                                                       */
  uint64_t sum_latency;  /* sum of max_dur over the path                                              */
  uint64_t bubbles;      /* ticks between the end of a stage of the path and the start of the next    */
} kp_path_row;

size_t kp_critical_bytes(int n_wg, int n_regions);
kp_status kp_stages_critical(const void* stages, int n_wg, int n_regions, int max_iter, void* out_paths,
                             void* stream);

/* ---- instrumented targets ---------------------------------------------------------------------
 *
 * region_mask: bit r (r < 26) enables the record sites of region r; bit 31 (KP_MASK_FLUSH)
 * selects the flush strategy instead of the default circular one (Sec. 4.2: "Circular" keeps
 * the newest records in LDS and copies them out once at kernel exit; "Flush" writes a full
 * LDS sub-ring back to HBM whenever it fills up).  region_mask with bits 0..26 all zero
 * launches the separately compiled uninstrumented kernel: no ring, no record sites; trace_buf
 * may then be NULL.  Instrumented and uninstrumented kernels produce bit-identical outputs.
 *
 * Bit 30 (KP_MASK_WAVE_GROUP) selects the granularity of the records (Sec. 3.1: the Granularity
 * option of the lowering; Sec. 4.2: one profiling space per warp group): 0 one record stream per
 * wave, 1 one per group of four consecutive waves, written by the first wave of the group on
 * behalf of all four.  The trace then describes waves / 4 "waves" per workgroup (its
 * waves_per_wg, the tag's wave field and total_written[] count streams), and every size below
 * that speaks of waves speaks of streams.
 *
 * Bit 28 (KP_MASK_REALTIME) selects the metric of the records (Sec. 3.1: the MetricType of the
 * counter read): 0 the shader clock, 1 the constant-rate 100 MHz clock; the trace then carries
 * KP_FLAG_REALTIME, its payloads and the headers' t_begin / t_end are in that clock's ticks and
 * kp_wg_hdr.reserved holds the span on the shader clock.
 *
 * Bit 27 (KP_MASK_COLLAB) selects the store of Sec. 4.2 ("AMD"): all 64 lanes of the wave write the
 * record to the same LDS address instead of one lane under a narrowed execution mask, and every
 * stream's wave leaves the low 12 bits of its hardware id register in kp_wg_hdr.wave_hw_id[]
 * (KP_FLAG_HW_IDS).  The records themselves are the same either way.
 * Bit 27 and the flush strategy go through the generic record sites (a site writes the records of the
 * site before it to LDS); in the 256x256x64 GEMM and the attention kernel every other combination keeps
 * the cheaper chained sites (the loop stores only the clocks of its sites, a fixed sequence, and the
 * records are made from them when the trace is copied out: the same records in the same slots), in the
 * small GEMM bits 28 and 30 and a partial region mask take the generic sites too.
 *
 * trace_buf: device, kp_trace_bytes(n_wg, streams, trace_cap) bytes, 16-byte aligned; headers and
 * records are fully written by the kernel (no pre-zeroing needed; slots beyond total_written
 * hold unspecified bytes).  trace_cap: record slots per workgroup in HBM; trace_cap / streams must
 * be a power of two >= 2, else KP_ERR_TRACE_TOO_SMALL.  Circular: the whole ring also lives in
 * LDS (KP_ERR_UNSUPPORTED_SHAPE if it exceeds the kernel's LDS budget: 32 KiB, of which wave-group
 * records take 16 bytes for themselves).
 */
#define KP_MASK_FLUSH 0x80000000u
#define KP_MASK_WAVE_GROUP 0x40000000u
#define KP_MASK_PHASES 0x20000000u
#define KP_MASK_REALTIME 0x10000000u
#define KP_MASK_COLLAB 0x08000000u
#define KP_MASK_UNFENCED 0x04000000u

/* Launch geometry kp_gemm_instrumented will use for M x N x K: recorded workgroups, waves per
 * workgroup, number of regions.  KP_ERR_UNSUPPORTED_SHAPE if no kernel covers the shape. */
kp_status kp_gemm_launch_shape(int M, int N, int K, int* n_wg, int* waves_per_wg, int* n_regions);

/*
 * C[M,N] = A[M,K] * B[K,N]; bf16 inputs, fp32 accumulation on MFMA, bf16 (round to nearest even)
 * output; all three row-major, device memory, 16-byte aligned.  The paper instruments
 * software-pipelined GEMMs stage by stage (Sec. 5.3 "Profiling Overhead", GEMM-SWP-2/3); the
 * regions here are
 *   M, N multiples of 256 with at least 16 tiles, K a multiple of 64: tile 256x256x64, 8 waves,
 *       per K-step, in this order: 0 the first sixteen MFMAs issued in the K-step's turn of the loop (the last
 *       eight of the K-step before, whose operands were read ahead of the barrier, and the first eight of
 *       this one), with the eight loads that send the next K-step's tiles from global memory straight to the
 *       other LDS stage threaded between them; 1 the other sixteen and the wait for those loads and for this
 *       wave's LDS reads; 2 barrier; 3 epilogue, once (it starts with the last eight MFMAs)
 *       With bit 29 of region_mask (KP_MASK_PHASES; this tile only, KP_ERR_INVALID_ARG otherwise) the
 *       stages of a K-step follow one another instead of being threaded into each other, and each is a
 *       region (5 regions, kp_trace_hdr.n_regions = 5; 4 sites and 8 records per K-step and wave):
 *       2 LDS write (the staging registers of the next K-step go to the other LDS stage), 0 global load
 *       issue (for the K-step after that), 3 MFMA, 1 wait (LDS traffic landed + barrier); 4 epilogue,
 *       once.  KP_MASK_PHASES with bits 0..4 all zero runs that schedule without record sites: a record
 *       site keeps its place in the instruction stream, so where the instrumented kernel has a site
 *       this one has a bare scheduling fence and the stages stay apart; with bit 26 (KP_MASK_UNFENCED)
 *       as well the fences are left out and the compiler threads the stages as it likes (for the
 *       comparison of the two; KP_ERR_INVALID_ARG with any region bit or without KP_MASK_PHASES).
 *   otherwise M, N multiples of 64 and K of 32: tile 64x64x32, 4 waves,
 *       0 global load, 1 LDS store, 2 MFMA (each once per K-step)
 * Other shapes: KP_ERR_UNSUPPORTED_SHAPE.
 */
kp_status kp_gemm_instrumented(const void* A, const void* B, void* C, int M, int N, int K,
                               uint32_t region_mask, void* trace_buf, size_t trace_cap, void* stream);

/* Launch geometry of kp_attn_instrumented: B*H*(S/128) workgroups of 4 waves, 3 regions. */
kp_status kp_attn_launch_shape(int B, int H, int S, int D, int* n_wg, int* waves_per_wg, int* n_regions);

/*
 * Attention forward O = softmax(scale * Q K^T + mask) V per (batch, head); Q, K, V, O are
 * [B, H, S, D] contiguous bf16 in device memory, 16-byte aligned; softmax and accumulation in
 * fp32; causal != 0 masks key j > query i.  D must be 128 and S a multiple of 128
 * (KP_ERR_UNSUPPORTED_SHAPE otherwise); scale must be positive and finite.
 * The paper's flash-attention study times the two GEMMs and the softmax of every KV iteration
 * (Sec. 5.2, Table 3); the regions here, once per KV tile of 64 keys, are
 *   0 Q K^T (MFMA), 1 online softmax, 2 P V (MFMA);
 * END of region 2 and START of region 0 of the next tile share one clock sample.  The samples that
 * close regions 0 and 2 are taken right behind the workgroup barrier that follows the region's work, so
 * the wait at that barrier belongs to the region that ends there (it also waits for the tile that the next
 * region reads: the K and V tiles go from global memory straight to LDS, each requested one barrier ahead
 * of its use -- the next K tile at the head of region 1, the next V tile at the head of region 0).
 * One workgroup (4 waves) handles 128 query rows; with causal masking block q records
 * 6 * 2 * (q + 1) times per wave.  region_mask, trace_buf, trace_cap as for the GEMM.
 */
kp_status kp_attn_instrumented(const void* Q, const void* K, const void* V, void* O, int B, int H, int S,
                               int D, int causal, float scale, uint32_t region_mask, void* trace_buf,
                               size_t trace_cap, void* stream);

/*
 * Timer calibration (Sec. 5.4 "Cycle-level Overhead": cost of one record; Sec. 4.3: that
 * constant is subtracted at replay).  Launches n_wg workgroups of `waves` waves, one workgroup
 * per CU at a time; every wave runs regions 0..n_regions-1 back to back, region r being
 *   mode bit0 = 0: cycles[r]/4 dependent v_fma_f32 (rounded down to a multiple of 16 FMAs)
 *   mode bit0 = 1: cycles[r]/64 executions of s_sleep 1
 * bracketed by a START and an END record; cycles[r] = 0 gives an empty region whose duration is
 * the cost of one record.  mode bit1 selects the flush strategy with an 8-slot LDS sub-ring.
 * mode bit2 selects the metric the records carry (the MetricType of the paper's ReadCounterOp,
 * Sec. 3.1): 0 the shader clock (s_memtime), 1 the constant-rate 100 MHz clock (s_memrealtime); the
 * payloads and the workgroup header's t_begin / t_end are in that clock's ticks, and the header's
 * reserved word holds the same span on the other clock.  mode bit3 selects wave-group granularity
 * as KP_MASK_WAVE_GROUP does (waves must then be a multiple of 4; the trace holds waves / 4 streams).
 * mode bits 4 and 5 select the form of the record sites, which the instrumented kernels also choose
 * among and which decides the constant a region is measured too long by: neither bit the generic sites
 * (region mask, either strategy, either clock, either store), bit 4 the lean sites (all regions, circular
 * strategy: the small GEMM), bit 5 the chained sites of the 256x256x64 GEMM and the attention kernel (the
 * loop keeps only the clocks of the sites, the records are made when the trace is copied out); with
 * either bit, bits 1..3 and 6 must be 0 (KP_ERR_INVALID_ARG otherwise).  mode bit6 selects the
 * store of KP_MASK_COLLAB (all lanes write the record; hardware ids in the workgroup header).
 *   cycles     HOST pointer to n_regions values (n_regions <= 32)
 *   trace_buf  device, kp_trace_bytes(n_wg, streams, trace_cap) bytes; trace_cap as above
 */
kp_status kp_calibrate(const uint32_t* cycles, int n_regions, int n_wg, int waves, int mode,
                       void* trace_buf, size_t trace_cap, void* stream);

/*
 * The constant that replay takes off every measured duration (Sec. 4.3: the record's own cost is
 * taken out as one constant per record; Sec. 5.4 measures it).  A region is measured from the clock
 * read of its START site to the clock read of its END site, which includes the instructions of the
 * sites themselves: an empty region of kp_calibrate reads exactly that constant.  Every trace recorded
 * after kp_set_rec_cost(ticks) carries `ticks` in kp_trace_hdr.rec_cost (process-wide, default 0; the
 * value is read when a recording call is made, not when its kernel runs).
 */
void kp_set_rec_cost(uint32_t ticks);
uint32_t kp_get_rec_cost(void);

#ifdef __cplusplus
}
#endif
#endif /* KPERF_H */

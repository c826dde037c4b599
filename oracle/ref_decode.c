/*
 * CPU oracle for the trace decode/reduce step  --  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, obviously-correct reference that the GPU decoder is compared
 * against bit for bit.  It shares no code, headers, tables or helpers with the
 * HIP library; only tests, the smoke check and the benchmark's cpu_baseline leg
 * may call it.  It re-declares the byte layouts it reads and writes.
 *
 * What the paper fixes (Sec. 4.2 "Profile Data Management", Sec. 4.3 "Trace
 * Replay"):
 *   - a record is 8 bytes: a 4-byte tag whose one flag bit says START or END,
 *     and a 4-byte payload holding the low 32 bits of the clock;
 *   - every warp(-group) owns a private run of slots inside the block's buffer;
 *   - START/END records are stored interleaved and unpaired; pairing happens at
 *     replay; the patterns to support are common, nested and multi-iteration;
 *   - the circular strategy keeps only the tail of each trace;
 *   - metadata carries block index, per-warp indices and recorded-slot counts;
 *   - 32-bit clocks are valid while an interval stays below 2^32 ticks;
 *     overflow is detected at post-processing;
 *   - replay subtracts a constant per-record measuring overhead.
 * Everything else (tag bit positions, sequence numbers, statistics) is this
 * project's reading and is stated step by step below.
 *
 * Raw trace (little endian):
 *   [0,64)    trace header: u32 magic 'KPRF', version(1), n_wg, waves (<=16),
 *             n_regions (<=128), cap_wave (power of two), rec_cost, flags
 *             (bit0: 0 circular, 1 flush), zero padding
 *   then n_wg workgroup headers of 128 B:
 *             u32 wg_id, u32 hw_id, u64 t_begin, u64 t_end, u64 reserved,
 *             u32 total_written[16], zero padding
 *   then records, segment of (wg, w) = cap_wave consecutive 8-byte slots at
 *             index (wg*waves + w)*cap_wave
 *   record:   u32 tag, u32 payload
 *             tag[31] phase (0 START, 1 END); tag[30:24] region; tag[23:20]
 *             wave; tag[19:0] seq = per-wave record counter mod 2^20
 *             payload = low 32 bits of (clock - t_begin)
 *
 * Stats block:
 *   16 x u64 header: n_slots_valid, n_pairs, n_orphan_start, n_orphan_end,
 *       n_invalid, n_dropped, n_disorder, n_span_overflow_wgs, n_nonmonotonic,
 *       n_overlap_wgs, status, n_wg, waves, n_regions, cap_wave, reserved
 *   u64 hist[R][64]; u64 cnt[R], sum[R], min[R], max[R]; u64 U[R];
 *   u64 O[R][R]; double F[R][R];
 *   per[n_wg][waves][R] of { u64 sum; u32 n; u32 max }
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define KPO_HDR_BYTES 64u
#define KPO_WGHDR_BYTES 128u
#define KPO_MAGIC 0x4652504Bu
#define KPO_SEQ_BITS 20u
#define KPO_SEQ_MASK ((1u << KPO_SEQ_BITS) - 1u)

size_t kpo_stats_bytes(uint32_t n_wg, uint32_t waves, uint32_t R) {
  return (size_t)128 + (size_t)8 * (64u * R + 5u * R + 2u * (size_t)R * R) +
         (size_t)16 * n_wg * waves * R;
}

typedef struct { uint64_t t; int32_t delta; uint32_t region; } kpo_event;

static int kpo_event_cmp(const void* a, const void* b) {
  const kpo_event* x = (const kpo_event*)a;
  const kpo_event* y = (const kpo_event*)b;
  if (x->t != y->t) return x->t < y->t ? -1 : 1;
  /* ends before starts at equal time; any order gives the same measure */
  return x->delta - y->delta;
}

typedef struct {
  uint64_t hdr[16];
  uint64_t* hist; uint64_t* cnt; uint64_t* sum; uint64_t* min; uint64_t* max;
  uint64_t* U; uint64_t* O;
} kpo_acc;

static int kpo_acc_init(kpo_acc* a, uint32_t R) {
  memset(a->hdr, 0, sizeof a->hdr);
  a->hist = (uint64_t*)calloc((size_t)64 * R, 8);
  a->cnt = (uint64_t*)calloc(R, 8); a->sum = (uint64_t*)calloc(R, 8);
  a->min = (uint64_t*)malloc((size_t)R * 8); a->max = (uint64_t*)calloc(R, 8);
  a->U = (uint64_t*)calloc(R, 8); a->O = (uint64_t*)calloc((size_t)R * R, 8);
  if (!a->hist || !a->cnt || !a->sum || !a->min || !a->max || !a->U || !a->O) return -1;
  for (uint32_t r = 0; r < R; ++r) a->min[r] = UINT64_MAX;
  return 0;
}
static void kpo_acc_free(kpo_acc* a) {
  free(a->hist); free(a->cnt); free(a->sum); free(a->min); free(a->max); free(a->U); free(a->O);
}

enum { H_SLOTS_VALID = 0, H_PAIRS, H_ORPHAN_START, H_ORPHAN_END, H_INVALID, H_DROPPED,
       H_DISORDER, H_SPAN_OVF, H_NONMONO, H_OVERLAP_WGS, H_STATUS, H_NWG, H_WAVES, H_NREG,
       H_CAP, H_RSVD };

/* floor(log2 d) with d in {0,1} both mapping to bin 0 */
static uint32_t kpo_bin(uint64_t d) {
  uint32_t b = 0;
  while (d > 1) { d >>= 1; ++b; }
  return b;
}

/* Decode one workgroup.  `per` points at this workgroup's [waves][R] block. */
static void kpo_decode_wg(const uint32_t* wh, const uint32_t* recs, uint32_t W, uint32_t R,
                          uint32_t cap, uint32_t rec_cost, int flush, kpo_acc* acc,
                          uint8_t* per, int32_t* slot_of_rank, uint32_t* seq_tag,
                          uint32_t* seq_ts, kpo_event* events) {
  uint64_t t_begin, t_end;
  memcpy(&t_begin, wh + 2, 8);
  memcpy(&t_end, wh + 4, 8);
  const uint64_t span = t_end - t_begin;
  uint64_t wg_invalid = 0, wg_nonmono = 0;
  size_t n_events = 0;

  for (uint32_t w = 0; w < W; ++w) {
    const uint32_t* seg = recs + (size_t)2 * w * cap;
    /* step 1: how many slots hold data, how many records were lost */
    const uint32_t T = wh[8 + w];
    const uint32_t V = T < cap ? T : cap;
    acc->hdr[H_DROPPED] += T - V;
    acc->hdr[H_SLOTS_VALID] += V;
    /* the circular strategy keeps the last V records, the flush strategy the first V */
    const uint32_t first_seq = flush ? 0u : T - V;

    /* step 2: order by sequence number; a later slot displaces an earlier one */
    for (uint32_t k = 0; k < V; ++k) slot_of_rank[k] = -1;
    for (uint32_t s = 0; s < V; ++s) {
      const uint32_t tag = seg[2 * s];
      const uint32_t seq = tag & KPO_SEQ_MASK;
      const uint32_t wave = (tag >> 20) & 0xFu;
      const uint32_t region = (tag >> 24) & 0x7Fu;
      const uint32_t k = (seq - first_seq) & KPO_SEQ_MASK;
      if (k >= V || wave != w || region >= R) { ++wg_invalid; continue; }
      if (slot_of_rank[k] >= 0) ++wg_invalid; /* the displaced record */
      slot_of_rank[k] = (int32_t)s;
    }
    uint32_t n = 0; /* length of the ordered sequence S_w */
    for (uint32_t k = 0; k < V; ++k) {
      if (slot_of_rank[k] < 0) continue;
      const uint32_t s = (uint32_t)slot_of_rank[k];
      const uint32_t tag = seg[2 * s];
      if (s != ((tag & KPO_SEQ_MASK) & (cap - 1))) acc->hdr[H_DISORDER] += 1;
      seq_tag[n] = tag; seq_ts[n] = seg[2 * s + 1]; ++n;
    }
    /* step 3: per-wave clock monotonicity (unsigned compare of adjacent payloads) */
    for (uint32_t i = 0; i + 1 < n; ++i)
      if (seq_ts[i + 1] < seq_ts[i]) ++wg_nonmono;

    /* steps 4-7: pair inside each region's subsequence, durations, statistics */
    for (uint32_t r = 0; r < R; ++r) {
      uint64_t p_sum = 0; uint32_t p_n = 0, p_max = 0;
      int have_prev = 0; uint32_t prev_phase = 0, prev_ts = 0;
      for (uint32_t i = 0; i < n; ++i) {
        if (((seq_tag[i] >> 24) & 0x7Fu) != r) continue;
        const uint32_t phase = seq_tag[i] >> 31;
        if (phase == 0) { /* START */
          if (have_prev && prev_phase == 0) acc->hdr[H_ORPHAN_START] += 1; /* START START */
        } else {          /* END */
          if (have_prev && prev_phase == 0) {
            const uint32_t d_raw = seq_ts[i] - prev_ts;           /* mod 2^32 */
            const uint32_t d = d_raw > rec_cost ? d_raw - rec_cost : 0u;
            acc->hdr[H_PAIRS] += 1;
            p_sum += d; p_n += 1; if (d > p_max) p_max = d;
            acc->hist[(size_t)r * 64 + kpo_bin(d)] += 1;
            acc->cnt[r] += 1; acc->sum[r] += d;
            if (d < acc->min[r]) acc->min[r] = d;
            if (d > acc->max[r]) acc->max[r] = d;
            events[n_events].t = prev_ts; events[n_events].delta = +1; events[n_events].region = r; ++n_events;
            events[n_events].t = (uint64_t)prev_ts + d_raw; events[n_events].delta = -1; events[n_events].region = r; ++n_events;
          } else {
            acc->hdr[H_ORPHAN_END] += 1;
          }
        }
        have_prev = 1; prev_phase = phase; prev_ts = seq_ts[i];
      }
      if (have_prev && prev_phase == 0) acc->hdr[H_ORPHAN_START] += 1; /* START at end of sequence */
      uint8_t* e = per + (size_t)16 * ((size_t)w * R + r);
      memcpy(e, &p_sum, 8); memcpy(e + 8, &p_n, 4); memcpy(e + 12, &p_max, 4);
    }
  }
  acc->hdr[H_INVALID] += wg_invalid;
  acc->hdr[H_NONMONO] += wg_nonmono;

  /* step 8: overlap, only for workgroups with a trustworthy timeline */
  const int span_overflow = span >= (1ull << 32);
  if (span_overflow) acc->hdr[H_SPAN_OVF] += 1;
  if (span_overflow || wg_invalid || wg_nonmono) return;
  acc->hdr[H_OVERLAP_WGS] += 1;
  qsort(events, n_events, sizeof(kpo_event), kpo_event_cmp);
  int32_t active[128];
  memset(active, 0, sizeof active);
  uint64_t prev_t = 0;
  for (size_t i = 0; i < n_events; ++i) {
    const uint64_t dt = events[i].t - prev_t;
    if (dt) {
      for (uint32_t a = 0; a < R; ++a) {
        if (active[a] <= 0) continue;
        acc->U[a] += dt;
        for (uint32_t b = 0; b < R; ++b)
          if (active[b] > 0) acc->O[(size_t)a * R + b] += dt;
      }
    }
    active[events[i].region] += events[i].delta;
    prev_t = events[i].t;
  }
}

/* Returns 0, or <0 when the header is not a valid trace of n_slots records. */
int kpo_decode(const void* raw, size_t n_slots, void* out, size_t out_bytes, int n_threads) {
  const uint32_t* hdr = (const uint32_t*)raw;
  if (!raw || !out) return -1;
  if (hdr[0] != KPO_MAGIC || hdr[1] != 1u) return -4;
  const uint32_t n_wg = hdr[2], W = hdr[3], R = hdr[4], cap = hdr[5], rec_cost = hdr[6];
  const int flush = (int)(hdr[7] & 1u);
  if (W == 0 || W > 16 || R == 0 || R > 128 || cap == 0 || (cap & (cap - 1)) || cap > (1u << 19)) return -4;
  if ((size_t)n_wg * W * cap != n_slots) return -4;
  if (out_bytes < kpo_stats_bytes(n_wg, W, R)) return -3;

  uint8_t* o = (uint8_t*)out;
  memset(o, 0, kpo_stats_bytes(n_wg, W, R));
  uint64_t* ohdr = (uint64_t*)o;
  uint64_t* ohist = ohdr + 16;
  uint64_t* ocnt = ohist + (size_t)64 * R;
  uint64_t* osum = ocnt + R; uint64_t* omin = osum + R; uint64_t* omax = omin + R;
  uint64_t* oU = omax + R; uint64_t* oO = oU + R;
  double* oF = (double*)(oO + (size_t)R * R);
  uint8_t* oper = (uint8_t*)(oF + (size_t)R * R);
  for (uint32_t r = 0; r < R; ++r) omin[r] = UINT64_MAX;

  const uint8_t* base = (const uint8_t*)raw;
  const uint32_t* wg_hdrs = (const uint32_t*)(base + KPO_HDR_BYTES);
  const uint32_t* records = (const uint32_t*)(base + KPO_HDR_BYTES + (size_t)KPO_WGHDR_BYTES * n_wg);
  int failed = 0;
  (void)n_threads;
#ifdef _OPENMP
#pragma omp parallel num_threads(n_threads > 0 ? n_threads : 1)
#endif
  {
    kpo_acc acc;
    int32_t* slot_of_rank = (int32_t*)malloc((size_t)cap * 4);
    uint32_t* seq_tag = (uint32_t*)malloc((size_t)cap * 4);
    uint32_t* seq_ts = (uint32_t*)malloc((size_t)cap * 4);
    kpo_event* events = (kpo_event*)malloc((size_t)W * cap * sizeof(kpo_event) + sizeof(kpo_event));
    int ok = kpo_acc_init(&acc, R) == 0 && slot_of_rank && seq_tag && seq_ts && events;
    if (!ok) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
      failed = 1;
    }
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 4)
#endif
    for (int64_t wg = 0; wg < (int64_t)n_wg; ++wg) {
      if (!ok) continue;
      kpo_decode_wg(wg_hdrs + (size_t)32 * wg, records + (size_t)2 * wg * W * cap, W, R, cap,
                    rec_cost, flush, &acc, oper + (size_t)16 * wg * W * R, slot_of_rank,
                    seq_tag, seq_ts, events);
    }
    if (ok) {
#ifdef _OPENMP
#pragma omp critical
#endif
      {
        for (int i = 0; i < 16; ++i) ohdr[i] += acc.hdr[i];
        for (size_t i = 0; i < (size_t)64 * R; ++i) ohist[i] += acc.hist[i];
        for (uint32_t r = 0; r < R; ++r) {
          ocnt[r] += acc.cnt[r]; osum[r] += acc.sum[r];
          if (acc.min[r] < omin[r]) omin[r] = acc.min[r];
          if (acc.max[r] > omax[r]) omax[r] = acc.max[r];
          oU[r] += acc.U[r];
        }
        for (size_t i = 0; i < (size_t)R * R; ++i) oO[i] += acc.O[i];
      }
    }
    kpo_acc_free(&acc);
    free(slot_of_rank); free(seq_tag); free(seq_ts); free(events);
  }
  if (failed) return -5;
  /* step 9: overlap fractions, one IEEE division of exactly converted integers */
  for (uint32_t a = 0; a < R; ++a)
    for (uint32_t b = 0; b < R; ++b)
      oF[(size_t)a * R + b] = oU[a] ? (double)oO[(size_t)a * R + b] / (double)oU[a] : 0.0;
  ohdr[H_STATUS] = 0; ohdr[H_NWG] = n_wg; ohdr[H_WAVES] = W; ohdr[H_NREG] = R; ohdr[H_CAP] = cap;
  return 0;
}

/*
 * Seeded synthetic raw-trace generator (test/bench input only).
 *
 * Produces a raw trace buffer in the on-disk/in-HBM trace format consumed by
 * the decoder: a 64-byte trace header, one 128-byte header per recorded
 * workgroup, then n_wg x waves x cap_wave 8-byte records (4-byte tag + 4-byte
 * 32-bit timestamp payload; the record size and tag/payload split follow the
 * paper's "Warp-level Region Data Structure" paragraph, Sec. 4.2).
 *
 * This file holds none of the decoder's arithmetic: it only draws region
 * instances (start time, duration, gap) from a counter-based RNG and encodes
 * them.  Neither the CPU oracle nor the HIP library includes or links it.
 *
 * Per wave: region ids cycle 0..R-1; each instance emits a START record at t
 * and (unless it is a start-only instance) an END record at t+d; then a gap.
 * Circular strategy keeps the last cap_wave records of a wave in slot
 * (seq mod cap_wave) (Sec. 4.2 "Shared Memory Circular Buffer": only the tail
 * of the trace survives); flush strategy keeps the first cap_wave records.
 * Afterwards a small fraction of slots is swapped with a nearby later slot to
 * model out-of-order flushes.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
  uint64_t seed;
  uint32_t n_wg;
  uint32_t waves;
  uint32_t n_regions;
  uint32_t cap_wave;        /* power of two */
  uint32_t total_per_wave;  /* records emitted per wave before any drop */
  uint32_t total_var;       /* per-wave total is reduced by U{0..total_var} */
  uint32_t dist;            /* 0: exponential(mean p0); 1: lognormal(mu p0, sigma p1) */
  uint32_t gap_max;         /* gap after an instance: U{1..gap_max} */
  uint32_t phase_min;       /* first timestamp of a wave: U{phase_min..phase_max} */
  uint32_t phase_max;
  uint32_t swap_max;        /* swap partner distance U{1..swap_max} */
  uint32_t rec_cost;        /* copied into the trace header */
  uint32_t flags;           /* bit0: 0 circular, 1 flush */
  uint32_t reserved;
  double p0, p1;
  double p_orphan;          /* probability that an instance emits START only */
  double p_swap;            /* per-slot swap probability */
} kpgen_params;

typedef struct {
  uint32_t wg, wave, region, seq_start, ts_start, dur, has_end, pad;
} kpgen_inst;

#define HDR_BYTES 64u
#define WGHDR_BYTES 128u
#define MAGIC 0x4652504Bu /* bytes 'K','P','R','F' */

static inline uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
typedef struct { uint64_t s; } rng_t;
static inline uint64_t rng_next(rng_t* r) {
  r->s += 0x9E3779B97F4A7C15ull;
  return mix64(r->s);
}
static inline double rng_unit(rng_t* r) { /* (0,1] */
  return ((double)(rng_next(r) >> 11) + 1.0) * (1.0 / 9007199254740992.0);
}
static inline uint32_t rng_range(rng_t* r, uint32_t lo, uint32_t hi) { /* inclusive */
  if (hi <= lo) return lo;
  return lo + (uint32_t)(rng_next(r) % (uint64_t)(hi - lo + 1));
}

size_t kpgen_trace_bytes(uint32_t n_wg, uint32_t waves, uint32_t cap_wave) {
  return (size_t)HDR_BYTES + (size_t)WGHDR_BYTES * n_wg +
         (size_t)8 * n_wg * waves * cap_wave;
}

/* Returns 0 on success.  `truth` may be NULL; otherwise receives one entry per
 * generated region instance (including instances whose records were dropped),
 * up to truth_cap entries per call; *n_truth gets the number produced. */
int kpgen_trace(const kpgen_params* p, void* out, size_t out_bytes,
                kpgen_inst* truth, size_t truth_cap, size_t* n_truth) {
  if (!p || !out) return -1;
  if (p->waves == 0 || p->waves > 16 || p->n_regions == 0 || p->n_regions > 128) return -1;
  if (p->cap_wave == 0 || (p->cap_wave & (p->cap_wave - 1))) return -1;
  if (p->total_per_wave >= (1u << 20)) return -1;
  if (out_bytes < kpgen_trace_bytes(p->n_wg, p->waves, p->cap_wave)) return -2;

  uint8_t* base = (uint8_t*)out;
  uint32_t* hdr = (uint32_t*)base;
  memset(hdr, 0, HDR_BYTES);
  hdr[0] = MAGIC; hdr[1] = 1; hdr[2] = p->n_wg; hdr[3] = p->waves;
  hdr[4] = p->n_regions; hdr[5] = p->cap_wave; hdr[6] = p->rec_cost; hdr[7] = p->flags;

  const uint32_t cap = p->cap_wave, W = p->waves;
  const int flush = (int)(p->flags & 1u);
  /* worst-case instances per wave = total_per_wave (all start-only) */
  const size_t inst_stride = (size_t)p->total_per_wave;
  size_t truth_needed = (size_t)p->n_wg * W * inst_stride;
  int want_truth = truth != NULL;
  if (want_truth && truth_cap < truth_needed) return -3;
  size_t* truth_count = NULL;
  if (want_truth) {
    truth_count = (size_t*)calloc((size_t)p->n_wg * W, sizeof(size_t));
    if (!truth_count) return -4;
  }

#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t wg = 0; wg < (int64_t)p->n_wg; ++wg) {
    uint32_t* wh = (uint32_t*)(base + HDR_BYTES + (size_t)WGHDR_BYTES * wg);
    memset(wh, 0, WGHDR_BYTES);
    rng_t rg = { mix64(p->seed ^ 0xA5A5A5A5ull) + 0x1000003ull * (uint64_t)wg };
    uint64_t t_begin = rng_next(&rg) & 0xFFFFFFFFFFull;
    wh[0] = (uint32_t)wg;
    wh[1] = (uint32_t)(rng_next(&rg) & 0xFFFu);
    uint32_t max_ts = 0;
    for (uint32_t w = 0; w < W; ++w) {
      rng_t r = { mix64(p->seed + 0x632BE59BD9B4E019ull * ((uint64_t)wg * 16u + w + 1u)) };
      uint32_t* seg = (uint32_t*)(base + HDR_BYTES + (size_t)WGHDR_BYTES * p->n_wg +
                                  (size_t)8 * (((size_t)wg * W + w) * cap));
      for (uint32_t s = 0; s < cap; ++s) { seg[2 * s] = 0xDEADBEEFu; seg[2 * s + 1] = 0xDEADBEEFu; }
      uint32_t T = p->total_per_wave - rng_range(&r, 0, p->total_var <= p->total_per_wave ? p->total_var : p->total_per_wave);
      uint32_t V = T < cap ? T : cap;
      uint32_t keep_from = flush ? 0u : T - V;       /* first surviving seq */
      uint32_t keep_to = flush ? V : T;              /* one past last surviving seq */
      uint64_t t = rng_range(&r, p->phase_min, p->phase_max);
      uint32_t seq = 0, region = 0;
      kpgen_inst* tw = want_truth ? truth + ((size_t)wg * W + w) * inst_stride : NULL;
      size_t nt = 0;
      while (seq < T) {
        double u1 = rng_unit(&r), u2 = rng_unit(&r), uo = rng_unit(&r);
        uint32_t gap = rng_range(&r, 1, p->gap_max);
        double dv;
        if (p->dist == 0) {
          dv = -p->p0 * log(u1);
        } else {
          double z = sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925 * u2);
          dv = exp(p->p0 + p->p1 * z);
        }
        if (dv > 1.0e6) dv = 1.0e6;
        uint32_t d = (uint32_t)floor(dv);
        if (d < 1) d = 1;
        int start_only = (T - seq == 1) || (uo <= p->p_orphan);
        if (tw) {
          kpgen_inst* e = &tw[nt++];
          e->wg = (uint32_t)wg; e->wave = w; e->region = region; e->seq_start = seq;
          e->ts_start = (uint32_t)t; e->dur = start_only ? 0 : d; e->has_end = !start_only; e->pad = 0;
        }
        if (seq >= keep_from && seq < keep_to) {
          uint32_t slot = seq & (cap - 1);
          seg[2 * slot] = (0u << 31) | (region << 24) | (w << 20) | (seq & 0xFFFFFu);
          seg[2 * slot + 1] = (uint32_t)t;
        }
        if ((uint32_t)t > max_ts) max_ts = (uint32_t)t;
        ++seq;
        if (!start_only) {
          t += d;
          if (seq >= keep_from && seq < keep_to) {
            uint32_t slot = seq & (cap - 1);
            seg[2 * slot] = (1u << 31) | (region << 24) | (w << 20) | (seq & 0xFFFFFu);
            seg[2 * slot + 1] = (uint32_t)t;
          }
          if ((uint32_t)t > max_ts) max_ts = (uint32_t)t;
          ++seq;
        }
        t += gap;
        region = (region + 1) % p->n_regions;
      }
      if (want_truth) truth_count[(size_t)wg * W + w] = nt;
      /* out-of-order flush model: swap a few slots with a later slot of the same segment */
      if (p->p_swap > 0.0 && V > 1) {
        for (uint32_t s = 0; s + 1 < V; ++s) {
          double us = rng_unit(&r);
          uint32_t dist = rng_range(&r, 1, p->swap_max ? p->swap_max : 1);
          if (us <= p->p_swap) {
            uint32_t q = s + dist; if (q > V - 1) q = V - 1;
            uint32_t a0 = seg[2 * s], a1 = seg[2 * s + 1];
            seg[2 * s] = seg[2 * q]; seg[2 * s + 1] = seg[2 * q + 1];
            seg[2 * q] = a0; seg[2 * q + 1] = a1;
          }
        }
      }
      wh[8 + w] = T; /* total_written[w] lives at byte offset 32 */
    }
    uint64_t t_end = t_begin + (uint64_t)max_ts + 1u + (rng_next(&rg) & 63u);
    memcpy(&wh[2], &t_begin, 8);
    memcpy(&wh[4], &t_end, 8);
  }

  if (want_truth) {
    /* compact per-wave truth lists into one contiguous list, in (wg, wave) order */
    size_t o = 0;
    for (size_t i = 0; i < (size_t)p->n_wg * W; ++i) {
      size_t c = truth_count[i];
      if (o != i * inst_stride) memmove(truth + o, truth + i * inst_stride, c * sizeof(kpgen_inst));
      o += c;
    }
    if (n_truth) *n_truth = o;
    free(truth_count);
  } else if (n_truth) {
    *n_truth = 0;
  }
  return 0;
}

"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Nothing in here computes what the method computes: the functions only draw
random workloads and encode them in the raw-trace format (64-byte trace
header, 128-byte workgroup headers, 8-byte records = 4-byte tag + 4-byte
32-bit clock payload, per the paper's Sec. 4.2 record description).  Neither
the CPU oracle nor the HIP library imports this package, and it imports
neither of them.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libkp_gen.so")
_lib = None

HDR_BYTES = 64
WGHDR_BYTES = 128
MAGIC = 0x4652504B
FLAG_FLUSH = 1
POISON = 0xDEADBEEF

PHASE_START = 0
PHASE_END = 1


def build(force: bool = False) -> str:
    """Compile the C generator with gcc (OpenMP)."""
    src = os.path.join(_HERE, "kp_gen.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB_PATH, src, "-lm"]
        )
    return _LIB_PATH


class _Params(ctypes.Structure):
    _fields_ = [
        ("seed", ctypes.c_uint64),
        ("n_wg", ctypes.c_uint32),
        ("waves", ctypes.c_uint32),
        ("n_regions", ctypes.c_uint32),
        ("cap_wave", ctypes.c_uint32),
        ("total_per_wave", ctypes.c_uint32),
        ("total_var", ctypes.c_uint32),
        ("dist", ctypes.c_uint32),
        ("gap_max", ctypes.c_uint32),
        ("phase_min", ctypes.c_uint32),
        ("phase_max", ctypes.c_uint32),
        ("swap_max", ctypes.c_uint32),
        ("rec_cost", ctypes.c_uint32),
        ("flags", ctypes.c_uint32),
        ("reserved", ctypes.c_uint32),
        ("p0", ctypes.c_double),
        ("p1", ctypes.c_double),
        ("p_orphan", ctypes.c_double),
        ("p_swap", ctypes.c_double),
    ]


TRUTH_DTYPE = np.dtype(
    [
        ("wg", "<u4"),
        ("wave", "<u4"),
        ("region", "<u4"),
        ("seq_start", "<u4"),
        ("ts_start", "<u4"),
        ("dur", "<u4"),
        ("has_end", "<u4"),
        ("pad", "<u4"),
    ]
)


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build()
        lib = ctypes.CDLL(_LIB_PATH)
        lib.kpgen_trace_bytes.restype = ctypes.c_size_t
        lib.kpgen_trace_bytes.argtypes = [ctypes.c_uint32] * 3
        lib.kpgen_trace.restype = ctypes.c_int
        lib.kpgen_trace.argtypes = [
            ctypes.POINTER(_Params),
            ctypes.c_void_p,
            ctypes.c_size_t,
            ctypes.c_void_p,
            ctypes.c_size_t,
            ctypes.POINTER(ctypes.c_size_t),
        ]
        _lib = lib
    return _lib


def trace_bytes(n_wg: int, waves: int, cap_wave: int) -> int:
    return HDR_BYTES + WGHDR_BYTES * n_wg + 8 * n_wg * waves * cap_wave


@dataclass
class TraceSpec:
    """Parameters of one synthetic trace (see kp_gen.c for the recipe)."""

    n_wg: int
    waves: int
    n_regions: int
    cap_wave: int
    total_per_wave: int
    seed: int = 0
    total_var: int = 0
    dist: str = "lognormal"  # or "exp"
    p0: float = 6.0
    p1: float = 1.0
    gap_max: int = 32
    phase_min: int = 0
    phase_max: int = 4095
    p_orphan: float = 0.0
    p_swap: float = 0.0
    swap_max: int = 15
    rec_cost: int = 0
    flush: bool = False

    @property
    def n_slots(self) -> int:
        return self.n_wg * self.waves * self.cap_wave


def gen_trace(spec: TraceSpec, want_truth: bool = False, out: np.ndarray | None = None):
    """Generate a raw trace.  Returns (raw_u32_words, truth_or_None)."""
    lib = _load()
    nbytes = trace_bytes(spec.n_wg, spec.waves, spec.cap_wave)
    if out is None:
        out = np.empty(nbytes // 4, dtype=np.uint32)
    assert out.dtype == np.uint32 and out.size * 4 >= nbytes and out.flags["C_CONTIGUOUS"]
    p = _Params(
        seed=spec.seed,
        n_wg=spec.n_wg,
        waves=spec.waves,
        n_regions=spec.n_regions,
        cap_wave=spec.cap_wave,
        total_per_wave=spec.total_per_wave,
        total_var=spec.total_var,
        dist=0 if spec.dist == "exp" else 1,
        gap_max=spec.gap_max,
        phase_min=spec.phase_min,
        phase_max=spec.phase_max,
        swap_max=spec.swap_max,
        rec_cost=spec.rec_cost,
        flags=FLAG_FLUSH if spec.flush else 0,
        reserved=0,
        p0=spec.p0,
        p1=spec.p1,
        p_orphan=spec.p_orphan,
        p_swap=spec.p_swap,
    )
    truth = None
    n_truth = ctypes.c_size_t(0)
    if want_truth:
        cap_t = spec.n_wg * spec.waves * spec.total_per_wave
        truth = np.zeros(cap_t, dtype=TRUTH_DTYPE)
        rc = lib.kpgen_trace(
            ctypes.byref(p), out.ctypes.data, out.size * 4, truth.ctypes.data, cap_t, ctypes.byref(n_truth)
        )
    else:
        rc = lib.kpgen_trace(ctypes.byref(p), out.ctypes.data, out.size * 4, None, 0, ctypes.byref(n_truth))
    if rc != 0:
        raise RuntimeError(f"kpgen_trace failed rc={rc}")
    if truth is not None:
        truth = truth[: n_truth.value]
    return out, truth


# --- the named workload shapes (recipes: per-wave cyclic regions, see kp_gen.c) ---------------

def spec_small_gemm_shape(seed: int = 1) -> TraceSpec:
    """Synthetic trace with the shape of the 256^3 instrumented GEMM: 64 WGs x 4 waves,
    3 regions x 8 K-steps, exponential(mean 200) durations, no drops, no disorder."""
    return TraceSpec(
        n_wg=64, waves=4, n_regions=3, cap_wave=128, total_per_wave=48, seed=seed,
        dist="exp", p0=200.0, gap_max=32, phase_min=1, phase_max=64,
    )


def spec_decode_standalone(log2_records: int = 28, seed: int = 4, wrap: bool = False) -> TraceSpec:
    """Standalone decode workload: 8 waves x 2048-record sub-rings x 16 regions,
    lognormal(6,1) durations, ~1% start-only records, 0.1% displaced slots.
    log2_records=28 gives the full 16384-workgroup trace; smaller values scale n_wg down."""
    n_wg = (1 << log2_records) // (8 * 2048)
    assert n_wg >= 1
    return TraceSpec(
        n_wg=n_wg, waves=8, n_regions=16, cap_wave=2048,
        total_per_wave=3 * 2048 if wrap else 2048, seed=seed,
        dist="lognormal", p0=6.0, p1=1.0, gap_max=32, phase_min=0, phase_max=4095,
        p_orphan=2.0 / 101.0, p_swap=1e-3, swap_max=15,
    )


# --- hand-built traces ------------------------------------------------------------------------

def make_tag(phase: int, region: int, wave: int, seq: int) -> int:
    return ((phase & 1) << 31) | ((region & 0x7F) << 24) | ((wave & 0xF) << 20) | (seq & 0xFFFFF)


def encode_trace(
    wgs: list[dict],
    waves: int,
    n_regions: int,
    cap_wave: int,
    rec_cost: int = 0,
    flush: bool = False,
) -> np.ndarray:
    """Encode explicit slot contents.

    Each element of `wgs` is a dict with keys
      t_begin, t_end            : 64-bit counter values
      totals                    : list[waves] of total_written
      slots                     : list[waves] of lists of (tag, payload) in slot order
                                  (shorter than cap_wave => rest poisoned)
    """
    n_wg = len(wgs)
    raw = np.empty(trace_bytes(n_wg, waves, cap_wave) // 4, dtype=np.uint32)
    raw[:] = POISON
    raw[:16] = 0
    raw[0:8] = [MAGIC, 1, n_wg, waves, n_regions, cap_wave, rec_cost, FLAG_FLUSH if flush else 0]
    rec0 = (HDR_BYTES + WGHDR_BYTES * n_wg) // 4
    for i, wg in enumerate(wgs):
        h = (HDR_BYTES + WGHDR_BYTES * i) // 4
        raw[h : h + 32] = 0
        raw[h] = wg.get("wg_id", i)
        raw[h + 1] = wg.get("hw_id", 0)
        tb = int(wg["t_begin"]) & 0xFFFFFFFFFFFFFFFF
        te = int(wg["t_end"]) & 0xFFFFFFFFFFFFFFFF
        raw[h + 2] = tb & 0xFFFFFFFF
        raw[h + 3] = tb >> 32
        raw[h + 4] = te & 0xFFFFFFFF
        raw[h + 5] = te >> 32
        for w in range(waves):
            raw[h + 8 + w] = wg["totals"][w]
            base = rec0 + 2 * ((i * waves + w) * cap_wave)
            for s, (tag, payload) in enumerate(wg["slots"][w]):
                assert s < cap_wave
                raw[base + 2 * s] = tag & 0xFFFFFFFF
                raw[base + 2 * s + 1] = payload & 0xFFFFFFFF
    return raw


def events_to_wg(wave_events: list[list[tuple]], cap_wave: int, t_begin: int = 1000,
                 t_end: int | None = None, flush: bool = False) -> dict:
    """Turn per-wave event lists [(phase, region, ts), ...] (program order) into a
    workgroup dict for encode_trace, applying the ring rule: circular keeps the last
    cap_wave records in slot seq mod cap_wave, flush keeps the first cap_wave."""
    slots, totals = [], []
    tmax = 0
    for w, evs in enumerate(wave_events):
        T = len(evs)
        totals.append(T)
        V = min(T, cap_wave)
        lo, hi = (0, V) if flush else (T - V, T)
        seg = [(POISON, POISON)] * V
        for seq, (ph, rg, ts) in enumerate(evs):
            tmax = max(tmax, ts)
            if lo <= seq < hi:
                seg[seq % cap_wave] = (make_tag(ph, rg, w, seq), ts)
        slots.append(seg)
    if t_end is None:
        t_end = t_begin + tmax + 1
    return {"t_begin": t_begin, "t_end": t_end, "totals": totals, "slots": slots}


def messy_trace(seed: int, n_wg: int = 6, waves: int = 4, n_regions: int = 5, cap_wave: int = 32,
                p_bad: float = 0.05, allow_nonmono: bool = True, flush: bool = False) -> np.ndarray:
    """Random trace with arbitrary START/END interleavings (nesting, repeats, orphans),
    ragged totals (including wrap), corrupted tags, duplicated sequence numbers,
    shuffled slots and occasional non-monotonic clocks.  Used to fuzz decoder parity."""
    rng = np.random.default_rng(seed)
    wgs = []
    for _ in range(n_wg):
        wave_events = []
        for _w in range(waves):
            T = int(rng.integers(0, 3 * cap_wave))
            t = int(rng.integers(0, 50))
            evs = []
            for _i in range(T):
                ph = int(rng.integers(0, 2))
                rg = int(rng.integers(0, n_regions))
                if allow_nonmono and rng.random() < 0.01:
                    t = max(0, t - int(rng.integers(1, 40)))
                else:
                    t += int(rng.integers(0, 30))
                evs.append((ph, rg, t))
            wave_events.append(evs)
        wg = events_to_wg(wave_events, cap_wave, t_begin=int(rng.integers(0, 1 << 40)), flush=flush)
        if rng.random() < 0.1:
            wg["t_end"] = wg["t_begin"] + (1 << 32) + 5  # span overflow
        # corrupt some records / shuffle some slots
        for w in range(waves):
            seg = wg["slots"][w]
            for s in range(len(seg)):
                u = rng.random()
                tag, pay = seg[s]
                if u < p_bad / 4:
                    tag = (tag & ~(0xF << 20)) | (((w + 1) % 16) << 20)  # wrong wave id
                elif u < 2 * p_bad / 4:
                    tag = (tag & ~(0x7F << 24)) | ((n_regions + int(rng.integers(0, 3))) << 24)  # bad region
                elif u < 3 * p_bad / 4:
                    tag = (tag & ~0xFFFFF) | int(rng.integers(0, 1 << 20))  # bad seq
                elif u < p_bad and s > 0:
                    tag = (tag & ~0xFFFFF) | (seg[s - 1][0] & 0xFFFFF)  # duplicate seq
                seg[s] = (tag, pay)
            if len(seg) > 2 and rng.random() < 0.5:
                i, j = rng.integers(0, len(seg), size=2)
                seg[i], seg[j] = seg[j], seg[i]
        wgs.append(wg)
    return encode_trace(wgs, waves, n_regions, cap_wave, rec_cost=int(rng.integers(0, 4)), flush=flush)


# --- dense-kernel inputs ----------------------------------------------------------------------

def gemm_inputs(M: int, N: int, K: int, seed: int, dist: str = "normal"):
    """A [M,K], B [K,N] as torch bfloat16 CPU tensors (row-major)."""
    import torch

    g = torch.Generator().manual_seed(seed)
    if dist == "uniform":
        a = torch.rand(M, K, generator=g) * 2 - 1
        b = torch.rand(K, N, generator=g) * 2 - 1
    else:
        a = torch.randn(M, K, generator=g)
        b = torch.randn(K, N, generator=g)
    return a.to(torch.bfloat16), b.to(torch.bfloat16)


def attn_inputs(B: int, H: int, S: int, D: int, seed: int):
    """Q, K, V [B,H,S,D] as torch bfloat16 CPU tensors, N(0,1)."""
    import torch

    g = torch.Generator().manual_seed(seed)
    q = torch.randn(B, H, S, D, generator=g).to(torch.bfloat16)
    k = torch.randn(B, H, S, D, generator=g).to(torch.bfloat16)
    v = torch.randn(B, H, S, D, generator=g).to(torch.bfloat16)
    return q, k, v

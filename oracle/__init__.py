"""CPU oracle -- TEST INFRASTRUCTURE ONLY.

Plain, slow reference implementations of what the hot path computes, written
from the paper (and, where the paper is silent, from the readings listed in the
design notes).  Only `tests/`, the smoke check and the benchmark's
`cpu_baseline` leg may import this package.  It imports nothing from the HIP
library or its Python binding, and shares no code with them.

  ref_decode.c : trace decode / pair / reduce (Sec. 4.2 record layout and
                 circular buffer, Sec. 4.3 trace replay)
  ref_pairs.c  : one timeline row per paired region instance, with its iteration
                 index (Sec. 3.2 decoded activity records, Sec. 3.3 iteration-based
                 timing)
  ref_waits.c  : waits behind asynchronous operations from the START / END / START
                 placement (Sec. 4.3, asynchronous instructions)
  ref_critical.c : the chain of stages each of which waited for the one before it (critical path)
  ref_stages.c : stage latencies per (workgroup, region, iteration) folded from the timeline
                 rows (Sec. 3.3 critical-path analysis, Sec. 5.2 / Table 4 overlap models)
  ref_dense.py : the dense kernels that get instrumented -- GEMM and causal
                 attention forward by their textbook definitions, fp64

All functions are pinned by `tests/test_oracle_*.py` against hand-worked
traces, a tick-by-tick brute force, construction truth from the generator,
closed forms and library routines; nothing here is "parity unpinned".
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libkp_oracle.so")
_lib = None

HEADER_FIELDS = (
    "n_slots_valid", "n_pairs", "n_orphan_start", "n_orphan_end", "n_invalid", "n_dropped",
    "n_disorder", "n_span_overflow_wgs", "n_nonmonotonic", "n_overlap_wgs", "status",
    "n_wg", "waves", "n_regions", "cap_wave", "reserved",
)

PER_DTYPE = np.dtype([("sum", "<u8"), ("n", "<u4"), ("max", "<u4")])


_SOURCES = ("ref_decode.c", "ref_pairs.c", "ref_waits.c", "ref_stages.c", "ref_critical.c")


def build(force: bool = False) -> str:
    srcs = [os.path.join(_HERE, f) for f in _SOURCES]
    stale = not os.path.exists(_LIB_PATH) or any(os.path.getmtime(_LIB_PATH) < os.path.getmtime(f) for f in srcs)
    if force or stale:
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB_PATH, *srcs])
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB_PATH)
        lib.kpo_stats_bytes.restype = ctypes.c_size_t
        lib.kpo_stats_bytes.argtypes = [ctypes.c_uint32] * 3
        lib.kpo_decode.restype = ctypes.c_int
        lib.kpo_decode.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int]
        lib.kpo_pairs_bytes.restype = ctypes.c_size_t
        lib.kpo_pairs_bytes.argtypes = [ctypes.c_uint32] * 3
        lib.kpo_pairs.restype = ctypes.c_int
        lib.kpo_pairs.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_size_t]
        lib.kpo_waits_bytes.restype = ctypes.c_size_t
        lib.kpo_waits_bytes.argtypes = [ctypes.c_uint32] * 3
        lib.kpo_waits.restype = ctypes.c_int
        lib.kpo_waits.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_size_t]
        lib.kpo_stages_bytes.restype = ctypes.c_size_t
        lib.kpo_stages_bytes.argtypes = [ctypes.c_uint32] * 3
        lib.kpo_stages.restype = ctypes.c_int
        lib.kpo_stages.argtypes = [ctypes.c_void_p] + [ctypes.c_uint32] * 5 + [ctypes.c_void_p, ctypes.c_size_t]
        lib.kpo_critical_bytes.restype = ctypes.c_size_t
        lib.kpo_critical_bytes.argtypes = [ctypes.c_uint32] * 2
        lib.kpo_critical.restype = ctypes.c_int
        lib.kpo_critical.argtypes = [ctypes.c_void_p] + [ctypes.c_uint32] * 3 + [ctypes.c_void_p, ctypes.c_size_t]
        _lib = lib
    return _lib


def stats_bytes(n_wg: int, waves: int, n_regions: int) -> int:
    return _load().kpo_stats_bytes(n_wg, waves, n_regions)


def decode_bytes(raw: np.ndarray, n_threads: int = 1) -> np.ndarray:
    """Run the reference decoder on a raw trace (uint32 words); returns the stats block bytes."""
    assert raw.dtype == np.uint32 and raw.flags["C_CONTIGUOUS"]
    n_wg, waves, R, cap = (int(x) for x in raw[2:6])
    n_slots = n_wg * waves * cap
    need = 64 + 128 * n_wg + 8 * n_slots
    if raw.size * 4 < need:
        raise ValueError("raw buffer shorter than its header claims")
    out = np.zeros(stats_bytes(n_wg, waves, R), dtype=np.uint8)
    rc = _load().kpo_decode(raw.ctypes.data, n_slots, out.ctypes.data, out.size, int(n_threads))
    if rc != 0:
        raise ValueError(f"kpo_decode rejected the trace (rc={rc})")
    return out


def view_stats(buf: np.ndarray) -> dict:
    """Split a stats block (uint8 array) into named numpy views."""
    b = np.ascontiguousarray(buf).view(np.uint8)
    hdr = b[:128].view("<u8")
    n_wg, W, R = int(hdr[11]), int(hdr[12]), int(hdr[13])
    o = 128
    def take(nbytes, dtype, shape):
        nonlocal o
        v = b[o : o + nbytes].view(dtype).reshape(shape)
        o += nbytes
        return v
    out = {name: int(hdr[i]) for i, name in enumerate(HEADER_FIELDS)}
    out["hist"] = take(8 * 64 * R, "<u8", (R, 64))
    for name in ("cnt", "sum", "min", "max", "U"):
        out[name] = take(8 * R, "<u8", (R,))
    out["O"] = take(8 * R * R, "<u8", (R, R))
    out["F"] = take(8 * R * R, "<f8", (R, R))
    out["per"] = take(16 * n_wg * W * R, PER_DTYPE, (n_wg, W, R))
    assert o == b.size, (o, b.size)
    return out


def decode(raw: np.ndarray, n_threads: int = 1) -> dict:
    return view_stats(decode_bytes(raw, n_threads))


PAIR_ROW_DTYPE = np.dtype([("start", "<u4"), ("dur", "<u4"), ("iter", "<u4"), ("region", "<u4")])


def pairs_bytes(n_wg: int, waves: int, cap_wave: int) -> int:
    return _load().kpo_pairs_bytes(n_wg, waves, cap_wave)


def pairs_raw(raw: np.ndarray, fill: int = 0xA5) -> np.ndarray:
    """Run the reference timeline decoder; returns the output block bytes (unwritten rows keep `fill`)."""
    assert raw.dtype == np.uint32 and raw.flags["C_CONTIGUOUS"]
    n_wg, waves, R, cap = (int(x) for x in raw[2:6])
    n_slots = n_wg * waves * cap
    if raw.size * 4 < 64 + 128 * n_wg + 8 * n_slots:
        raise ValueError("raw buffer shorter than its header claims")
    out = np.full(pairs_bytes(n_wg, waves, cap), fill, dtype=np.uint8)
    rc = _load().kpo_pairs(raw.ctypes.data, n_slots, out.ctypes.data, out.size)
    if rc != 0:
        raise ValueError(f"kpo_pairs rejected the trace (rc={rc})")
    return out


def view_pairs(buf: np.ndarray, n_wg: int, waves: int, cap_wave: int):
    """Split a pairs block into (count[n_wg, waves], rows[n_wg, waves, cap_wave // 2])."""
    b = np.ascontiguousarray(buf).view(np.uint8)
    n_seg = n_wg * waves
    head = ((n_seg + 3) // 4) * 16
    count = b[: 4 * n_seg].view("<u4").reshape(n_wg, waves)
    rows = b[head : head + 16 * n_seg * (cap_wave // 2)].view(PAIR_ROW_DTYPE).reshape(n_wg, waves, cap_wave // 2)
    return count, rows


def pairs(raw: np.ndarray):
    """Reference timeline rows: list over (wg, wave) of structured arrays, plus the counts."""
    n_wg, waves, _R, cap = (int(x) for x in raw[2:6])
    return view_pairs(pairs_raw(raw), n_wg, waves, cap)


WAITS_HEADER_FIELDS = ("n_waits", "n_uncovered", "n_async", "_3", "_4", "_5", "_6", "_7",
                       "n_wg", "waves", "n_regions", "cap_wave", "rec_cost", "_13", "_14", "_15")


def waits_bytes(n_wg: int, waves: int, n_regions: int) -> int:
    return _load().kpo_waits_bytes(n_wg, waves, n_regions)


def waits_raw(raw: np.ndarray) -> np.ndarray:
    """Run the reference wait replay on a raw trace (uint32 words); returns the output block bytes."""
    assert raw.dtype == np.uint32 and raw.flags["C_CONTIGUOUS"]
    n_wg, waves, R, cap = (int(x) for x in raw[2:6])
    n_slots = n_wg * waves * cap
    if raw.size * 4 < 64 + 128 * n_wg + 8 * n_slots:
        raise ValueError("raw buffer shorter than its header claims")
    out = np.full(waits_bytes(n_wg, waves, R), 0xEE, dtype=np.uint8)
    rc = _load().kpo_waits(raw.ctypes.data, n_slots, out.ctypes.data, out.size)
    if rc != 0:
        raise ValueError(f"kpo_waits rejected the trace (rc={rc})")
    return out


def view_waits(buf: np.ndarray) -> dict:
    """Split a waits block (uint8 array) into named numpy views."""
    b = np.ascontiguousarray(buf).view(np.uint8)
    hdr = b[:128].view("<u8")
    n_wg, W, R = int(hdr[8]), int(hdr[9]), int(hdr[10])
    out = {name: int(hdr[i]) for i, name in enumerate(WAITS_HEADER_FIELDS) if not name.startswith("_")}
    o = 128
    out["hist"] = b[o : o + 8 * 64 * R].view("<u8").reshape(R, 64)
    o += 8 * 64 * R
    for name in ("cnt", "sum", "min", "max", "uncovered", "async_cnt", "async_sum"):
        out[name] = b[o : o + 8 * R].view("<u8")
        o += 8 * R
    out["per"] = b[o : o + 16 * n_wg * W * R].view(PER_DTYPE).reshape(n_wg, W, R)
    assert o + 16 * n_wg * W * R == b.size
    return out


def waits(raw: np.ndarray) -> dict:
    return view_waits(waits_raw(raw))


STAGE_DTYPE = np.dtype([("max_dur", "<u4"), ("min_start", "<u4"), ("max_end", "<u4"), ("n_waves", "<u4")])


def stages_raw(pairs_block: np.ndarray, n_wg: int, waves: int, cap_wave: int, n_regions: int, max_iter: int) -> np.ndarray:
    """Fold a timeline block (bytes, as pairs_raw returns it) into the stage table; returns the block bytes."""
    blk = np.ascontiguousarray(pairs_block).view(np.uint8)
    assert blk.size >= pairs_bytes(n_wg, waves, cap_wave)
    out = np.full(_load().kpo_stages_bytes(n_wg, n_regions, max_iter), 0xEE, dtype=np.uint8)
    rc = _load().kpo_stages(blk.ctypes.data, n_wg, waves, cap_wave, n_regions, max_iter, out.ctypes.data, out.size)
    if rc != 0:
        raise ValueError(f"kpo_stages rejected its arguments (rc={rc})")
    return out


def view_stages(buf: np.ndarray, n_wg: int, n_regions: int, max_iter: int):
    """Split a stage block into (header dict, table[n_wg, n_regions, max_iter])."""
    b = np.ascontiguousarray(buf).view(np.uint8)
    h = b[:32].view("<u8")
    hdr = {"n_rows": int(h[0]), "n_clipped": int(h[1]), "n_bad_region": int(h[2])}
    tab = b[32 : 32 + 16 * n_wg * n_regions * max_iter].view(STAGE_DTYPE).reshape(n_wg, n_regions, max_iter)
    return hdr, tab


def stages(raw: np.ndarray, max_iter: int):
    """Reference stage table of a raw trace: timeline rows first, then the fold."""
    n_wg, waves, R, cap = (int(x) for x in raw[2:6])
    return view_stages(stages_raw(pairs_raw(raw), n_wg, waves, cap, R, max_iter), n_wg, R, max_iter)


PATH_DTYPE = np.dtype([("n_stages", "<u4"), ("last_stage", "<u4"), ("first_start", "<u4"), ("last_end", "<u4"),
                       ("sum_latency", "<u8"), ("bubbles", "<u8")])


def stage_block(table: np.ndarray) -> np.ndarray:
    """Bytes of a stage block around a table[n_wg, n_regions, max_iter] of STAGE_DTYPE (header words zero)."""
    t = np.ascontiguousarray(table, dtype=STAGE_DTYPE)
    return np.concatenate([np.zeros(32, dtype=np.uint8), t.reshape(-1).view(np.uint8)])


def critical_raw(stage_blk: np.ndarray, n_wg: int, n_regions: int, max_iter: int) -> np.ndarray:
    """Critical path of every workgroup of a stage block (bytes, as stages_raw returns it); returns the block bytes."""
    blk = np.ascontiguousarray(stage_blk).view(np.uint8)
    assert blk.size >= 32 + 16 * n_wg * n_regions * max_iter
    out = np.full(_load().kpo_critical_bytes(n_wg, n_regions), 0xEE, dtype=np.uint8)
    rc = _load().kpo_critical(blk.ctypes.data, n_wg, n_regions, max_iter, out.ctypes.data, out.size)
    if rc != 0:
        raise ValueError(f"kpo_critical rejected its arguments (rc={rc})")
    return out


def view_critical(buf: np.ndarray, n_wg: int, n_regions: int):
    """Split a critical-path block into (header dict, per-region array[R, 2], rows[n_wg])."""
    b = np.ascontiguousarray(buf).view(np.uint8)
    h = b[:64].view("<u8")
    hdr = {"n_wg": int(h[0]), "n_regions": int(h[1]), "max_iter": int(h[2]), "n_paths": int(h[3]),
           "n_path_stages": int(h[4]), "sum_latency": int(h[5]), "sum_bubbles": int(h[6])}
    per_region = b[64 : 64 + 16 * n_regions].view("<u8").reshape(n_regions, 2)
    rows = b[64 + 16 * n_regions : 64 + 16 * n_regions + 32 * n_wg].view(PATH_DTYPE)
    return hdr, per_region, rows


from .ref_dense import ref_gemm, ref_attn, bf16_round  # noqa: E402,F401

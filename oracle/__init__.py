"""CPU oracle -- TEST INFRASTRUCTURE ONLY.

Plain, slow reference implementations of what the hot path computes, written
from the paper (and, where the paper is silent, from the readings listed in the
design notes).  Only `tests/`, the smoke check and the benchmark's
`cpu_baseline` leg may import this package.  It imports nothing from the HIP
library or its Python binding, and shares no code with them.

  ref_decode.c : trace decode / pair / reduce (Sec. 4.2 record layout and
                 circular buffer, Sec. 4.3 trace replay)
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


def build(force: bool = False) -> str:
    src = os.path.join(_HERE, "ref_decode.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB_PATH, src])
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build()
        lib = ctypes.CDLL(_LIB_PATH)
        lib.kpo_stats_bytes.restype = ctypes.c_size_t
        lib.kpo_stats_bytes.argtypes = [ctypes.c_uint32] * 3
        lib.kpo_decode.restype = ctypes.c_int
        lib.kpo_decode.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int]
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


from .ref_dense import ref_gemm, ref_attn, bf16_round  # noqa: E402,F401

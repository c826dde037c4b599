"""ctypes binding of libkperf.so -- same names as the C ABI in include/kperf.h.

Argument marshalling only.  Tensors must live on the GPU (device pointers are
passed through unchanged); `stream` defaults to torch's current stream.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkperf.so")

KP_OK = 0
KP_ERR_INVALID_ARG = -1
KP_ERR_UNSUPPORTED_SHAPE = -2
KP_ERR_TRACE_TOO_SMALL = -3
KP_ERR_BAD_TRACE = -4
KP_ERR_HIP = -5

KP_FLAG_FLUSH = 1
KP_MASK_FLUSH = 1 << 31
KP_MASK_WAVE_GROUP = 1 << 30  # one record stream per group of four waves
KP_MASK_PHASES = 1 << 29      # 256x256x64 GEMM: the stages of a K step one after the other, 5 regions
KP_MASK_REALTIME = 1 << 28    # records carry the constant-rate 100 MHz clock
KP_MASK_COLLAB = 1 << 27      # all lanes store a record; hardware ids of the waves in the workgroup header
KP_MASK_UNFENCED = 1 << 26    # with KP_MASK_PHASES and no region: the staged K step without scheduling fences
KP_FLAG_REALTIME = 2
KP_FLAG_HW_IDS = 4


class KperfError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"libkperf status {status}: {message}")
        self.status = status


class kp_trace_hdr(ctypes.Structure):
    _fields_ = [
        ("magic", ctypes.c_uint32), ("version", ctypes.c_uint32), ("n_wg", ctypes.c_uint32),
        ("waves_per_wg", ctypes.c_uint32), ("n_regions", ctypes.c_uint32), ("cap_wave", ctypes.c_uint32),
        ("rec_cost", ctypes.c_uint32), ("flags", ctypes.c_uint32), ("pad", ctypes.c_uint32 * 8),
    ]


_lib = None


def lib() -> ctypes.CDLL:
    """Load libkperf.so; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'`"
            )
        # The caller's device buffers come from torch, which ships its own copy of the HIP runtime.
        # That copy has to be the first one in the process: if this library pulled in the system's
        # runtime before torch loaded its own, the two would not share a device context and every
        # launch from here would fail with "no ROCm-capable device".
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, ci, u32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_uint32
        L.kp_last_error.restype = ctypes.c_char_p
        L.kp_last_error.argtypes = []
        L.kp_trace_bytes.restype = sz
        L.kp_trace_bytes.argtypes = [ci, ci, ci]
        L.kp_stats_bytes.restype = sz
        L.kp_stats_bytes.argtypes = [ci, ci, ci]
        L.kp_trace_reduce.restype = ci
        L.kp_trace_reduce.argtypes = [vp, sz, vp, vp]
        L.kp_trace_reduce_hdr.restype = ci
        L.kp_trace_reduce_hdr.argtypes = [vp, sz, ctypes.POINTER(kp_trace_hdr), vp, vp]
        L.kp_trace_reduce_hdr_events.restype = ci
        L.kp_trace_reduce_hdr_events.argtypes = [vp, sz, ctypes.POINTER(kp_trace_hdr), vp, vp, vp, vp]
        L.kp_trace_reduce_steps.restype = ci
        L.kp_trace_reduce_steps.argtypes = [vp, sz, ctypes.POINTER(kp_trace_hdr), vp, ci, vp]
        L.kp_pairs_bytes.restype = sz
        L.kp_pairs_bytes.argtypes = [ci, ci, ci]
        L.kp_trace_pairs.restype = ci
        L.kp_trace_pairs.argtypes = [vp, sz, vp, vp]
        L.kp_trace_pairs_hdr.restype = ci
        L.kp_trace_pairs_hdr.argtypes = [vp, sz, ctypes.POINTER(kp_trace_hdr), vp, vp]
        L.kp_waits_bytes.restype = sz
        L.kp_waits_bytes.argtypes = [ci, ci, ci]
        L.kp_trace_waits.restype = ci
        L.kp_trace_waits.argtypes = [vp, sz, vp, vp]
        L.kp_trace_waits_hdr.restype = ci
        L.kp_trace_waits_hdr.argtypes = [vp, sz, ctypes.POINTER(kp_trace_hdr), vp, vp]
        L.kp_stages_bytes.restype = sz
        L.kp_stages_bytes.argtypes = [ci, ci, ci]
        L.kp_pairs_stages.restype = ci
        L.kp_pairs_stages.argtypes = [vp, ci, ci, ci, ci, ci, vp, vp]
        L.kp_critical_bytes.restype = sz
        L.kp_critical_bytes.argtypes = [ci, ci]
        L.kp_stages_critical.restype = ci
        L.kp_stages_critical.argtypes = [vp, ci, ci, ci, vp, vp]
        L.kp_set_rec_cost.restype = None
        L.kp_set_rec_cost.argtypes = [u32]
        L.kp_get_rec_cost.restype = u32
        L.kp_get_rec_cost.argtypes = []
        _optional(L)
        _lib = L
    return _lib


def _optional(L):
    vp, sz, ci, u32, fl = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_uint32, ctypes.c_float
    ip = ctypes.POINTER(ctypes.c_int)
    sigs = {
        "kp_gemm_launch_shape": [ci, ci, ci, ip, ip, ip],
        "kp_gemm_instrumented": [vp, vp, vp, ci, ci, ci, u32, vp, sz, vp],
        "kp_attn_launch_shape": [ci, ci, ci, ci, ip, ip, ip],
        "kp_attn_instrumented": [vp, vp, vp, vp, ci, ci, ci, ci, ci, fl, u32, vp, sz, vp],
        "kp_calibrate": [ctypes.POINTER(u32), ci, ci, ci, ci, vp, sz, vp],
    }
    for name, args in sigs.items():
        if hasattr(L, name):
            f = getattr(L, name)
            f.restype = ci
            f.argtypes = args


def _check(status: int):
    if status != KP_OK:
        raise KperfError(status, kp_last_error())


def _ptr(t) -> int:
    if t is None:
        return 0
    if not t.is_cuda:
        raise ValueError("libkperf takes device memory: tensor must be on the GPU")
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return t.data_ptr()


def _stream(stream) -> int:
    import torch

    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def kp_last_error() -> str:
    return lib().kp_last_error().decode()


def kp_trace_bytes(n_wg: int, waves_per_wg: int, cap_per_wg: int) -> int:
    return lib().kp_trace_bytes(n_wg, waves_per_wg, cap_per_wg)


def kp_stats_bytes(n_wg: int, waves_per_wg: int, n_regions: int) -> int:
    return lib().kp_stats_bytes(n_wg, waves_per_wg, n_regions)


def kp_set_rec_cost(ticks: int) -> None:
    lib().kp_set_rec_cost(int(ticks))


def kp_get_rec_cost() -> int:
    return int(lib().kp_get_rec_cost())


def kp_trace_reduce(raw, n: int, out_stats, stream=None) -> None:
    _check(lib().kp_trace_reduce(_ptr(raw), n, _ptr(out_stats), _stream(stream)))


def make_hdr(n_wg: int, waves_per_wg: int, n_regions: int, cap_wave: int, rec_cost: int = 0,
             flags: int = 0) -> kp_trace_hdr:
    h = kp_trace_hdr()
    h.magic, h.version = 0x4652504B, 1
    h.n_wg, h.waves_per_wg, h.n_regions, h.cap_wave = n_wg, waves_per_wg, n_regions, cap_wave
    h.rec_cost, h.flags = rec_cost, flags
    return h


def kp_trace_reduce_hdr(raw, n: int, hdr_host: kp_trace_hdr, out_stats, stream=None) -> None:
    _check(lib().kp_trace_reduce_hdr(_ptr(raw), n, ctypes.byref(hdr_host), _ptr(out_stats), _stream(stream)))


def kp_trace_reduce_hdr_events(raw, n: int, hdr_host: kp_trace_hdr, out_stats, main_begin, main_end, stream=None) -> None:
    """main_begin, main_end: torch.cuda.Event objects with timing enabled that have been recorded before (an
    event's handle exists from its first record on), raw hipEvent_t handles as int, or None."""
    def handle(ev):
        if ev is None or isinstance(ev, int):
            return ev
        h = ev.cuda_event
        if not h:
            raise ValueError("record the event once before passing it: it has no handle yet")
        return h
    _check(lib().kp_trace_reduce_hdr_events(_ptr(raw), n, ctypes.byref(hdr_host), _ptr(out_stats), _stream(stream),
                                            handle(main_begin), handle(main_end)))


def kp_trace_reduce_steps(raw, n: int, hdr_host: kp_trace_hdr, out_stats, last_step: int, stream=None) -> None:
    _check(lib().kp_trace_reduce_steps(_ptr(raw), n, ctypes.byref(hdr_host), _ptr(out_stats), last_step,
                                       _stream(stream)))


def kp_pairs_bytes(n_wg: int, waves_per_wg: int, cap_per_wg: int) -> int:
    return lib().kp_pairs_bytes(n_wg, waves_per_wg, cap_per_wg)


def kp_trace_pairs(raw, n: int, out_pairs, stream=None) -> None:
    _check(lib().kp_trace_pairs(_ptr(raw), n, _ptr(out_pairs), _stream(stream)))


def kp_trace_pairs_hdr(raw, n: int, hdr_host: kp_trace_hdr, out_pairs, stream=None) -> None:
    _check(lib().kp_trace_pairs_hdr(_ptr(raw), n, ctypes.byref(hdr_host), _ptr(out_pairs), _stream(stream)))


PAIR_ROW_DTYPE = [("start", "<u4"), ("dur", "<u4"), ("iter", "<u4"), ("region", "<u4")]


def parse_pairs(buf, n_wg: int, waves_per_wg: int, cap_per_wg: int):
    """Split a pairs block (host bytes: numpy array or CPU tensor) into (count[n_wg, waves],
    rows[n_wg, waves, cap_wave // 2]); only the first count[wg, wave] rows of a wave are meaningful."""
    import numpy as np

    b = np.ascontiguousarray(buf.cpu().numpy() if hasattr(buf, "numpy") else buf).view(np.uint8)
    n_seg, half = n_wg * waves_per_wg, cap_per_wg // waves_per_wg // 2
    head = ((n_seg + 3) // 4) * 16
    count = b[: 4 * n_seg].view("<u4").reshape(n_wg, waves_per_wg)
    rows = b[head : head + 16 * n_seg * half].view(np.dtype(PAIR_ROW_DTYPE)).reshape(n_wg, waves_per_wg, half)
    return count, rows


def kp_waits_bytes(n_wg: int, waves_per_wg: int, n_regions: int) -> int:
    return lib().kp_waits_bytes(n_wg, waves_per_wg, n_regions)


def kp_trace_waits(raw, n: int, out_waits, stream=None) -> None:
    _check(lib().kp_trace_waits(_ptr(raw), n, _ptr(out_waits), _stream(stream)))


def kp_trace_waits_hdr(raw, n: int, hdr_host: kp_trace_hdr, out_waits, stream=None) -> None:
    _check(lib().kp_trace_waits_hdr(_ptr(raw), n, ctypes.byref(hdr_host), _ptr(out_waits), _stream(stream)))


WAITS_HEADER_FIELDS = ("n_waits", "n_uncovered", "n_async", None, None, None, None, None,
                       "n_wg", "waves_per_wg", "n_regions", "cap_wave", "rec_cost", None, None, None)


def parse_waits(buf) -> dict:
    """Split a waits block (bytes on the host: numpy uint8 array or CPU tensor) into fields."""
    if hasattr(buf, "numpy"):
        buf = buf.cpu().numpy()
    b = np.ascontiguousarray(buf).view(np.uint8)
    hdr = b[:128].view("<u8")
    out = {k: int(hdr[i]) for i, k in enumerate(WAITS_HEADER_FIELDS) if k}
    n_wg, W, R = out["n_wg"], out["waves_per_wg"], out["n_regions"]
    pos = 128
    out["hist"] = b[pos : pos + 8 * 64 * R].view("<u8").reshape(R, 64)
    pos += 8 * 64 * R
    for name in ("cnt", "sum", "min", "max", "uncovered", "async_cnt", "async_sum"):
        out[name] = b[pos : pos + 8 * R].view("<u8")
        pos += 8 * R
    out["per"] = b[pos : pos + 16 * n_wg * W * R].view(WAVE_REGION_DTYPE).reshape(n_wg, W, R)
    return out


def kp_stages_bytes(n_wg: int, n_regions: int, max_iter: int) -> int:
    return lib().kp_stages_bytes(n_wg, n_regions, max_iter)


def kp_pairs_stages(pairs, n_wg: int, waves_per_wg: int, cap_per_wg: int, n_regions: int, max_iter: int,
                    out_stages, stream=None) -> None:
    _check(lib().kp_pairs_stages(_ptr(pairs), n_wg, waves_per_wg, cap_per_wg, n_regions, max_iter,
                                 _ptr(out_stages), _stream(stream)))


STAGE_ROW_DTYPE = [("max_dur", "<u4"), ("min_start", "<u4"), ("max_end", "<u4"), ("n_waves", "<u4")]
PATH_ROW_DTYPE = [("n_stages", "<u4"), ("last_stage", "<u4"), ("first_start", "<u4"), ("last_end", "<u4"),
                  ("sum_latency", "<u8"), ("bubbles", "<u8")]


def kp_critical_bytes(n_wg: int, n_regions: int) -> int:
    return int(lib().kp_critical_bytes(n_wg, n_regions))


def kp_stages_critical(stages, n_wg: int, n_regions: int, max_iter: int, out_paths, stream=None) -> None:
    _check(lib().kp_stages_critical(_ptr(stages), n_wg, n_regions, max_iter, _ptr(out_paths), _stream(stream)))


def parse_critical(buf, n_wg: int, n_regions: int):
    """Split a critical-path block (host bytes) into (header dict, per-region array[R, 2], rows[n_wg])."""
    b = np.ascontiguousarray(buf.cpu().numpy() if hasattr(buf, "numpy") else buf).view(np.uint8)
    h = b[:64].view("<u8")
    hdr = {"n_wg": int(h[0]), "n_regions": int(h[1]), "max_iter": int(h[2]), "n_paths": int(h[3]),
           "n_path_stages": int(h[4]), "sum_latency": int(h[5]), "sum_bubbles": int(h[6])}
    per_region = b[64 : 64 + 16 * n_regions].view("<u8").reshape(n_regions, 2)
    rows = b[64 + 16 * n_regions : 64 + 16 * n_regions + 32 * n_wg].view(np.dtype(PATH_ROW_DTYPE))
    return hdr, per_region, rows


def parse_stages(buf, n_wg: int, n_regions: int, max_iter: int):
    """Split a stage block (host bytes) into (header dict, table[n_wg, n_regions, max_iter])."""
    b = np.ascontiguousarray(buf.cpu().numpy() if hasattr(buf, "numpy") else buf).view(np.uint8)
    h = b[:32].view("<u8")
    hdr = {"n_rows": int(h[0]), "n_clipped": int(h[1]), "n_bad_region": int(h[2])}
    tab = b[32 : 32 + 16 * n_wg * n_regions * max_iter].view(np.dtype(STAGE_ROW_DTYPE)).reshape(n_wg, n_regions, max_iter)
    return hdr, tab


def kp_gemm_launch_shape(M: int, N: int, K: int) -> tuple[int, int, int]:
    a, b, c = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    _check(lib().kp_gemm_launch_shape(M, N, K, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)))
    return a.value, b.value, c.value


def kp_gemm_instrumented(A, B, C, M: int, N: int, K: int, region_mask: int, trace_buf, trace_cap: int,
                         stream=None) -> None:
    _check(lib().kp_gemm_instrumented(_ptr(A), _ptr(B), _ptr(C), M, N, K, region_mask & 0xFFFFFFFF,
                                      _ptr(trace_buf), trace_cap, _stream(stream)))


def kp_attn_launch_shape(B: int, H: int, S: int, D: int) -> tuple[int, int, int]:
    a, b, c = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    _check(lib().kp_attn_launch_shape(B, H, S, D, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)))
    return a.value, b.value, c.value


def kp_attn_instrumented(Q, K, V, O, B: int, H: int, S: int, D: int, causal: bool, scale: float,
                         region_mask: int, trace_buf, trace_cap: int, stream=None) -> None:
    _check(lib().kp_attn_instrumented(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), B, H, S, D, int(bool(causal)),
                                      float(scale), region_mask & 0xFFFFFFFF, _ptr(trace_buf), trace_cap,
                                      _stream(stream)))


def kp_calibrate(cycles, n_wg: int, waves: int, mode: int, trace_buf, trace_cap: int, stream=None) -> None:
    arr = (ctypes.c_uint32 * len(cycles))(*[int(c) for c in cycles])
    _check(lib().kp_calibrate(arr, len(cycles), n_wg, waves, mode, _ptr(trace_buf), trace_cap, _stream(stream)))


# ---- views of the statistics block (layout documented in include/kperf.h) ------------------------

STATS_HEADER_FIELDS = (
    "n_slots_valid", "n_pairs", "n_orphan_start", "n_orphan_end", "n_invalid", "n_dropped",
    "n_disorder", "n_span_overflow_wgs", "n_nonmonotonic", "n_overlap_wgs", "status",
    "n_wg", "waves_per_wg", "n_regions", "cap_wave", "reserved",
)
WAVE_REGION_DTYPE = np.dtype([("sum", "<u8"), ("n", "<u4"), ("max", "<u4")])


def parse_stats(buf) -> dict:
    """Split a statistics block (bytes on the host: numpy uint8 array or CPU tensor) into fields."""
    if hasattr(buf, "numpy"):
        buf = buf.cpu().numpy()
    b = np.ascontiguousarray(buf).view(np.uint8)
    hdr = b[:128].view("<u8")
    out = {k: int(hdr[i]) for i, k in enumerate(STATS_HEADER_FIELDS)}
    n_wg, W, R = out["n_wg"], out["waves_per_wg"], out["n_regions"]
    pos = 128
    for name, count, dt, shape in (
        ("hist", 64 * R, "<u8", (R, 64)), ("cnt", R, "<u8", (R,)), ("sum", R, "<u8", (R,)),
        ("min", R, "<u8", (R,)), ("max", R, "<u8", (R,)), ("U", R, "<u8", (R,)),
        ("O", R * R, "<u8", (R, R)), ("F", R * R, "<f8", (R, R)),
    ):
        out[name] = b[pos : pos + 8 * count].view(dt).reshape(shape)
        pos += 8 * count
    out["per"] = b[pos : pos + 16 * n_wg * W * R].view(WAVE_REGION_DTYPE).reshape(n_wg, W, R)
    return out

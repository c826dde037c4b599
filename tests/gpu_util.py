"""Helpers for the GPU parity tests: move a raw trace to the device, run the decoder through the
C ABI binding, bring the statistics block back."""
import numpy as np
import torch

import paper_2505_21661_amd as kp


def geometry(raw: np.ndarray):
    n_wg, W, R, cap, rec_cost, flags = (int(x) for x in raw[2:8])
    return n_wg, W, R, cap, rec_cost, flags


def gpu_decode_bytes(raw: np.ndarray, use_hdr: bool = False, dev_raw=None) -> np.ndarray:
    n_wg, W, R, cap, rec_cost, flags = geometry(raw)
    if dev_raw is None:
        dev_raw = torch.from_numpy(raw.view(np.int32)).cuda()
    out = torch.full((kp.kp_stats_bytes(n_wg, W, R),), 0xAB, dtype=torch.uint8, device="cuda")
    n = n_wg * W * cap
    if use_hdr:
        kp.kp_trace_reduce_hdr(dev_raw, n, kp.make_hdr(n_wg, W, R, cap, rec_cost, flags), out)
    else:
        kp.kp_trace_reduce(dev_raw, n, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def assert_stats_equal(want: np.ndarray, got: np.ndarray, oracle_mod):
    if np.array_equal(want, got):
        return
    a, b = oracle_mod.view_stats(want), kp.parse_stats(got)
    for k in a:
        if isinstance(a[k], int):
            assert a[k] == b[k.replace("waves", "waves_per_wg") if k == "waves" else k], (k, a[k], b.get(k))
    for k in ("hist", "cnt", "sum", "min", "max", "U", "O", "F"):
        assert np.array_equal(a[k], b[k]), (k, a[k], b[k])
    bad = np.argwhere((a["per"]["sum"] != b["per"]["sum"]) | (a["per"]["n"] != b["per"]["n"]) | (a["per"]["max"] != b["per"]["max"]))
    assert bad.size == 0, ("per", bad[:5], a["per"][tuple(bad[0])], b["per"][tuple(bad[0])])
    raise AssertionError("stats blocks differ outside the named fields")

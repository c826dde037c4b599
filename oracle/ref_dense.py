"""CPU oracle for the dense kernels that carry the instrumentation -- TEST INFRASTRUCTURE ONLY.

The instrumented targets are a GEMM and an attention forward pass (the paper's
evaluation profiles GEMM and Flash-Attention kernels, Sec. 5.1 "Benchmarks");
recording timestamps must not change what they compute, so the reference is
simply the textbook definition evaluated in fp64:

  GEMM       C[i,j] = sum_k A[i,k] * B[k,j]
  attention  O = softmax(scale * Q K^T + mask) V, row-wise, mask[i,j] = -inf for j > i
             when causal

numpy's matmul serves as the contraction primitive; there is no blocking,
fusion or online-softmax reordering here.  Shares no code with the HIP library.
"""
from __future__ import annotations

import numpy as np


def _to_f64(x) -> np.ndarray:
    """bf16/float tensors or arrays -> float64 numpy (exact for bf16/fp32 inputs)."""
    if hasattr(x, "detach"):
        import torch

        return x.detach().to("cpu").to(torch.float64).numpy()
    return np.asarray(x, dtype=np.float64)


def bf16_round(x) -> np.ndarray:
    """Round float values to the nearest bfloat16 (ties to even); returns float32 values."""
    f = np.asarray(x, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = ((u + 0x7FFF + lsb) >> 16) << 16
    out = r.astype(np.uint32).view(np.float32)
    return np.where(np.isnan(f), f, out).astype(np.float32)


def ref_gemm(A, B, rows=None) -> np.ndarray:
    """fp64 C = A @ B (A [M,K], B [K,N]); `rows` selects a subset of output rows."""
    a = _to_f64(A)
    b = _to_f64(B)
    if rows is not None:
        a = a[np.asarray(rows)]
    return a @ b


def ref_attn(Q, K, V, causal: bool = True, scale: float | None = None, rows=None) -> np.ndarray:
    """fp64 attention forward for one head.  Q,K,V: [S,D]; returns [len(rows) or S, D]."""
    q = _to_f64(Q)
    k = _to_f64(K)
    v = _to_f64(V)
    S, D = q.shape
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    idx = np.arange(S) if rows is None else np.asarray(rows)
    s = (q[idx] @ k.T) * scale
    if causal:
        j = np.arange(k.shape[0])[None, :]
        s = np.where(j > idx[:, None], -np.inf, s)
    m = s.max(axis=1, keepdims=True)
    p = np.exp(s - m)
    p /= p.sum(axis=1, keepdims=True)
    return p @ v

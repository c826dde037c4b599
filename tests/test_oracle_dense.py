"""Pins for the dense-kernel oracle (GEMM, causal attention forward): closed forms,
special cases and library routines (no GPU)."""
import numpy as np
import torch

import inputs
from oracle import bf16_round, ref_attn, ref_gemm


def test_gemm_identity_and_ones():
    _, b = inputs.gemm_inputs(64, 48, 64, seed=0)
    eye = torch.eye(64, dtype=torch.bfloat16)
    assert np.array_equal(ref_gemm(eye, b), b.double().numpy())
    ones_a = torch.ones(8, 256, dtype=torch.bfloat16)
    ones_b = torch.ones(256, 8, dtype=torch.bfloat16)
    assert np.all(ref_gemm(ones_a, ones_b) == 256.0)


def test_gemm_is_not_transposed():
    a = torch.zeros(2, 3, dtype=torch.bfloat16); a[0, 2] = 1.0      # picks row 2 of B into row 0 of C
    b = torch.arange(12, dtype=torch.float32).reshape(3, 4).to(torch.bfloat16)
    c = ref_gemm(a, b)
    assert c.shape == (2, 4) and c[0].tolist() == [8.0, 9.0, 10.0, 11.0] and not c[1].any()


def test_gemm_matches_library_matmul():
    a, b = inputs.gemm_inputs(96, 80, 160, seed=3, dist="uniform")
    want = torch.matmul(a.double(), b.double()).numpy()
    np.testing.assert_allclose(ref_gemm(a, b), want, rtol=1e-13, atol=1e-13)
    rows = [5, 17, 95]
    np.testing.assert_allclose(ref_gemm(a, b, rows=rows), want[rows], rtol=1e-13, atol=1e-13)


def test_bf16_round_matches_torch():
    x = torch.randn(4096, generator=torch.Generator().manual_seed(1)) * 37.0
    x[:4] = torch.tensor([1.00390625, 1.01171875, -1.00390625, 0.0])  # exact ties and zero
    want = x.to(torch.bfloat16).float().numpy()
    assert np.array_equal(bf16_round(x.numpy()), want)


def test_attention_special_cases():
    q, k, v = inputs.attn_inputs(1, 1, 33, 16, seed=2)
    q, k, v = q[0, 0], k[0, 0], v[0, 0]
    o = ref_attn(q, k, v, causal=True)
    # first query row sees only key 0
    np.testing.assert_allclose(o[0], v[0].double().numpy(), rtol=0, atol=1e-15)
    # constant V rows come back unchanged
    vc = torch.full_like(v, 0.75)
    np.testing.assert_allclose(ref_attn(q, k, vc), 0.75, rtol=1e-14)
    # Q = 0 gives uniform weights over the visible prefix
    o0 = ref_attn(torch.zeros_like(q), k, v, causal=True)
    vd = v.double().numpy()
    want = np.cumsum(vd, axis=0) / np.arange(1, 34)[:, None]
    np.testing.assert_allclose(o0, want, rtol=1e-12, atol=1e-12)
    # without the mask the last row equals the plain mean
    on = ref_attn(torch.zeros_like(q), k, v, causal=False)
    np.testing.assert_allclose(on[0], vd.mean(axis=0), rtol=1e-12, atol=1e-12)


def test_attention_matches_library_sdpa():
    q, k, v = inputs.attn_inputs(1, 2, 70, 32, seed=5)
    for causal in (True, False):
        want = torch.nn.functional.scaled_dot_product_attention(
            q.double(), k.double(), v.double(), is_causal=causal)[0, 1].numpy()
        got = ref_attn(q[0, 1], k[0, 1], v[0, 1], causal=causal)
        np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-12)
        rows = [0, 33, 69]
        np.testing.assert_allclose(ref_attn(q[0, 1], k[0, 1], v[0, 1], causal=causal, rows=rows), want[rows],
                                   rtol=1e-10, atol=1e-12)
    # explicit scale
    want = torch.nn.functional.scaled_dot_product_attention(
        q.double(), k.double(), v.double(), is_causal=True, scale=0.3)[0, 0].numpy()
    np.testing.assert_allclose(ref_attn(q[0, 0], k[0, 0], v[0, 0], scale=0.3), want, rtol=1e-10, atol=1e-12)

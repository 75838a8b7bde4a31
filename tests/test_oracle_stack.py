"""Pins for the oracle's model steps around the path (RMSNorm, projections, SwiGLU, Q/K/V with RoPE)."""
import math

import numpy as np
import torch

from oracle import fusionrag_oracle as orc


def test_rmsnorm_closed_form_and_library():
    x = np.full((2, 8), 3.0)
    g = np.arange(1, 9, dtype=np.float64)
    assert np.allclose(orc.rmsnorm(x, g, 0.0), np.tile(g, (2, 1)), rtol=1e-14)         # x / |x|_rms = 1
    assert np.allclose(orc.rmsnorm(x, g, 7.0), np.tile(g, (2, 1)) * 3.0 / 4.0, rtol=1e-14)   # sqrt(9 + 7) = 4
    rng = np.random.default_rng(0)
    x, g = rng.standard_normal((5, 32)), rng.standard_normal(32)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (32,), torch.from_numpy(g), eps=1e-5).numpy()
    assert np.allclose(orc.rmsnorm(x, g, 1e-5), ref, rtol=1e-12)


def test_linear_and_swiglu_against_library():
    rng = np.random.default_rng(1)
    a, w, r = rng.standard_normal((7, 12)), rng.standard_normal((10, 12)), rng.standard_normal((7, 10))
    ref = torch.nn.functional.linear(torch.from_numpy(a), torch.from_numpy(w)).numpy()
    assert np.allclose(orc.linear(a, w), ref, rtol=1e-12)
    assert np.allclose(orc.linear(a, w, r), ref + r, rtol=1e-12)
    # scalar check of one entry: transposed-operand mistakes fail here
    assert math.isclose(orc.linear(a, w)[2, 3], sum(a[2, t] * w[3, t] for t in range(12)), rel_tol=1e-12)
    gate = torch.nn.functional.linear(torch.from_numpy(a), torch.from_numpy(w[0::2]))
    up = torch.nn.functional.linear(torch.from_numpy(a), torch.from_numpy(w[1::2]))
    assert np.allclose(orc.linear_swiglu(a, w), (torch.nn.functional.silu(gate) * up).numpy(), rtol=1e-12)


def test_qkv_rope_layout_and_positions():
    rng = np.random.default_rng(2)
    Hq, Hkv, d, K, M = 4, 2, 8, 16, 5
    a, w = rng.standard_normal((M, K)), rng.standard_normal(((Hq + 2 * Hkv) * d, K))
    pos = np.array([0, 3, 3, 17, 900])
    q, k, v = orc.qkv_rope(a, w, pos, Hq, Hkv, d, 10000.0)
    y = a @ w.T
    assert np.allclose(v, y[:, (Hq + Hkv) * d:].reshape(M, Hkv, d), rtol=1e-13)          # values are not rotated
    assert np.allclose(q[0], y[0, : Hq * d].reshape(Hq, d), rtol=1e-13)                   # position 0: no rotation
    # head 1 of q, row 3, pair 0 (theta = 1): rotation by 17 rad
    a0, b0 = y[3, d], y[3, d + 1]
    assert np.allclose(q[3, 1, :2], [a0 * math.cos(17) - b0 * math.sin(17), b0 * math.cos(17) + a0 * math.sin(17)], rtol=1e-12)
    # key heads follow the query heads in the weight matrix
    k_plain = y[:, Hq * d: (Hq + Hkv) * d].reshape(M, Hkv, d)
    assert np.allclose(k, orc.rope_rotate(k_plain, pos, 10000.0), rtol=1e-13)
    # rows at the same position get the same rotation
    assert np.allclose(np.linalg.norm(q[1]), np.linalg.norm(y[1, : Hq * d]), rtol=1e-12)

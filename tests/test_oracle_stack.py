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


# ---- selective_prefill_layer (eq. 9 row set through one decoder layer of Sec. 2.1) ------------------------------
def _tiny_layer(seed=0, hidden=8, Hq=2, Hkv=1, d=4, ffn=12, L=11, q_index=(1, 4, 5, 8, 9, 10)):
    rng = np.random.default_rng(seed)
    q_index = np.asarray(q_index, dtype=np.int64)
    R = len(q_index)
    weights = {
        "g1": rng.uniform(0.5, 1.5, hidden), "g2": rng.uniform(0.5, 1.5, hidden),
        "w_qkv": rng.standard_normal(((Hq + 2 * Hkv) * d, hidden)) * 0.5,
        "w_o": rng.standard_normal((hidden, Hq * d)) * 0.5,
        "w_gate_up": rng.standard_normal((2 * ffn, hidden)) * 0.5,
        "w_down": rng.standard_normal((hidden, ffn)) * 0.5,
    }
    h = rng.standard_normal((R, hidden))
    k_cache, v_cache = rng.standard_normal((L, Hkv, d)), rng.standard_normal((L, Hkv, d))
    return dict(h=h, q_index=q_index, k_cache=k_cache, v_cache=v_cache, weights=weights, Hq=Hq, Hkv=Hkv, d=d,
                rope_base=100.0, eps=1e-5)


def _scalar_layer(h, q_index, k_cache, v_cache, weights, Hq, Hkv, d, rope_base, eps):
    """The same layer with every sum written as a Python loop over scalars (no numpy arithmetic on arrays, no call
    into the oracle): pre-norm, projections, rotary pairs (2p, 2p+1) at the row's position, attention over the
    cache with the fed rows' own fresh K/V at their positions, output projection + residual, second norm, gated
    feed-forward (gate and up rows interleaved) + residual."""
    R, hidden = h.shape
    L = k_cache.shape[0]
    G = Hq // Hkv
    ffn = weights["w_down"].shape[1]

    def norm(row, gain):
        ms = sum(v * v for v in row) / len(row)
        return [v / math.sqrt(ms + eps) * g for v, g in zip(row, gain)]

    def matvec(w, x):
        return [sum(w[o][t] * x[t] for t in range(len(x))) for o in range(len(w))]

    def rot(vec, pos):
        out = list(vec)
        for p in range(d // 2):
            ang = pos * rope_base ** (-2.0 * p / d)
            a, b = vec[2 * p], vec[2 * p + 1]
            out[2 * p], out[2 * p + 1] = a * math.cos(ang) - b * math.sin(ang), b * math.cos(ang) + a * math.sin(ang)
        return out

    qs, ks, vs = [], [], []
    for r in range(R):
        y = matvec(weights["w_qkv"], norm(h[r], weights["g1"]))
        qs.append([rot(y[hh * d:(hh + 1) * d], int(q_index[r])) for hh in range(Hq)])
        ks.append([rot(y[(Hq + g) * d:(Hq + g + 1) * d], int(q_index[r])) for g in range(Hkv)])
        vs.append([y[(Hq + Hkv + g) * d:(Hq + Hkv + g + 1) * d] for g in range(Hkv)])
    row_of = {int(p): r for r, p in enumerate(q_index)}
    out = []
    for r in range(R):
        attn = []
        for hh in range(Hq):
            g = hh // G
            logits, vals = [], []
            for j in range(int(q_index[r]) + 1):
                kj = ks[row_of[j]][g] if j in row_of else list(k_cache[j, g])
                vj = vs[row_of[j]][g] if j in row_of else list(v_cache[j, g])
                logits.append(sum(a * b for a, b in zip(qs[r][hh], kj)) / math.sqrt(d))
                vals.append(vj)
            m = max(logits)
            w = [math.exp(s - m) for s in logits]
            z = sum(w)
            attn += [sum(w[j] * vals[j][c] for j in range(len(w))) / z for c in range(d)]
        h1 = [a + b for a, b in zip(matvec(weights["w_o"], attn), h[r])]
        y = matvec(weights["w_gate_up"], norm(h1, weights["g2"]))
        act = [y[2 * j] / (1.0 + math.exp(-y[2 * j])) * y[2 * j + 1] for j in range(ffn)]
        out.append([a + b for a, b in zip(matvec(weights["w_down"], act), h1)])
    return np.array(out), np.array(ks), np.array(vs)


def test_layer_against_scalar_loops():
    for seed, (Hq, Hkv) in enumerate([(2, 1), (2, 2), (4, 2)]):
        t = _tiny_layer(seed=seed, Hq=Hq, Hkv=Hkv)
        got_h, got_k, got_v = orc.selective_prefill_layer(**t)
        want_h, want_k, want_v = _scalar_layer(**t)
        assert np.allclose(got_h, want_h, rtol=1e-11, atol=1e-12)
        assert np.allclose(got_k, want_k, rtol=1e-12) and np.allclose(got_v, want_v, rtol=1e-12)


def test_layer_identities():
    t = _tiny_layer(seed=3)
    full_h, full_k, full_v = orc.selective_prefill_layer(**t)
    # both residual branches switched off: the layer is the identity on the hidden rows
    w0 = dict(t["weights"], w_o=np.zeros_like(t["weights"]["w_o"]), w_down=np.zeros_like(t["weights"]["w_down"]))
    assert np.array_equal(orc.selective_prefill_layer(**dict(t, weights=w0))[0], t["h"])
    # only the feed-forward branch off: what is left is input + attention branch, so the second norm's gain is unused
    w1 = dict(t["weights"], w_down=np.zeros_like(t["weights"]["w_down"]))
    h_a = orc.selective_prefill_layer(**dict(t, weights=w1))[0]
    h_b = orc.selective_prefill_layer(**dict(t, weights=dict(w1, g2=w1["g2"] * 3.0)))[0]
    assert np.array_equal(h_a, h_b) and not np.allclose(h_a, t["h"])
    # a subset of rows equals the same rows of the full call; K/V are always those of every fed row
    rows = np.array([4, 0, 3])
    sub_h, sub_k, sub_v = orc.selective_prefill_layer(**t, rows=rows)
    assert np.allclose(sub_h, full_h[rows], rtol=1e-13) and np.array_equal(sub_k, full_k) and np.array_equal(sub_v, full_v)
    # an identity round_fn changes nothing; a real one is applied to what a pipeline stores
    same = orc.selective_prefill_layer(**t, round_fn=lambda a: a)
    assert all(np.array_equal(a, b) for a, b in zip(same, (full_h, full_k, full_v)))
    calls = []
    orc.selective_prefill_layer(**t, round_fn=lambda a: (calls.append(a.shape), a)[1])
    R, hidden = t["h"].shape
    assert calls.count((R, hidden)) == 4 and len(calls) == 9   # x, q, k, v, attn, h1, x2, act, h2
    # the stale cache entries of the fed tokens are never used
    kc = t["k_cache"].copy()
    kc[t["q_index"]] = 1e6
    assert np.allclose(orc.selective_prefill_layer(**dict(t, k_cache=kc))[0], full_h, rtol=1e-13)


def test_layer_with_every_row_fed_is_a_dense_decoder_layer():
    """Every position in the Q index (100 % recompute plus the question): the cache contents are irrelevant and the
    layer is an ordinary pre-norm decoder layer, here composed from torch's float64 library routines (rms_norm, linear,
    scaled_dot_product_attention with is_causal, silu) and a complex-number rotary embedding."""
    F = torch.nn.functional
    t = _tiny_layer(seed=4, Hq=4, Hkv=2, L=9, q_index=tuple(range(9)))
    w = {k: torch.from_numpy(v) for k, v in t["weights"].items()}
    h = torch.from_numpy(t["h"])
    Hq, Hkv, d, L = t["Hq"], t["Hkv"], t["d"], 9

    def rope(x):   # [L, heads, d], pairs (2p, 2p+1) as one complex number times exp(i pos theta_p)
        theta = t["rope_base"] ** (-2.0 * torch.arange(d // 2, dtype=torch.float64) / d)
        z = torch.view_as_complex(x.reshape(L, -1, d // 2, 2).contiguous())
        z = z * torch.polar(torch.ones(L, 1, d // 2, dtype=torch.float64), torch.arange(L, dtype=torch.float64)[:, None, None] * theta)
        return torch.view_as_real(z).reshape(L, -1, d)

    y = F.linear(F.rms_norm(h, (h.shape[1],), w["g1"], eps=t["eps"]), w["w_qkv"])
    q = rope(y[:, : Hq * d].reshape(L, Hq, d))
    k = rope(y[:, Hq * d:(Hq + Hkv) * d].reshape(L, Hkv, d))
    v = y[:, (Hq + Hkv) * d:].reshape(L, Hkv, d)
    kr, vr = k.repeat_interleave(Hq // Hkv, dim=1), v.repeat_interleave(Hq // Hkv, dim=1)
    attn = F.scaled_dot_product_attention(q.transpose(0, 1)[None], kr.transpose(0, 1)[None], vr.transpose(0, 1)[None],
                                          is_causal=True)[0].transpose(0, 1).reshape(L, Hq * d)
    h1 = h + F.linear(attn, w["w_o"])
    gu = F.linear(F.rms_norm(h1, (h.shape[1],), w["g2"], eps=t["eps"]), w["w_gate_up"])
    want = h1 + F.linear(F.silu(gu[:, 0::2]) * gu[:, 1::2], w["w_down"])
    got_h, got_k, got_v = orc.selective_prefill_layer(**t)
    assert np.allclose(got_h, want.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(got_k, k.numpy(), rtol=1e-11) and np.allclose(got_v, v.numpy(), rtol=1e-11)
    # and with garbage in the cache: same result (eq. 9 at 100 % is full prefill)
    junk = dict(t, k_cache=t["k_cache"] * 7 + 3, v_cache=t["v_cache"] * -2)
    assert np.allclose(orc.selective_prefill_layer(**junk)[0], got_h, rtol=1e-13)

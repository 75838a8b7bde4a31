"""Pins for the oracle's sparse prefill attention (eq. 9, Sec. 4.3), scatter and full attention (eq. 2)."""
import math

import numpy as np
import pytest
import scipy.special
import torch

from oracle import fusionrag_oracle as orc
from tests.conftest import read_golden_table


def brute_attention_row(qvec, keys, vals):
    """One query against explicit lists of keys/values, scalar loops."""
    d = len(qvec)
    logit = [sum(qvec[t] * kk[t] for t in range(d)) / math.sqrt(d) for kk in keys]
    mx = max(logit)
    w = [math.exp(x - mx) for x in logit]
    z = sum(w)
    return [sum(w[j] * vals[j][t] for j in range(len(keys))) / z for t in range(d)], mx + math.log(z)


def make_case(rng, L_ctx=13, nq=3, Hq=4, Hkv=2, d=8, k=4):
    L = L_ctx + nq
    q_full = rng.standard_normal((L, Hq, d))
    k_full = rng.standard_normal((L, Hkv, d))
    v_full = rng.standard_normal((L, Hkv, d))
    k_cache = rng.standard_normal((L, Hkv, d))
    v_cache = rng.standard_normal((L, Hkv, d))
    sel = np.sort(rng.choice(L_ctx, size=k, replace=False))
    qi = np.concatenate([sel, L_ctx + np.arange(nq)])
    return q_full, k_full, v_full, k_cache, v_cache, qi


def test_sparse_attention_brute_force():
    rng = np.random.default_rng(0)
    q_full, k_full, v_full, k_cache, v_cache, qi = make_case(rng)
    out, lse = orc.sparse_prefill_attn(q_full[qi], qi, k_cache, v_cache, k_full[qi], v_full[qi])
    Hq, Hkv = q_full.shape[1], k_full.shape[1]
    G = Hq // Hkv
    recomputed = {int(p): r for r, p in enumerate(qi)}
    for r, p in enumerate(qi):
        for h in range(Hq):
            g = h // G
            keys, vals = [], []
            for j in range(int(p) + 1):                     # up to and including own position
                if j in recomputed:                          # fresh entry replaces the stale one
                    keys.append(k_full[qi[recomputed[j]], g]); vals.append(v_full[qi[recomputed[j]], g])
                else:
                    keys.append(k_cache[j, g]); vals.append(v_cache[j, g])
            want, want_lse = brute_attention_row(q_full[p, h], keys, vals)
            assert np.allclose(out[r, h], want, rtol=1e-12, atol=1e-13)
            assert math.isclose(lse[r, h], want_lse, rel_tol=1e-12)


def test_full_causal_brute_force_and_torch_sdpa():
    rng = np.random.default_rng(1)
    L, Hq, Hkv, d = 9, 4, 2, 8
    q, k, v = rng.standard_normal((L, Hq, d)), rng.standard_normal((L, Hkv, d)), rng.standard_normal((L, Hkv, d))
    out = orc.full_causal_attention(q, k, v)
    for i in range(L):
        for h in range(Hq):
            want, _ = brute_attention_row(q[i, h], list(k[: i + 1, h // 2]), list(v[: i + 1, h // 2]))
            assert np.allclose(out[i, h], want, rtol=1e-12, atol=1e-13)
    # third opinion: the library's scaled-dot-product attention in float64
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(np.repeat(k, 2, axis=1)).permute(1, 0, 2)[None]
    tv = torch.from_numpy(np.repeat(v, 2, axis=1)).permute(1, 0, 2)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).numpy()
    assert np.allclose(out, ref, rtol=1e-10, atol=1e-12)


def test_recomputing_everything_is_full_prefill():
    # ratio 100 %: whatever the stale cache holds, the result is full causal attention (eq. 2)
    rng = np.random.default_rng(2)
    q_full, k_full, v_full, k_cache, v_cache, _ = make_case(rng, L_ctx=20, nq=4)
    L = q_full.shape[0]
    qi = np.arange(L)
    out, _ = orc.sparse_prefill_attn(q_full, qi, k_cache * 100.0, v_cache - 7.0, k_full, v_full)
    assert np.allclose(out, orc.full_causal_attention(q_full, k_full, v_full), rtol=1e-11, atol=1e-12)


def test_recomputing_nothing_is_question_only_prefill():
    # ratio 0 % (Full Reuse, eq. 6): the question rows attend to the stitched cache and to themselves
    rng = np.random.default_rng(3)
    q_full, k_full, v_full, k_cache, v_cache, _ = make_case(rng, L_ctx=15, nq=5)
    L_ctx, L = 15, 20
    qi = L_ctx + np.arange(5)
    out, _ = orc.sparse_prefill_attn(q_full[qi], qi, k_cache, v_cache, k_full[qi], v_full[qi])
    k_all = np.concatenate([k_cache[:L_ctx], k_full[L_ctx:]])
    v_all = np.concatenate([v_cache[:L_ctx], v_full[L_ctx:]])
    assert np.allclose(out, orc.full_causal_attention(q_full, k_all, v_all)[L_ctx:], rtol=1e-11, atol=1e-12)


def test_sparse_rows_are_rows_of_dense_attention_over_effective_kv():
    rng = np.random.default_rng(4)
    q_full, k_full, v_full, k_cache, v_cache, qi = make_case(rng, L_ctx=30, nq=6, k=9)
    out, _ = orc.sparse_prefill_attn(q_full[qi], qi, k_cache, v_cache, k_full[qi], v_full[qi])
    k_eff, v_eff = orc.effective_kv(qi, k_cache, v_cache, k_full[qi], v_full[qi])
    dense = orc.full_causal_attention(q_full, k_eff, v_eff)
    assert np.allclose(out, dense[qi], rtol=1e-11, atol=1e-12)
    # the row subset argument computes the same rows
    sub = np.array([0, 3, 14])
    out_sub, _ = orc.sparse_prefill_attn(q_full[qi], qi, k_cache, v_cache, k_full[qi], v_full[qi], rows=sub)
    assert np.allclose(out_sub, out[sub], rtol=1e-13)
    # k_new = None: the cache already holds the fresh entries
    out2, _ = orc.sparse_prefill_attn(q_full[qi], qi, k_eff, v_eff, None, None)
    assert np.allclose(out2, out, rtol=1e-13)


def test_weights_sum_to_one_and_lse():
    rng = np.random.default_rng(5)
    q_full, k_full, v_full, k_cache, v_cache, qi = make_case(rng, Hq=2, Hkv=2)
    ones = np.ones_like(v_cache)
    out, lse = orc.sparse_prefill_attn(q_full[qi], qi, k_cache, ones, k_full[qi], ones[qi])
    assert np.allclose(out, 1.0, rtol=1e-13)                 # V = 1 -> every output is the weight sum
    k_eff, _ = orc.effective_kv(qi, k_cache, v_cache, k_full[qi], v_full[qi])
    for r, p in enumerate(qi):
        for h in range(2):
            logits = k_eff[: p + 1, h] @ q_full[p, h] / math.sqrt(8)
            assert math.isclose(lse[r, h], scipy.special.logsumexp(logits), rel_tol=1e-12)


def test_mha_is_gqa_with_repeated_heads():
    rng = np.random.default_rng(6)
    q_full, k_full, v_full, k_cache, v_cache, qi = make_case(rng, Hq=4, Hkv=2)
    rep = lambda a: np.repeat(a, 2, axis=1)
    a, _ = orc.sparse_prefill_attn(q_full[qi], qi, k_cache, v_cache, k_full[qi], v_full[qi])
    b, _ = orc.sparse_prefill_attn(q_full[qi], qi, rep(k_cache), rep(v_cache), rep(k_full[qi]), rep(v_full[qi]))
    assert np.allclose(a, b, rtol=1e-13)


def test_worked_mask_example():
    rows = read_golden_table("sparse_prefill_mask_example.txt")
    pos_1based = [int(v) for v in rows[0][1:]]
    want = np.array([[int(v) for v in r] for r in rows[1:]], dtype=bool)
    got = orc.visibility(np.array(pos_1based) - 1, want.shape[1])
    assert got.shape == (4, 8) and np.array_equal(got, want)
    # first row as the paper prints it: X[3] sees X[1:3] and nothing of X[4:8]
    assert got[0, :3].all() and not got[0, 3:].any()


def test_scatter_exact_untouched_idempotent():
    rng = np.random.default_rng(7)
    q_full, k_full, v_full, k_cache, v_cache, qi = make_case(rng)
    k1, v1 = orc.kv_scatter(qi, k_full[qi], v_full[qi], k_cache, v_cache)
    assert np.array_equal(k1[qi], k_full[qi]) and np.array_equal(v1[qi], v_full[qi])
    rest = np.setdiff1d(np.arange(k_cache.shape[0]), qi)
    assert np.array_equal(k1[rest], k_cache[rest]) and np.array_equal(v1[rest], v_cache[rest])
    k2, v2 = orc.kv_scatter(qi, k_full[qi], v_full[qi], k1, v1)
    assert np.array_equal(k2, k1) and np.array_equal(v2, v1)
    # scatter-then-attend over the plain cache equals attending with the fresh rows passed in
    a, _ = orc.sparse_prefill_attn(q_full[qi], qi, k_cache, v_cache, k_full[qi], v_full[qi])
    b, _ = orc.sparse_prefill_attn(q_full[qi], qi, k1, v1, None, None)
    assert np.allclose(a, b, rtol=1e-13)


def test_offline_preprocess_attn_pins():
    """eq. 10 against three things it must reduce to."""
    rng = np.random.default_rng(11)
    Hq, Hkv, d, P, n = 4, 2, 8, 13, 6
    q = rng.standard_normal((P + n, Hq, d))
    k = rng.standard_normal((P + n, Hkv, d))
    v = rng.standard_normal((P + n, Hkv, d))
    got = orc.offline_preprocess_attn(q[P:], k[P:], v[P:], k[:P], v[:P])
    # (1) the last n rows of ordinary causal attention over cat(prefix, chunk)
    assert np.allclose(got, orc.full_causal_attention(q, k, v)[P:], rtol=1e-12, atol=1e-12)
    # (2) no prefix: causal attention of the chunk alone
    empty = np.zeros((0, Hkv, d))
    assert np.allclose(orc.offline_preprocess_attn(q[P:], k[P:], v[P:], empty, empty),
                       orc.full_causal_attention(q[P:], k[P:], v[P:]), rtol=1e-12, atol=1e-12)
    # (3) the sparse prefill with no context token chosen: Q index = the chunk's own positions
    qi = np.arange(P, P + n)
    cache_k = np.concatenate([k[:P], rng.standard_normal((n, Hkv, d))])     # reserved rows: never read
    cache_v = np.concatenate([v[:P], rng.standard_normal((n, Hkv, d))])
    sp, _ = orc.sparse_prefill_attn(q[P:], qi, cache_k, cache_v, k[P:], v[P:])
    assert np.allclose(got, sp, rtol=1e-12, atol=1e-12)
    # first chunk token with a one-entry prefix: two keys, weights by hand
    q1, k1, v1 = q[P:P + 1], k[P:P + 1], v[P:P + 1]
    o = orc.offline_preprocess_attn(q1, k1, v1, k[:1], v[:1])
    s0, s1 = (k[0, 0] @ q1[0, 0]) / np.sqrt(d), (k1[0, 0] @ q1[0, 0]) / np.sqrt(d)
    w0 = 1.0 / (1.0 + np.exp(s1 - s0))
    assert np.allclose(o[0, 0], w0 * v[0, 0] + (1.0 - w0) * v1[0, 0], rtol=1e-12)

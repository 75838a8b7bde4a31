"""Pins of the batch-decoding oracle (Sec. 4.3): it must agree with the prefill path's definitions."""
import numpy as np

from oracle import fusionrag_oracle as orc

BASE = 10000.0


def _setup(rng, Hq=4, Hkv=2, d=8, lens=(5, 7, 4), src_pos0=(0, 3, 11), nq=3, n_gen=2, crit=(2, 6, 13)):
    """One query whose prompt is chunks 0..2 of a small store, placed back to back; it recomputed the tokens
    `crit` (prompt positions), then its question, then generated n_gen tokens (the last one is decoding)."""
    offs = np.concatenate([[0], np.cumsum(lens)])
    L_ctx = int(offs[-1])
    k_store = rng.standard_normal((L_ctx, Hkv, d))           # as cached: chunk c at positions src_pos0[c] ..
    v_store = rng.standard_normal((L_ctx, Hkv, d))
    L = L_ctx + nq + n_gen
    q_all = rng.standard_normal((L, Hq, d))                  # everything below is at prompt positions
    k_fresh = rng.standard_normal((L, Hkv, d))
    v_fresh = rng.standard_normal((L, Hkv, d))
    return offs, L_ctx, L, k_store, v_store, q_all, k_fresh, v_fresh, np.asarray(src_pos0), np.asarray(crit)


def test_decode_is_the_last_row_of_causal_attention_over_the_effective_cache():
    rng = np.random.default_rng(21)
    offs, L_ctx, L, k_store, v_store, q_all, k_fresh, v_fresh, src, crit = _setup(rng)
    # prefill path: shift the chunk keys to their prompt positions, replace the critical rows, append the rest
    k_ctx = orc.rope_shift(k_store, offs, src, None, BASE)
    qi = np.concatenate([crit, np.arange(L_ctx, L)])
    k_cache = np.concatenate([k_ctx, np.zeros((L - L_ctx,) + k_ctx.shape[1:])])
    v_cache = np.concatenate([v_store, np.zeros((L - L_ctx,) + k_ctx.shape[1:])])
    k_eff, v_eff = orc.effective_kv(qi, k_cache, v_cache, k_fresh[qi], v_fresh[qi])
    want = orc.full_causal_attention(q_all, k_eff, v_eff)[-1]
    # decode path: shared store untouched, critical rows masked, page = fresh critical + question + generated
    segs = [[(int(offs[c]), int(offs[c + 1] - offs[c]), int(offs[c] - src[c])) for c in range(len(src))]]
    got, lse = orc.decode_attn(q_all[-1:], k_store, v_store, segs, [crit], [k_fresh[qi]], [v_fresh[qi]], BASE)
    assert np.allclose(got[0], want, rtol=1e-11, atol=1e-12)
    # lse against the prefill oracle's own log-sum-exp of the last row
    _, lse_pf = orc.sparse_prefill_attn(q_all[qi], qi, k_cache, v_cache, k_fresh[qi], v_fresh[qi], rows=[len(qi) - 1])
    assert np.allclose(lse[0], lse_pf[0], rtol=1e-11)


def test_decode_brute_force_and_invariances():
    rng = np.random.default_rng(22)
    Hq, Hkv, d = 2, 1, 4
    k_store = rng.standard_normal((6, Hkv, d))
    v_store = rng.standard_normal((6, Hkv, d))
    k_page = rng.standard_normal((2, Hkv, d))
    v_page = rng.standard_normal((2, Hkv, d))
    q = rng.standard_normal((1, Hq, d))
    segs = [[(0, 3, 5), (3, 3, -2)]]
    stale = [[1, 4]]
    got, _ = orc.decode_attn(q, k_store, v_store, segs, stale, [k_page], [v_page], BASE)
    # scalar loops, rotation written out pair by pair
    theta = BASE ** (-2.0 * np.arange(d // 2) / d)
    for h in range(Hq):
        num, den = np.zeros(d), 0.0
        items = []
        for (row0, n, delta) in segs[0]:
            for r in range(row0, row0 + n):
                if r in stale[0]:
                    continue
                k = k_store[r, 0].copy()
                for p_ in range(d // 2):
                    c, s_ = np.cos(delta * theta[p_]), np.sin(delta * theta[p_])
                    a, b_ = k[2 * p_], k[2 * p_ + 1]
                    k[2 * p_], k[2 * p_ + 1] = a * c - b_ * s_, b_ * c + a * s_
                items.append((k, v_store[r, 0]))
        items += [(k_page[i, 0], v_page[i, 0]) for i in range(2)]
        for k, v in items:
            w = np.exp(float(k @ q[0, h]) / np.sqrt(d))
            num += w * v
            den += w
        assert np.allclose(got[0, h], num / den, rtol=1e-12)
    # the order of the segments does not matter; the content of a stale row does not matter
    got2, _ = orc.decode_attn(q, k_store, v_store, [segs[0][::-1]], stale, [k_page], [v_page], BASE)
    assert np.allclose(got, got2, rtol=1e-12)
    k_poison = k_store.copy()
    k_poison[[1, 4]] = 1e6
    got3, _ = orc.decode_attn(q, k_poison, v_store, segs, stale, [k_page], [v_page], BASE)
    assert np.array_equal(got, got3)
    # two queries that share the store but mask different rows get different results, each equal to its solo run
    gotb, _ = orc.decode_attn(np.concatenate([q, q]), k_store, v_store, [segs[0], segs[0]], [[1, 4], [0]],
                              [k_page, k_page], [v_page, v_page], BASE)
    solo, _ = orc.decode_attn(q, k_store, v_store, segs, [[0]], [k_page], [v_page], BASE)
    assert np.allclose(gotb[0], got[0]) and np.allclose(gotb[1], solo[0]) and not np.allclose(gotb[0], gotb[1])

"""CPU oracle for the online selective-prefill path of FusionRAG (arXiv 2601.12904).

TEST INFRASTRUCTURE ONLY.  Plain numpy in float64, written from the paper's
definitions with no blocking, fusion or reordering, so it can be checked against
the paper by eye.  Only the test-suite, the smoke check and the benchmark's
``cpu_baseline`` leg may import it; the HIP library never does, shares no code
with it, and the oracle imports nothing from the HIP package.

Conventions (the paper counts tokens from 1; everything here counts from 0):

* tensors are token-major ``[tokens, heads, head_dim]``;
* query head ``h`` reads KV head ``h // G`` with ``G = Hq // Hkv`` (the grouped-query
  convention of the Llama / Qwen / Mistral models the paper runs, Sec. 5.1);
* attention logits are scaled by ``1/sqrt(head_dim)`` (Sec. 2.1).

Pins (see tests/test_oracle_*.py): every function below is pinned to a closed form,
a brute-force loop, a library routine or a worked example of the paper; what cannot
be pinned is which of the readings listed in the design notes the authors' own code
used -- parity with the authors' implementation is unpinned, parity with the paper's
stated definitions is pinned.
"""
from __future__ import annotations

import math
from typing import Optional, Sequence

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------------------
# recompute budget
# --------------------------------------------------------------------------------------
def topk_count(L_ctx: int, ratio: float) -> int:
    """Number of context tokens to recompute for a recompute ratio (Sec. 1.1, Sec. 5.4:
    the ratio is the share of tokens recomputed; the question is always computed and is
    not part of the base).  Round half up, clamped to [0, L_ctx]."""
    k = int(math.floor(ratio * L_ctx + 0.5))
    return max(0, min(int(L_ctx), k))


# --------------------------------------------------------------------------------------
# Appendix A: rotary position recovery
# --------------------------------------------------------------------------------------
def rope_frequencies(d: int, base: float, index_base: int = 0) -> np.ndarray:
    """theta_p for the d/2 rotary pairs.  ``index_base=1`` is the appendix's printed form
    theta_i = base^(-2i/d), i = 1..d/2 (Appendix A, frequency definition); ``index_base=0`` is the usual
    theta_p = base^(-2p/d), p = 0..d/2-1 that the cached keys of a real model carry."""
    p = np.arange(d // 2, dtype=F64) + index_base
    return np.asarray(base, dtype=F64) ** (-2.0 * p / d)


def _pair_views(x: np.ndarray, layout: str):
    d = x.shape[-1]
    if layout == "interleaved":            # pairs (0,1), (2,3), ...: theta = [t1,t1,t2,t2,...] (Appendix A)
        return x[..., 0::2], x[..., 1::2]
    if layout == "half":                   # pairs (p, p + d/2)
        return x[..., : d // 2], x[..., d // 2:]
    raise ValueError(layout)


def rope_rotate(x: np.ndarray, positions: np.ndarray, base: float, layout: str = "interleaved",
                index_base: int = 0) -> np.ndarray:
    """RoPE(x, s) = x * cos(s theta) + rotate(x) * sin(s theta) with
    rotate(x) = [-x2, x1, -x4, x3, ...] (Appendix A, definition), one position ``s`` per token row."""
    x = np.asarray(x, dtype=F64)
    d = x.shape[-1]
    theta = rope_frequencies(d, base, index_base)                   # [d/2]
    ang = np.asarray(positions, dtype=F64)[:, None, None] * theta   # [T, 1, d/2]
    c, s = np.cos(ang), np.sin(ang)
    a, b = _pair_views(x, layout)
    out = np.empty_like(x)
    oa, ob = _pair_views(out, layout)
    oa[...] = a * c - b * s
    ob[...] = b * c + a * s
    return out


def rope_shift(k_cached: np.ndarray, chunk_offsets: Sequence[int], src_pos0: Sequence[int],
               dst_pos0: Optional[Sequence[int]], base: float, layout: str = "interleaved",
               index_base: int = 0, dst_base: int = 0) -> np.ndarray:
    """Move every cached chunk's keys from the positions they were cached at to their
    positions in the assembled prompt (Sec. 2.2.1 footnote, Appendix A).  Because RoPE is
    additive (Appendix A, proof) a key cached at position s1 reaches position s2 by one more
    rotation by s2 - s1; all tokens of chunk c share Delta_c = dst_pos0[c] - src_pos0[c]
    (Appendix A's example: [2,3,4,5] -> [5,6,7,8], Delta = 3).  Values are untouched.
    ``dst_pos0 = None`` means the chunk lands at ``chunk_offsets[c] + dst_base``."""
    k_cached = np.asarray(k_cached, dtype=F64)
    offs = np.asarray(chunk_offsets, dtype=np.int64)
    C = len(offs) - 1
    dst = offs[:-1] + dst_base if dst_pos0 is None else np.asarray(dst_pos0, dtype=np.int64)
    src = np.asarray(src_pos0, dtype=np.int64)
    out = np.empty_like(k_cached)
    for c in range(C):
        s, e = int(offs[c]), int(offs[c + 1])
        delta = np.full(e - s, dst[c] - src[c], dtype=np.int64)
        out[s:e] = rope_rotate(k_cached[s:e], delta, base, layout, index_base)
    return out


# --------------------------------------------------------------------------------------
# Sec. 3.2: Query-Guided Selection
# --------------------------------------------------------------------------------------
def critical_scores(q_question: np.ndarray, k_ctx: np.ndarray, chunk_offsets: Sequence[int],
                    norm: str = "per_chunk") -> np.ndarray:
    """Critical score of every context token (Sec. 3.2): for each chunk, the attention-weight
    matrix between the question's queries (rows) and the chunk's keys (columns); the score of
    a token is the sum of its column, accumulated over all query heads.

    ``norm`` is the reading of "attention weights" (Sec. 2.1 calls softmax outputs weights):
      per_chunk  softmax over the columns of the chunk's own matrix (default: the matrix is
                 built per chunk, so each of its rows sums to one);
      global     one softmax over all context keys;
      raw        no softmax: the scaled logits themselves (the literal "multiplying").
    """
    q = np.asarray(q_question, dtype=F64)
    k = np.asarray(k_ctx, dtype=F64)
    nq, Hq, d = q.shape
    L_ctx, Hkv, _ = k.shape
    G = Hq // Hkv
    offs = np.asarray(chunk_offsets, dtype=np.int64)
    assert offs[0] == 0 and offs[-1] == L_ctx
    scores = np.zeros(L_ctx, dtype=F64)
    for h in range(Hq):
        logits = (q[:, h, :] @ k[:, h // G, :].T) / math.sqrt(d)        # [nq, L_ctx]
        if norm == "raw":
            scores += logits.sum(axis=0)
        elif norm == "global":
            w = np.exp(logits - logits.max(axis=1, keepdims=True))
            w /= w.sum(axis=1, keepdims=True)
            scores += w.sum(axis=0)
        elif norm == "per_chunk":
            for c in range(len(offs) - 1):
                s, e = int(offs[c]), int(offs[c + 1])
                if e == s:
                    continue
                blk = logits[:, s:e]
                w = np.exp(blk - blk.max(axis=1, keepdims=True))
                w /= w.sum(axis=1, keepdims=True)
                scores[s:e] += w.sum(axis=0)
        else:
            raise ValueError(norm)
    return scores


def select_q_index(scores: np.ndarray, k: int, nq: int) -> np.ndarray:
    """argTopk of the critical scores (Table 1, Sec. 3.2) followed by the Q index of
    Sec. 4.3: the ascending list of the tokens computed in this step = the k critical
    context tokens, then the nq question tokens (positions L_ctx .. L_ctx+nq-1).
    Equal scores: the lower index wins."""
    scores = np.asarray(scores)
    L_ctx = scores.shape[0]
    assert 0 <= k <= L_ctx
    order = np.lexsort((np.arange(L_ctx), -scores))     # score descending, then index ascending
    sel = np.sort(order[:k])
    return np.concatenate([sel, L_ctx + np.arange(nq)]).astype(np.int64)


# --------------------------------------------------------------------------------------
# eq. 9 / Sec. 4.3: sparse prefill over the assembled cache
# --------------------------------------------------------------------------------------
def effective_kv(q_index: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray,
                 k_new: np.ndarray, v_new: np.ndarray):
    """The K/V every computed row attends to: the assembled cache with the entries of the
    recomputed tokens replaced by their fresh K/V (Sec. 4.3: stale entries of critical tokens
    are excluded and the newly computed ones are used instead)."""
    k_eff = np.array(k_cache, dtype=F64, copy=True)
    v_eff = np.array(v_cache, dtype=F64, copy=True)
    k_eff[q_index] = np.asarray(k_new, dtype=F64)
    v_eff[q_index] = np.asarray(v_new, dtype=F64)
    return k_eff, v_eff


def visibility(q_index: np.ndarray, L: int) -> np.ndarray:
    """Boolean [R, L]: row r (token at position q_index[r]) sees key j iff j <= q_index[r]
    (Sec. 2.2.2: each token attends to those up to and including its own position; in the
    worked example X[3] sees X[1:3])."""
    return np.arange(L)[None, :] <= np.asarray(q_index)[:, None]


def sparse_prefill_attn(q_rows: np.ndarray, q_index: np.ndarray, k_cache: np.ndarray,
                        v_cache: np.ndarray, k_new: Optional[np.ndarray], v_new: Optional[np.ndarray],
                        rows: Optional[np.ndarray] = None):
    """Attention of the computed rows only (eq. 9): row r holds the query of the token at
    position q_index[r]; it attends causally, by position, to the effective K/V.
    Returns (O [R', Hq, d], lse [R', Hq]) for ``rows`` (default: all R rows).
    ``k_new = None`` means the cache already holds the fresh entries."""
    q_index = np.asarray(q_index, dtype=np.int64)
    if k_new is None:
        k_eff, v_eff = np.asarray(k_cache, dtype=F64), np.asarray(v_cache, dtype=F64)
    else:
        k_eff, v_eff = effective_kv(q_index, k_cache, v_cache, k_new, v_new)
    q = np.asarray(q_rows, dtype=F64)
    if rows is not None:
        rows = np.asarray(rows, dtype=np.int64)
        q, pos = q[rows], q_index[rows]
    else:
        pos = q_index
    R, Hq, d = q.shape
    L, Hkv, _ = k_eff.shape
    G = Hq // Hkv
    vis = visibility(pos, L)                                            # [R, L]
    out = np.empty((R, Hq, d), dtype=F64)
    lse = np.empty((R, Hq), dtype=F64)
    for h in range(Hq):
        g = h // G
        s = (q[:, h, :] @ k_eff[:, g, :].T) / math.sqrt(d)              # [R, L]
        s = np.where(vis, s, -np.inf)
        m = s.max(axis=1, keepdims=True)
        p = np.exp(s - m)
        l = p.sum(axis=1, keepdims=True)
        out[:, h, :] = (p / l) @ v_eff[:, g, :]
        lse[:, h] = (m + np.log(l))[:, 0]
    return out, lse


def kv_scatter(q_index: np.ndarray, k_new: np.ndarray, v_new: np.ndarray,
               k_cache: np.ndarray, v_cache: np.ndarray):
    """Place the recomputed K/V at their tokens' rows of the cache (Sec. 4.3, last step of the
    worked example).  Returns new arrays; exact copies, no arithmetic."""
    k_out, v_out = np.array(k_cache, copy=True), np.array(v_cache, copy=True)
    q_index = np.asarray(q_index, dtype=np.int64)
    k_out[q_index] = k_new
    v_out[q_index] = v_new
    return k_out, v_out


# --------------------------------------------------------------------------------------
# eq. 2: Full Attention, written separately from the sparse routine (row by row, no mask
# array) so that the two can be checked against each other
# --------------------------------------------------------------------------------------
def full_causal_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray) -> np.ndarray:
    """Ordinary causal prefill attention over the whole prompt (eq. 2): token i attends to
    tokens 0..i."""
    q, k, v = (np.asarray(a, dtype=F64) for a in (q, k, v))
    L, Hq, d = q.shape
    G = Hq // k.shape[1]
    out = np.empty_like(q)
    for h in range(Hq):
        kh, vh = k[:, h // G, :], v[:, h // G, :]
        for i in range(L):
            s = kh[: i + 1] @ q[i, h] / math.sqrt(d)
            w = np.exp(s - s.max())
            out[i, h] = (w / w.sum()) @ vh[: i + 1]
    return out


# --------------------------------------------------------------------------------------
# Sec. 4.3: batch decoding over shared chunk caches and per-query exclusive pages
# --------------------------------------------------------------------------------------
def decode_attn(q: np.ndarray, k_shared: np.ndarray, v_shared: np.ndarray, segments: Sequence[Sequence[tuple]],
                stale_rows: Sequence[Sequence[int]], k_pages: Sequence[np.ndarray], v_pages: Sequence[np.ndarray],
                base: float, layout: str = "interleaved", index_base: int = 0):
    """One decoding step for a batch of queries (Sec. 2.1: the last token attends to all past
    K/V; Sec. 4.3: the chunk caches are shared by the batch and never modified, every query keeps
    the recomputed K/V of its critical tokens, of its question and of its generated tokens in an
    exclusive page, and the shared entries of its critical tokens are masked out).

    q [B, Hq, d]: the decoding token's queries, rotated at their positions.
    k_shared / v_shared [N, Hkv, d]: the chunk store as cached.  ``segments[b]`` lists
    (row0, length, delta): query b's prompt contains store rows [row0, row0 + length), and their
    keys, cached ``delta`` positions away from where they sit in this prompt, are first moved
    there (Appendix A: one more rotation by delta).  ``stale_rows[b]``: store rows whose entries
    query b must not read.  k_pages[b] / v_pages[b] [P_b, Hkv, d]: the exclusive page, keys at their
    positions in the prompt (the decoding token's own entry included).
    Returns (O [B, Hq, d], lse [B, Hq])."""
    q = np.asarray(q, dtype=F64)
    ks, vs = np.asarray(k_shared, dtype=F64), np.asarray(v_shared, dtype=F64)
    B, Hq, d = q.shape
    G = Hq // ks.shape[1]
    out = np.empty_like(q)
    lse = np.empty((B, Hq), dtype=F64)
    for b in range(B):
        stale = set(int(r) for r in stale_rows[b])
        keys, vals = [], []
        for (row0, length, delta) in segments[b]:
            rows = [r for r in range(row0, row0 + length) if r not in stale]
            if rows:
                keys.append(rope_rotate(ks[rows], np.full(len(rows), delta, dtype=np.int64), base, layout, index_base))
                vals.append(vs[rows])
        keys.append(np.asarray(k_pages[b], dtype=F64))
        vals.append(np.asarray(v_pages[b], dtype=F64))
        kb, vb = np.concatenate(keys), np.concatenate(vals)            # [n_b, Hkv, d]
        for h in range(Hq):
            s = kb[:, h // G, :] @ q[b, h] / math.sqrt(d)
            m = s.max()
            w = np.exp(s - m)
            out[b, h] = (w / w.sum()) @ vb[:, h // G, :]
            lse[b, h] = m + math.log(w.sum())
    return out, lse


# --------------------------------------------------------------------------------------
# eq. 10: similarity-guided offline preprocessing (Sec. 3.1) -- attention of the chunk being cached
# --------------------------------------------------------------------------------------
def offline_preprocess_attn(q_chunk: np.ndarray, k_chunk: np.ndarray, v_chunk: np.ndarray,
                            k_prefix: np.ndarray, v_prefix: np.ndarray) -> np.ndarray:
    """Attention of chunk C_i while its cache is rebuilt offline (eq. 10): the chunk is fed at the
    positions that follow X = cat(S, C_top1..C_topn), so its token t attends to every entry of the
    concatenated prefix cache (already at its positions in X) and to the chunk's own tokens 0..t.
    q_chunk [n, Hq, d], k_chunk / v_chunk [n, Hkv, d] are rotated at positions |X| + t;
    k_prefix / v_prefix [|X|, Hkv, d]."""
    q, kc, vc, kp, vp = (np.asarray(a, dtype=F64) for a in (q_chunk, k_chunk, v_chunk, k_prefix, v_prefix))
    n, Hq, d = q.shape
    G = Hq // kc.shape[1]
    out = np.empty_like(q)
    for h in range(Hq):
        g = h // G
        for t in range(n):
            keys = np.concatenate([kp[:, g, :], kc[: t + 1, g, :]])
            vals = np.concatenate([vp[:, g, :], vc[: t + 1, g, :]])
            s = keys @ q[t, h] / math.sqrt(d)
            w = np.exp(s - s.max())
            out[t, h] = (w / w.sum()) @ vals
    return out


# --------------------------------------------------------------------------------------
# eq. 7-8: KV deviation and the CacheBlend selector (a comparison selector; same top-k)
# --------------------------------------------------------------------------------------
def kv_deviation(kv_fa: np.ndarray, kv_fr: np.ndarray) -> np.ndarray:
    """Delta_KV of one layer (eq. 7): per token, the sum over all components of the squared
    difference between the Full-Attention and the Full-Reuse entries."""
    a = np.asarray(kv_fa, dtype=F64)
    b = np.asarray(kv_fr, dtype=F64)
    return ((a - b) ** 2).reshape(a.shape[0], -1).sum(axis=1)


# --------------------------------------------------------------------------------------
# The model steps around the path (Sec. 2.1: each layer multiplies its input by the query, key and
# value weight matrices and adds positional embeddings by position index; eq. 9: only the rows
# cat(X[C_idx], Q) are fed).  RMSNorm and the SwiGLU feed-forward are those of the Llama-3-8B
# shaped layer that the full-stack configuration names; they are ordinary textbook definitions.
# --------------------------------------------------------------------------------------
def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """y = x / sqrt(mean(x^2) + eps) * gain, row by row."""
    x = np.asarray(x, dtype=F64)
    return x / np.sqrt((x * x).mean(axis=-1, keepdims=True) + eps) * np.asarray(gain, dtype=F64)


def linear(a: np.ndarray, w: np.ndarray, residual: Optional[np.ndarray] = None) -> np.ndarray:
    """out = a . w^T (+ residual); a [M, K], w [N, K]."""
    out = np.asarray(a, dtype=F64) @ np.asarray(w, dtype=F64).T
    return out if residual is None else out + np.asarray(residual, dtype=F64)


def linear_swiglu(a: np.ndarray, w_gate_up: np.ndarray) -> np.ndarray:
    """out[:, j] = silu(a . w[2j]) * (a . w[2j+1]), silu(t) = t / (1 + exp(-t)); gate and up rows interleaved."""
    y = linear(a, w_gate_up)
    gate, up = y[:, 0::2], y[:, 1::2]
    return gate / (1.0 + np.exp(-gate)) * up


def qkv_rope(a: np.ndarray, w_qkv: np.ndarray, positions: np.ndarray, Hq: int, Hkv: int, d: int, base: float,
             layout: str = "interleaved", index_base: int = 0):
    """Q/K/V projection of the fed rows, rotary embedding at each row's own position on q and k (eq. 9 feeds
    the positions cat(C_idx, question positions)).  Weight rows: query heads, key heads, value heads."""
    y = linear(a, w_qkv)
    M = y.shape[0]
    q = y[:, : Hq * d].reshape(M, Hq, d)
    k = y[:, Hq * d: (Hq + Hkv) * d].reshape(M, Hkv, d)
    v = y[:, (Hq + Hkv) * d:].reshape(M, Hkv, d)
    return rope_rotate(q, positions, base, layout, index_base), rope_rotate(k, positions, base, layout, index_base), v


def selective_prefill_layer(h: np.ndarray, q_index: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray, weights: dict,
                            Hq: int, Hkv: int, d: int, rope_base: float, eps: float, round_fn=None, rows=None):
    """One decoder layer of the sparse prefill (eq. 9) for the fed rows h [R, hidden] at positions q_index:
    RMSNorm -> Q/K/V with RoPE -> sparse attention over the cache with the fresh K/V -> output projection +
    residual -> RMSNorm -> SwiGLU feed-forward + residual.  Returns (h_out, k_new, v_new).  `round_fn`, if
    given, is applied wherever a real pipeline stores a tensor (so that a reduced-precision pipeline can be
    followed store by store); `rows` restricts everything after the K/V projection to a subset of rows."""
    r = round_fn if round_fn is not None else (lambda t: t)
    x = r(rmsnorm(h, weights["g1"], eps))
    q, k_new, v_new = (r(t) for t in qkv_rope(x, weights["w_qkv"], q_index, Hq, Hkv, d, rope_base))
    sel = np.arange(len(q_index)) if rows is None else np.asarray(rows)
    attn, _ = sparse_prefill_attn(q, q_index, k_cache, v_cache, k_new, v_new, rows=sel)
    attn = r(attn).reshape(len(sel), Hq * d)
    h1 = r(linear(attn, weights["w_o"], np.asarray(h, dtype=F64)[sel]))
    x2 = r(rmsnorm(h1, weights["g2"], eps))
    act = r(linear_swiglu(x2, weights["w_gate_up"]))
    h2 = r(linear(act, weights["w_down"], h1))
    return h2, k_new, v_new

"""GPU parity of the sparse prefill attention over a shared chunk store (Sec. 4.3): against the oracle's
position shift + effective cache + sparse attention, and against the library's own three-call path."""
import numpy as np
import pytest
import torch

from oracle import fusionrag_oracle as orc
from paper_2601_12904_amd import binding as B
from paper_2601_12904_amd import synth
from tests import harness as H

pytestmark = pytest.mark.gpu


def scattered_store(w, rng, pad=7):
    """The workload's cached chunks placed in a store in another order, with unrelated rows between them."""
    order = rng.permutation(w.n_chunks)
    Hkv, d = w.shape.n_kv_heads, w.shape.head_dim
    parts_k, parts_v, row0, at = [], [], np.zeros(w.n_chunks, dtype=np.int32), 0
    for c in order:
        s, e = int(w.chunk_offsets[c]), int(w.chunk_offsets[c + 1])
        junk = lambda: synth.round_to_storage((50.0 * rng.standard_normal((pad, Hkv, d))).astype(np.float32), w.shape.dtype)
        parts_k += [junk(), w.k_cached[s:e]]
        parts_v += [junk(), w.v_cached[s:e]]
        row0[c] = at + pad
        at += pad + (e - s)
    return np.concatenate(parts_k), np.concatenate(parts_v), row0


@pytest.mark.parametrize("layout", [B.FR_ROPE_INTERLEAVED, B.FR_ROPE_HALF])
@pytest.mark.parametrize("ratio", [0.0, 0.15, 1.0])
def test_shared_store_prefill_matches_oracle_and_three_call_path(ratio, layout):
    w = synth.config_small_bf16(seed=7, ratio=ratio, chunk_lens=(200, 0, 333, 91, 256))
    dt, tdt = "bf16", torch.bfloat16
    Hq, Hkv, d = w.shape.n_q_heads, w.shape.n_kv_heads, w.shape.head_dim
    rng = np.random.default_rng(3)
    lay = "half" if layout == B.FR_ROPE_HALF else "interleaved"
    src_pos0 = rng.integers(0, 5000, size=w.n_chunks).astype(np.int32)
    k_store, v_store, row0 = scattered_store(w, rng)
    k = orc.topk_count(w.L_ctx, ratio)
    qi = np.concatenate([np.sort(rng.choice(w.L_ctx, size=k, replace=False)), w.L_ctx + np.arange(w.nq)]).astype(np.int64)
    R = len(qi)
    ctx = H.make_ctx(w.shape, w.L, w.n_chunks, w.nq, rope_layout=layout)
    q_rows, k_new, v_new = H.dev(w.q_full[qi], dt), H.dev(w.k_full[qi], dt), H.dev(w.v_full[qi], dt)
    qi_d = torch.from_numpy(qi.astype(np.int32)).cuda()
    out = torch.zeros((R, Hq, d), dtype=tdt, device="cuda")
    lse = torch.zeros((R, Hq), dtype=torch.float32, device="cuda")
    ctx.fr_sparse_prefill_attn_shared(q_rows, qi_d, R, H.dev(k_store, dt), H.dev(v_store, dt), len(k_store), w.chunk_offsets,
                                      row0, src_pos0, w.L, k_new, v_new, out, lse)
    torch.cuda.synchronize()
    # oracle: shift the chunk keys to their prompt positions, then the sparse prefill over the effective cache
    k_ctx = synth.round_to_storage(orc.rope_shift(w.k_cached, w.chunk_offsets, src_pos0, None, w.shape.rope_base, lay), dt)
    pad = np.zeros((w.nq, Hkv, d))
    want, want_lse = orc.sparse_prefill_attn(w.q_full[qi], qi, np.concatenate([k_ctx, pad]),
                                             np.concatenate([w.v_cached, pad]), w.k_full[qi], w.v_full[qi])
    H.assert_close(H.host(out), want, dt, "shared-store attention")
    assert np.max(np.abs(lse.cpu().numpy() - want_lse)) <= 2e-3
    # the library's own path: shift into a per-query cache, then attend (the scatter does not change the output)
    k_cache = torch.zeros((w.L, Hkv, d), dtype=tdt, device="cuda")
    v_cache = torch.zeros((w.L, Hkv, d), dtype=tdt, device="cuda")
    v_cache[: w.L_ctx] = H.dev(w.v_cached, dt)
    ctx.fr_rope_shift(H.dev(w.k_cached, dt), k_cache, w.chunk_offsets, src_pos0)
    out2 = torch.zeros_like(out)
    ctx.fr_sparse_prefill_attn(q_rows, qi_d, R, k_cache, v_cache, w.L, k_new, v_new, out2)
    torch.cuda.synchronize()
    assert H.max_rel_err(H.host(out), H.host(out2)) <= 2.0 ** -7     # same inputs up to the key rotation's last bit
    ctx.close()


@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (4, 2), (16, 2)])
def test_shared_store_prefill_group_sizes(Hq, Hkv):
    """Group sizes 1, 2 and 8 of the tiled kernels over the chunk store: one query, and the same query twice through
    the batch call."""
    shape = synth.LayerShape(n_q_heads=Hq, n_kv_heads=Hkv, head_dim=128, dtype="bf16", rope_base=500000.0)
    w = synth.config_small_bf16(seed=Hkv, ratio=0.2, chunk_lens=(130, 0, 333, 61), nq=37, shape=shape)
    dt, tdt = "bf16", torch.bfloat16
    rng = np.random.default_rng(Hq)
    src_pos0 = rng.integers(0, 5000, size=w.n_chunks).astype(np.int32)
    k_store, v_store, row0 = scattered_store(w, rng)
    ks_d, vs_d = H.dev(k_store, dt), H.dev(v_store, dt)
    k = orc.topk_count(w.L_ctx, 0.2)
    qi = np.concatenate([np.sort(rng.choice(w.L_ctx, size=k, replace=False)), w.L_ctx + np.arange(w.nq)]).astype(np.int64)
    R = len(qi)
    ctx = H.make_ctx(shape, w.L, w.n_chunks, w.nq)
    ctx.fr_set_option(B.FR_OPT_ATTN_SPLIT, B.FR_ATTN_SPLIT_OFF)
    q_rows, k_new, v_new = H.dev(w.q_full[qi], dt), H.dev(w.k_full[qi], dt), H.dev(w.v_full[qi], dt)
    qi_d = torch.from_numpy(qi.astype(np.int32)).cuda()
    out = torch.zeros((R, Hq, 128), dtype=tdt, device="cuda")
    lse = torch.zeros((R, Hq), dtype=torch.float32, device="cuda")
    ctx.fr_sparse_prefill_attn_shared(q_rows, qi_d, R, ks_d, vs_d, len(k_store), w.chunk_offsets, row0, src_pos0, w.L,
                                      k_new, v_new, out, lse)
    torch.cuda.synchronize()
    k_ctx = synth.round_to_storage(orc.rope_shift(w.k_cached, w.chunk_offsets, src_pos0, None, shape.rope_base), dt)
    pad = np.zeros((w.nq, Hkv, 128))
    want, want_lse = orc.sparse_prefill_attn(w.q_full[qi], qi, np.concatenate([k_ctx, pad]),
                                             np.concatenate([w.v_cached, pad]), w.k_full[qi], w.v_full[qi])
    H.assert_close(H.host(out), want, dt, "shared-store attention")
    assert np.max(np.abs(lse.cpu().numpy() - want_lse)) <= 2e-3
    mkq = lambda: dict(q_rows=q_rows, q_index=qi_d, R=R, chunk_offsets=w.chunk_offsets, chunk_store_row0=row0,
                       chunk_src_pos0=src_pos0, L=w.L, k_new=k_new, v_new=v_new,
                       out=torch.zeros_like(out), lse_out=torch.zeros_like(lse))
    batch = [mkq(), mkq()]
    ws = torch.empty(ctx.fr_shared_batch_workspace_bytes(2, w.L), dtype=torch.uint8, device="cuda")
    ctx.fr_sparse_prefill_attn_shared_batch(batch, ks_d, vs_d, len(k_store), ws)
    torch.cuda.synchronize()
    for q in batch:
        assert torch.equal(q["out"], out) and torch.equal(q["lse_out"], lse)
    ctx.close()


def test_shared_store_prefill_argument_errors():
    w = synth.config_small_bf16(seed=1)
    ctx = H.make_ctx(w.shape, w.L, w.n_chunks, w.nq)
    P = 4096
    with pytest.raises(B.FusionRAGError):      # a chunk reaches past the end of the store
        ctx.fr_sparse_prefill_attn_shared(P, P, 5, P, P, 10, [0, 8, 16], [0, 4], [0, 0], 20, P, P, P)
    with pytest.raises(B.FusionRAGError):      # the page is required
        ctx.fr_sparse_prefill_attn_shared(P, P, 5, P, P, 100, [0, 8, 16], [0, 8], [0, 0], 20, None, None, P)
    ctx.close()


GENERIC_SHAPES = {
    "f32_d64": synth.TINY_F32,
    "f32_d128_g2": synth.LayerShape(n_q_heads=4, n_kv_heads=2, head_dim=128, dtype="f32", rope_base=500000.0),
    "bf16_d64_g4": synth.LayerShape(n_q_heads=8, n_kv_heads=2, head_dim=64, dtype="bf16", rope_base=10000.0),
    "bf16_d128_g3": synth.LayerShape(n_q_heads=6, n_kv_heads=2, head_dim=128, dtype="bf16", rope_base=500000.0),
}


@pytest.mark.parametrize("layout", [B.FR_ROPE_INTERLEAVED, B.FR_ROPE_HALF])
@pytest.mark.parametrize("name", sorted(GENERIC_SHAPES))
def test_shared_store_entry_points_on_shapes_without_tiled_kernels(name, layout):
    """fp32, head_dim 64 and group sizes the tiled kernels do not take: the shared-store entry points gather the
    query's keys (moved to their prompt positions) and values into the context's workspace and run the generic
    kernels.  Selection scores, index set and attention output against the oracle; the batch call against the
    one-query call, bit for bit."""
    shape = GENERIC_SHAPES[name]
    dt = shape.dtype
    tdt = torch.bfloat16 if dt == "bf16" else torch.float32
    w = synth.config_small_bf16(seed=13, ratio=0.2, chunk_lens=(70, 0, 133, 41, 96), nq=19, shape=shape)
    Hq, Hkv, d = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    rng = np.random.default_rng(5)
    lay = "half" if layout == B.FR_ROPE_HALF else "interleaved"
    src_pos0 = rng.integers(0, 3000, size=w.n_chunks).astype(np.int32)
    k_store, v_store, row0 = scattered_store(w, rng)
    ks_d, vs_d = H.dev(k_store, dt), H.dev(v_store, dt)
    ctx = H.make_ctx(shape, w.L, w.n_chunks, w.nq, rope_layout=layout)
    k_ctx = synth.round_to_storage(orc.rope_shift(w.k_cached, w.chunk_offsets, src_pos0, None, shape.rope_base, lay), dt)
    # selection
    k = orc.topk_count(w.L_ctx, 0.2)
    for norm, scope in ((B.FR_NORM_PER_CHUNK, "per_chunk"), (B.FR_NORM_GLOBAL, "global")):
        scores = torch.zeros(w.L_ctx, dtype=torch.float32, device="cuda")
        qi_d = torch.full((k + w.nq,), -1, dtype=torch.int32, device="cuda")
        ctx.fr_score_select_shared(H.dev(w.q_question, dt), w.nq, ks_d, len(k_store), w.chunk_offsets, row0, src_pos0, k,
                                   norm, scores, qi_d)
        torch.cuda.synchronize()
        want = orc.critical_scores(w.q_question, k_ctx, w.chunk_offsets, scope)
        assert H.max_rel_err(scores.cpu().numpy().astype(np.float64), want) <= (2e-3 if dt == "bf16" else 1e-5)
        H.assert_index_set(qi_d.cpu().numpy().astype(np.int64), want, k, w.nq)
    # attention, one query and the same query twice through the batch call
    qi = qi_d.cpu().numpy().astype(np.int64)
    R = len(qi)
    q_rows, k_new, v_new = H.dev(w.q_full[qi], dt), H.dev(w.k_full[qi], dt), H.dev(w.v_full[qi], dt)
    out = torch.zeros((R, Hq, d), dtype=tdt, device="cuda")
    lse = torch.zeros((R, Hq), dtype=torch.float32, device="cuda")
    ctx.fr_sparse_prefill_attn_shared(q_rows, qi_d, R, ks_d, vs_d, len(k_store), w.chunk_offsets, row0, src_pos0, w.L,
                                      k_new, v_new, out, lse)
    torch.cuda.synchronize()
    pad = np.zeros((w.nq, Hkv, d))
    want, want_lse = orc.sparse_prefill_attn(w.q_full[qi], qi, np.concatenate([k_ctx, pad]),
                                             np.concatenate([w.v_cached, pad]), w.k_full[qi], w.v_full[qi])
    H.assert_close(H.host(out), want, dt, "shared-store attention, generic kernels")
    assert np.max(np.abs(lse.cpu().numpy() - want_lse)) <= (2e-3 if dt == "bf16" else 1e-5)
    assert ctx.fr_shared_batch_workspace_bytes(2, w.L) == 0       # served from the context's own workspace
    mkq = lambda: dict(q_rows=q_rows, q_index=qi_d, R=R, chunk_offsets=w.chunk_offsets, chunk_store_row0=row0,
                       chunk_src_pos0=src_pos0, L=w.L, k_new=k_new, v_new=v_new,
                       out=torch.zeros_like(out), lse_out=torch.zeros_like(lse))
    batch = [mkq(), mkq()]
    ctx.fr_sparse_prefill_attn_shared_batch(batch, ks_d, vs_d, len(k_store), None, 0)
    torch.cuda.synchronize()
    for q in batch:
        assert torch.equal(q["out"], out) and torch.equal(q["lse_out"], lse)
    ctx.close()


def test_shared_store_prefill_batch_of_queries():
    """Several queries over one chunk store in one call (Sec. 4.3): different chunk subsets and orders, lengths, ratios
    and index sets (one query recomputes nothing, one has no rows at all).  Each query's output equals the one-query
    entry point's bit for bit (same kernels, same summation order with the key-range split off) and the oracle's
    within the bf16 tolerance."""
    dt, tdt = "bf16", torch.bfloat16
    rng = np.random.default_rng(11)
    base = synth.config_small_bf16(seed=5, chunk_lens=(200, 64, 333, 91, 256, 130))
    Hq, Hkv, d = base.shape.n_q_heads, base.shape.n_kv_heads, base.shape.head_dim
    k_store, v_store, row0_all = scattered_store(base, rng)
    ks_d, vs_d = H.dev(k_store, dt), H.dev(v_store, dt)
    chunk_len = np.diff(base.chunk_offsets)
    ctx = H.make_ctx(base.shape, base.L + 64, base.n_chunks, base.nq)
    ctx.fr_set_option(B.FR_OPT_ATTN_SPLIT, B.FR_ATTN_SPLIT_OFF)
    plans = [((0, 2, 4), 0.15, base.nq), ((5, 1), 0.0, 7), ((3, 0, 1, 2, 4, 5), 0.4, 33), ((2,), 1.0, 1), ((4, 3), 0.15, 0)]
    queries, keep = [], []
    for chunks, ratio, nq in plans:
        lens = [int(chunk_len[c]) for c in chunks]
        offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        L_ctx = int(offs[-1]); L = L_ctx + nq
        src_pos0 = rng.integers(0, 3000, size=len(chunks)).astype(np.int32)
        k = orc.topk_count(L_ctx, ratio) if nq > 0 else 0
        qi = np.concatenate([np.sort(rng.choice(L_ctx, size=k, replace=False)), L_ctx + np.arange(nq)]).astype(np.int64)
        R = len(qi)
        mk = lambda n, heads, scale: synth.round_to_storage((scale * rng.standard_normal((n, heads, d))).astype(np.float32), dt)
        q_rows, k_new, v_new = mk(R, Hq, 1.0), mk(R, Hkv, 1.0), mk(R, Hkv, 1.0)
        k_cached = np.concatenate([base.k_cached[base.chunk_offsets[c]:base.chunk_offsets[c + 1]] for c in chunks])
        v_cached = np.concatenate([base.v_cached[base.chunk_offsets[c]:base.chunk_offsets[c + 1]] for c in chunks])
        q = dict(q_rows=H.dev(q_rows, dt), q_index=torch.from_numpy(qi.astype(np.int32)).cuda(), R=R, chunk_offsets=offs,
                 chunk_store_row0=row0_all[list(chunks)], chunk_src_pos0=src_pos0, L=L, k_new=H.dev(k_new, dt),
                 v_new=H.dev(v_new, dt), out=torch.zeros((R, Hq, d), dtype=tdt, device="cuda"),
                 lse_out=torch.zeros((R, Hq), dtype=torch.float32, device="cuda"))
        queries.append(q)
        keep.append((qi, q_rows, k_new, v_new, k_cached, v_cached, offs, src_pos0, nq))
    n_ws = ctx.fr_shared_batch_workspace_bytes(len(queries), max(q["L"] for q in queries))
    assert n_ws > 0
    ws = torch.empty(n_ws, dtype=torch.uint8, device="cuda")
    ctx.fr_sparse_prefill_attn_shared_batch(queries, ks_d, vs_d, len(k_store), ws)
    torch.cuda.synchronize()
    for q, (qi, q_rows, k_new, v_new, k_cached, v_cached, offs, src_pos0, nq) in zip(queries, keep):
        R = q["R"]
        if R == 0:
            continue
        single = torch.zeros_like(q["out"])
        single_lse = torch.zeros_like(q["lse_out"])
        ctx.fr_sparse_prefill_attn_shared(q["q_rows"], q["q_index"], R, ks_d, vs_d, len(k_store), offs, q["chunk_store_row0"],
                                          src_pos0, q["L"], q["k_new"], q["v_new"], single, single_lse)
        torch.cuda.synchronize()
        assert torch.equal(single, q["out"]) and torch.equal(single_lse, q["lse_out"])
        k_ctx = synth.round_to_storage(orc.rope_shift(k_cached, offs, src_pos0, None, base.shape.rope_base, "interleaved"), dt)
        pad = np.zeros((nq, Hkv, d))
        want, want_lse = orc.sparse_prefill_attn(q_rows, qi, np.concatenate([k_ctx, pad]), np.concatenate([v_cached, pad]),
                                                 k_new, v_new)
        H.assert_close(H.host(q["out"]), want, dt, "batched shared-store attention")
        assert np.max(np.abs(q["lse_out"].cpu().numpy() - want_lse)) <= 2e-3
    # too small a workspace, and a bad query, are refused before anything runs
    with pytest.raises(B.FusionRAGError) as ei:
        ctx.fr_sparse_prefill_attn_shared_batch(queries, ks_d, vs_d, len(k_store), ws, workspace_bytes=4096)
    assert ei.value.status == B.FR_ERR_WORKSPACE
    bad = dict(queries[0]); bad["chunk_store_row0"] = np.array([len(k_store)] * 3, dtype=np.int32)
    with pytest.raises(B.FusionRAGError) as ei:
        ctx.fr_sparse_prefill_attn_shared_batch([queries[1], bad], ks_d, vs_d, len(k_store), ws)
    assert "query 1" in str(ei.value)
    ctx.close()


def test_shared_store_batch_full_size_sampled():
    """The launch configuration `bench.py --config 8` times (Llama-3-8B layer shape, queries of 16 chunks x 1024 tokens
    drawn from a 32-chunk store, 512 question tokens, 15 %), three queries per call: sampled output rows against the
    oracle, which forms each sampled row over the query's effective K/V."""
    shape = synth.LLAMA3_8B_BF16
    Hq, Hkv, d = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    dt, tdt = "bf16", torch.bfloat16
    nb, n_store_chunks, cpq, clen, nq, ratio = 3, 32, 16, 1024, 512, 0.15
    L_ctx, L = cpq * clen, cpq * clen + nq
    rng = np.random.default_rng(21)
    sig = 1.0 / np.sqrt(d)
    N = n_store_chunks * clen
    mk = lambda n, heads, scale: synth.round_to_storage((scale * rng.standard_normal((n, heads, d))).astype(np.float32), dt)
    k_store, v_store = mk(N, Hkv, sig), mk(N, Hkv, sig)
    ks_d, vs_d = H.dev(k_store, dt), H.dev(v_store, dt)
    k_sel = orc.topk_count(L_ctx, ratio)
    R = k_sel + nq
    offs = np.arange(0, L_ctx + 1, clen, dtype=np.int32)
    ctx = H.make_ctx(shape, L, cpq, nq)
    queries, keep = [], []
    for b in range(nb):
        ids = rng.choice(n_store_chunks, size=cpq, replace=False)
        row0 = (ids * clen).astype(np.int32)
        src = rng.integers(0, 4096, size=cpq).astype(np.int32)
        qi = np.concatenate([np.sort(rng.choice(L_ctx, size=k_sel, replace=False)), L_ctx + np.arange(nq)]).astype(np.int64)
        q_rows, k_new, v_new = mk(R, Hq, np.sqrt(d)), mk(R, Hkv, sig), mk(R, Hkv, sig)
        queries.append(dict(q_rows=H.dev(q_rows, dt), q_index=torch.from_numpy(qi.astype(np.int32)).cuda(), R=R,
                            chunk_offsets=offs, chunk_store_row0=row0, chunk_src_pos0=src, L=L, k_new=H.dev(k_new, dt),
                            v_new=H.dev(v_new, dt), out=torch.zeros((R, Hq, d), dtype=tdt, device="cuda")))
        keep.append((ids, src, qi, q_rows, k_new, v_new))
    ws = torch.empty(ctx.fr_shared_batch_workspace_bytes(nb, L), dtype=torch.uint8, device="cuda")
    ctx.fr_sparse_prefill_attn_shared_batch(queries, ks_d, vs_d, N, ws)
    torch.cuda.synchronize()
    for q, (ids, src, qi, q_rows, k_new, v_new) in zip(queries, keep):
        gather = np.concatenate([np.arange(i * clen, (i + 1) * clen) for i in ids])
        k_ctx = synth.round_to_storage(orc.rope_shift(k_store[gather], offs, src, None, shape.rope_base, "interleaved"), dt)
        pad = np.zeros((nq, Hkv, d))
        rows = np.unique(np.concatenate([[0, R - 1], rng.choice(R, size=30, replace=False)]))
        want, _ = orc.sparse_prefill_attn(q_rows, qi, np.concatenate([k_ctx, pad]), np.concatenate([v_store[gather], pad]),
                                          k_new, v_new, rows=rows)
        H.assert_close(H.host(q["out"][torch.from_numpy(rows).cuda()]), want, dt, "sampled rows of the batched launch")
    ctx.close()


@pytest.mark.parametrize("layout", [B.FR_ROPE_INTERLEAVED, B.FR_ROPE_HALF])
@pytest.mark.parametrize("norm", [B.FR_NORM_PER_CHUNK, B.FR_NORM_GLOBAL])
def test_shared_store_score_select(norm, layout):
    """Query-Guided Selection straight from the shared store: the keys are moved to their prompt positions inside the
    scoring kernels.  Scores against the oracle (position shift, then critical scores on the shifted keys as stored),
    index set by the tie-window rule, and agreement with the library's own fr_rope_shift + fr_score_select."""
    w = synth.config_small_bf16(seed=9, chunk_lens=(200, 0, 333, 91, 256, 130))
    dt = "bf16"
    Hkv, d = w.shape.n_kv_heads, w.shape.head_dim
    rng = np.random.default_rng(17)
    lay = "half" if layout == B.FR_ROPE_HALF else "interleaved"
    src_pos0 = rng.integers(0, 5000, size=w.n_chunks).astype(np.int32)
    k_store, _, row0 = scattered_store(w, rng)
    ks_d = H.dev(k_store, dt)
    k = orc.topk_count(w.L_ctx, 0.15)
    ctx = H.make_ctx(w.shape, w.L, w.n_chunks, w.nq, rope_layout=layout)
    qq = H.dev(w.q_question, dt)
    scores = torch.zeros(w.L_ctx, dtype=torch.float32, device="cuda")
    qi = torch.full((k + w.nq,), -1, dtype=torch.int32, device="cuda")
    ctx.fr_score_select_shared(qq, w.nq, ks_d, len(k_store), w.chunk_offsets, row0, src_pos0, k, norm, scores, qi)
    torch.cuda.synchronize()
    k_ctx = synth.round_to_storage(orc.rope_shift(w.k_cached, w.chunk_offsets, src_pos0, None, w.shape.rope_base, lay), dt)
    want = orc.critical_scores(w.q_question, k_ctx, w.chunk_offsets, "global" if norm == B.FR_NORM_GLOBAL else "per_chunk")
    got = scores.cpu().numpy().astype(np.float64)
    assert H.max_rel_err(got, want) <= 2e-3      # the kernel's shifted keys may differ from the oracle's in the last bf16 bit
    H.assert_index_set(qi.cpu().numpy().astype(np.int64), want, k, w.nq)
    # the two-call path of the same library
    k_shift = torch.zeros((w.L_ctx, Hkv, d), dtype=torch.bfloat16, device="cuda")
    ctx.fr_rope_shift(H.dev(w.k_cached, dt), k_shift, w.chunk_offsets, src_pos0)
    scores2 = torch.zeros_like(scores)
    qi2 = torch.zeros_like(qi)
    ctx.fr_score_select(qq, w.nq, k_shift, w.chunk_offsets, k, norm, scores2, qi2)
    torch.cuda.synchronize()
    assert H.max_rel_err(got, scores2.cpu().numpy().astype(np.float64)) <= 2e-3
    # no question rows: all scores zero, the first k tokens win the ties
    ctx.fr_score_select_shared(None, 0, ks_d, len(k_store), w.chunk_offsets, row0, src_pos0, 5, norm, scores, qi)
    torch.cuda.synchronize()
    assert float(scores.abs().max()) == 0.0 and qi[:5].cpu().tolist() == [0, 1, 2, 3, 4]
    with pytest.raises(B.FusionRAGError):
        ctx.fr_score_select_shared(qq, w.nq, ks_d, len(k_store), w.chunk_offsets, row0, src_pos0, k, B.FR_NORM_RAW, scores, qi)
    with pytest.raises(B.FusionRAGError):      # a chunk reaches past the end of the store
        ctx.fr_score_select_shared(qq, w.nq, ks_d, 100, w.chunk_offsets, row0, src_pos0, k, norm, scores, qi)
    ctx.close()

"""GPU parity: every entry point of the C-ABI library against the fp64 oracle, element by element,
on seeded synthetic inputs that span several kernel tiles and ragged tails."""
import numpy as np
import pytest
import torch

from oracle import fusionrag_oracle as orc
from paper_2601_12904_amd import binding as B
from paper_2601_12904_amd import synth
from tests import harness as H

pytestmark = pytest.mark.gpu

BF16_D64_G2 = synth.LayerShape(n_q_heads=4, n_kv_heads=2, head_dim=64, dtype="bf16", rope_base=10000.0)
F32_D128_G4 = synth.LayerShape(n_q_heads=8, n_kv_heads=2, head_dim=128, dtype="f32", rope_base=500000.0)


def workloads():
    return {
        "tiny_f32": lambda seed: synth.config_tiny(seed=seed),
        "small_bf16": lambda seed: synth.config_small_bf16(seed=seed),
        "small_bf16_d64": lambda seed: synth.config_small_bf16(seed=seed, shape=BF16_D64_G2, chunk_lens=(70, 130, 3)),
        "small_f32_d128": lambda seed: synth.make_workload("f32_d128", F32_D128_G4, [100, 1, 77], nq=9, ratio=0.2,
                                                           seed=seed, focus_frac=0.05),
    }


CASES = [(n, s) for n in workloads() for s in (0, 1)]


def staged(w: synth.Workload):
    """Oracle results of every stage, each fed with the oracle's previous stage rounded to storage."""
    dt = w.shape.dtype
    k_ctx = synth.round_to_storage(orc.rope_shift(w.k_cached, w.chunk_offsets, w.src_pos0, None, w.shape.rope_base), dt)
    scores = orc.critical_scores(w.q_question, k_ctx, w.chunk_offsets)
    k = orc.topk_count(w.L_ctx, w.ratio)
    qi = orc.select_q_index(scores, k, w.nq)
    return k_ctx, scores, k, qi


def assembled_cache(w: synth.Workload, k_ctx: np.ndarray, seed: int = 99):
    """Per-query cache [L]: shifted stale keys / stale values, then nq reserved rows (arbitrary content)."""
    rng = np.random.default_rng(seed)
    pad = lambda: synth.round_to_storage(rng.standard_normal((w.nq,) + k_ctx.shape[1:]).astype(np.float32), w.shape.dtype)
    return np.concatenate([k_ctx, pad()]), np.concatenate([w.v_cached, pad()])


@pytest.mark.parametrize("name,seed", CASES)
def test_rope_shift(name, seed):
    w = workloads()[name](seed)
    dt = w.shape.dtype
    ctx = H.make_ctx(w.shape, w.L, w.n_chunks, w.nq)
    src = H.dev(w.k_cached, dt)
    dst = torch.empty_like(src)
    ctx.fr_rope_shift(src, dst, w.chunk_offsets, w.src_pos0)
    torch.cuda.synchronize()
    want = orc.rope_shift(w.k_cached, w.chunk_offsets, w.src_pos0, None, w.shape.rope_base)
    got = H.host(dst)
    H.assert_close(got, want, dt, "rope_shift")
    # element-wise: the result is the fp64 value rounded once to storage, give or take one unit
    ulp = 2.0 ** -7 if dt == "bf16" else 2.0 ** -21
    assert np.all(np.abs(got - want) <= ulp * np.abs(want) + 1e-30 + (1e-6 if dt == "f32" else 1e-4) * np.abs(want).max())
    # in place gives the same bits
    ctx.fr_rope_shift(src, src, w.chunk_offsets, w.src_pos0)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    ctx.close()


@pytest.mark.parametrize("layout,index_base", [(B.FR_ROPE_HALF, 0), (B.FR_ROPE_INTERLEAVED, 1), (B.FR_ROPE_HALF, 1)])
@pytest.mark.parametrize("name", ["tiny_f32", "small_bf16"])
def test_rope_shift_variants(name, layout, index_base):
    w = workloads()[name](3)
    dt = w.shape.dtype
    ctx = H.make_ctx(w.shape, w.L, w.n_chunks, w.nq, rope_layout=layout, rope_index_base=index_base)
    rng = np.random.default_rng(5)
    src_pos = rng.integers(0, 50, size=w.n_chunks)
    dst_pos = rng.integers(0, 40000, size=w.n_chunks)
    src = H.dev(w.k_cached, dt)
    dst = torch.empty_like(src)
    ctx.fr_rope_shift(src, dst, w.chunk_offsets, src_pos, dst_pos)
    torch.cuda.synchronize()
    want = orc.rope_shift(w.k_cached, w.chunk_offsets, src_pos, dst_pos, w.shape.rope_base,
                          "half" if layout == B.FR_ROPE_HALF else "interleaved", index_base)
    H.assert_close(H.host(dst), want, dt, "rope_shift variant")
    ctx.close()


def test_rope_shift_batched_layers_and_empty_chunk():
    shape = synth.LLAMA3_8B_BF16
    w = synth.make_workload("b", shape, [40, 0, 90, 33], nq=4, ratio=0.15, seed=4, sigma_q=1, sigma_kv=1)
    ctx = H.make_ctx(shape, w.L, w.n_chunks, w.nq)
    n_batch, pad = 3, 64
    layer = w.L_ctx * shape.n_kv_heads * shape.head_dim
    rng = np.random.default_rng(0)
    layers = [synth.round_to_storage(rng.standard_normal(w.k_cached.shape).astype(np.float32), "bf16") for _ in range(n_batch)]
    buf = torch.zeros(n_batch * (layer + pad), dtype=torch.bfloat16, device="cuda")
    for b in range(n_batch):
        buf[b * (layer + pad): b * (layer + pad) + layer] = H.dev(layers[b], "bf16").reshape(-1)
    out = torch.full_like(buf, 7.0)
    ctx.fr_rope_shift(buf, out, w.chunk_offsets, w.src_pos0, dst_base=1000, n_batch=n_batch,
                      src_batch_stride=layer + pad, dst_batch_stride=layer + pad)
    torch.cuda.synchronize()
    for b in range(n_batch):
        want = orc.rope_shift(layers[b], w.chunk_offsets, w.src_pos0, None, shape.rope_base, dst_base=1000)
        got = H.host(out[b * (layer + pad): b * (layer + pad) + layer]).reshape(want.shape)
        H.assert_close(got, want, "bf16", f"layer {b}")
        assert torch.all(out[b * (layer + pad) + layer: (b + 1) * (layer + pad)] == 7.0)   # padding untouched
    ctx.close()


@pytest.mark.parametrize("norm", [B.FR_NORM_PER_CHUNK, B.FR_NORM_GLOBAL, B.FR_NORM_RAW])
@pytest.mark.parametrize("name,seed", CASES)
def test_score_select(name, seed, norm):
    w = workloads()[name](seed)
    dt = w.shape.dtype
    k_ctx, _, k, _ = staged(w)
    norm_name = {0: "per_chunk", 1: "global", 2: "raw"}[norm]
    want_scores = orc.critical_scores(w.q_question, k_ctx, w.chunk_offsets, norm_name)
    ctx = H.make_ctx(w.shape, w.L, w.n_chunks, w.nq)
    scores = torch.empty(w.L_ctx, dtype=torch.float32, device="cuda")
    qi = torch.full((k + w.nq,), -1, dtype=torch.int32, device="cuda")
    ctx.fr_score_select(H.dev(w.q_question, dt), w.nq, H.dev(k_ctx, dt), w.chunk_offsets, k, norm, scores, qi)
    torch.cuda.synchronize()
    got = scores.cpu().numpy().astype(np.float64)
    err = H.max_rel_err(got, want_scores)
    assert err <= 1e-4, f"scores: max relative error {err:.2e}"
    H.assert_index_set(qi.cpu().numpy(), want_scores, k, w.nq)
    # the selection itself is exact on the scores the kernel saw
    assert np.array_equal(qi.cpu().numpy(), orc.select_q_index(scores.cpu().numpy(), k, w.nq))
    # scores_out = NULL gives the same index
    qi2 = torch.full_like(qi, -1)
    ctx.fr_score_select(H.dev(w.q_question, dt), w.nq, H.dev(k_ctx, dt), w.chunk_offsets, k, norm, None, qi2)
    torch.cuda.synchronize()
    assert torch.equal(qi, qi2)
    ctx.close()


TILED_SCORE_CASES = [
    # (query heads, KV heads, question tokens, chunk lengths): group sizes 1, 2, 4, 8; question columns (G x tokens)
    # below, at and above one 64-column tile and one 256-column workgroup; chunks below, at and above one 64-key
    # tile and one 256-key workgroup, empty chunks, a single chunk
    (4, 4, 1, (5,)),
    (4, 4, 64, (64, 65, 1)),
    (4, 4, 65, (256, 0, 257)),
    (4, 2, 32, (63, 64)),
    (4, 2, 33, (300, 7, 129)),
    (8, 2, 16, (64,)),
    (8, 2, 17, (0, 200, 0, 70)),
    (8, 2, 130, (191, 513)),
    (16, 2, 8, (100, 28)),
    (16, 2, 9, (64, 320)),
    (16, 2, 71, (33, 0, 450)),
]


@pytest.mark.parametrize("norm", [B.FR_NORM_PER_CHUNK, B.FR_NORM_GLOBAL])
@pytest.mark.parametrize("Hq,Hkv,nq,chunk_lens", TILED_SCORE_CASES)
def test_score_select_tiled_kernel_shapes(Hq, Hkv, nq, chunk_lens, norm):
    """The matrix-core scoring passes (bf16, head_dim 128) at every group size and at tile boundaries of both
    operands, against the oracle; the chunk-store entry point on the same keys gives the same scores."""
    shape = synth.LayerShape(n_q_heads=Hq, n_kv_heads=Hkv, head_dim=128, dtype="bf16", rope_base=500000.0)
    w = synth.config_small_bf16(seed=Hq + nq, chunk_lens=chunk_lens, nq=nq, shape=shape)
    dt = "bf16"
    k_ctx = synth.round_to_storage(orc.rope_shift(w.k_cached, w.chunk_offsets, w.src_pos0, None, shape.rope_base), dt)
    want = orc.critical_scores(w.q_question, k_ctx, w.chunk_offsets, "global" if norm == B.FR_NORM_GLOBAL else "per_chunk")
    k = orc.topk_count(w.L_ctx, 0.3)
    ctx = H.make_ctx(shape, w.L, w.n_chunks, w.nq)
    scores = torch.full((w.L_ctx,), -7.0, dtype=torch.float32, device="cuda")
    qi = torch.full((k + w.nq,), -1, dtype=torch.int32, device="cuda")
    qq, kc = H.dev(w.q_question, dt), H.dev(k_ctx, dt)
    ctx.fr_score_select(qq, w.nq, kc, w.chunk_offsets, k, norm, scores, qi)
    torch.cuda.synchronize()
    got = scores.cpu().numpy().astype(np.float64)
    assert H.max_rel_err(got, want) <= 1e-4
    H.assert_index_set(qi.cpu().numpy(), want, k, w.nq)
    # the same keys as a chunk store with zero position shift (chunks in reverse order, a gap in front)
    gap = 3
    order = list(range(w.n_chunks))[::-1]
    row0 = np.zeros(w.n_chunks, dtype=np.int32)
    parts, at = [np.zeros((gap,) + k_ctx.shape[1:], dtype=k_ctx.dtype)], gap
    for c in order:
        row0[c] = at
        parts.append(k_ctx[w.chunk_offsets[c]:w.chunk_offsets[c + 1]])
        at += int(w.chunk_offsets[c + 1] - w.chunk_offsets[c])
    store = np.concatenate(parts)
    scores2 = torch.full_like(scores, -7.0)
    qi2 = torch.full_like(qi, -1)
    ctx.fr_score_select_shared(qq, w.nq, H.dev(store, dt), len(store), w.chunk_offsets, row0, w.chunk_offsets[:-1], k, norm,
                               scores2, qi2)
    torch.cuda.synchronize()
    assert torch.equal(scores, scores2) and torch.equal(qi, qi2)     # a rotation by zero positions leaves the keys as stored
    ctx.close()


@pytest.mark.parametrize("n,k,nq", [(1, 1, 0), (1, 0, 3), (7, 3, 2), (1000, 150, 5), (1024, 1024, 0), (4097, 1, 1),
                                    (16384, 2458, 512), (20001, 3000, 0), (50000, 7500, 17), (16384, 16383, 0)])
def test_select_topk_exact(n, k, nq):
    ctx = H.make_ctx(synth.TINY_F32, 70000, 4, 600)
    rng = np.random.default_rng(n + k)
    for kind in ("uniform", "ties", "signed", "constant", "clustered", "full_range"):
        if kind == "uniform":
            s = rng.random(n).astype(np.float32)
        elif kind == "ties":
            s = rng.integers(0, 8, size=n).astype(np.float32)          # heavy ties: lowest index must win
        elif kind == "signed":
            s = rng.standard_normal(n).astype(np.float32)
        elif kind == "clustered":                                       # narrow key range, as real score vectors
            s = (16.0 * np.exp(0.6 * rng.standard_normal(n))).astype(np.float32)
        elif kind == "full_range":                                      # extremes that span all 32 key bits
            s = (16.0 * np.exp(0.6 * rng.standard_normal(n))).astype(np.float32)
            s[n // 2] = -3.0e38
            s[n // 3] = 3.0e38
        else:
            s = np.full(n, 0.25, dtype=np.float32)
        out = torch.full((k + nq,), -7, dtype=torch.int32, device="cuda")
        ctx.fr_select_topk(torch.from_numpy(s).cuda(), n, k, nq, out)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), orc.select_q_index(s, k, nq)), kind
    ctx.close()


@pytest.mark.parametrize("n,k,nq", [(32769, 4915, 3), (40000, 40000, 2), (33000, 1, 0), (40000, 0, 5), (300000, 45000, 9),
                                    (1 << 20, 157286, 0), (1234567, 1234, 1), (9000001, 1350000, 2)])
def test_select_topk_many_workgroups(n, k, nq):
    """Score vectors beyond one workgroup's registers take the multi-pass selection: same definition, same oracle.
    `narrow_cluster` puts more keys into one 24-bit prefix than the candidate list holds (the last level then re-reads
    the scores); `ties` and `constant` exercise the equal-key budget across waves and tiles.  The largest case spans
    two steps of the emitting pass's look-back over the tiles before a tile."""
    ctx = H.make_ctx(synth.TINY_F32, 4096, 4, 16)
    rng = np.random.default_rng(n ^ k)
    for kind in ("signed", "ties", "clustered", "full_range", "constant", "narrow_cluster"):
        if kind == "signed":
            s = rng.standard_normal(n).astype(np.float32)
        elif kind == "ties":
            s = rng.integers(0, 8, size=n).astype(np.float32)
        elif kind == "clustered":
            s = (16.0 * np.exp(0.6 * rng.standard_normal(n))).astype(np.float32)
        elif kind == "full_range":
            s = (16.0 * np.exp(0.6 * rng.standard_normal(n))).astype(np.float32)
            s[n // 2] = -3.0e38
            s[n // 3] = 3.0e38
        elif kind == "constant":
            s = np.full(n, 0.25, dtype=np.float32)
        else:
            s = (np.float32(1.0) + rng.integers(0, 256, size=n).astype(np.float32) * np.float32(2.0 ** -23)).astype(np.float32)
            s[n // 5] = 1.0e30
        out = torch.full((k + nq,), -7, dtype=torch.int32, device="cuda")
        ctx.fr_select_topk(torch.from_numpy(s).cuda(), n, k, nq, out)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), orc.select_q_index(s, k, nq)), kind
    ctx.close()


@pytest.mark.parametrize("name", ["tiny_f32", "offline_bf16"])
def test_offline_preprocess_attention(name):
    """eq. 10, the offline stage's attention: the retrieved chunks' cached keys are moved to their positions in
    X = cat(S, C_top1..n) (fr_rope_shift), and the rows of the chunk being cached, fed at the positions after X,
    attend to that prefix and causally to themselves (fr_sparse_prefill_attn with a contiguous Q index: no context
    token is recomputed).  The generator's question part stands in for the chunk C_i."""
    if name == "tiny_f32":
        w = synth.config_tiny(seed=2)
    else:   # prefix: system prompt 64 + three retrieved chunks; chunk being cached: 150 tokens (3 row tiles, ragged)
        w = synth.config_small_bf16(seed=2, chunk_lens=(64, 200, 130, 257), nq=150)
    dt = w.shape.dtype
    ctx = H.make_ctx(w.shape, w.L, len(w.chunk_offsets) - 1, w.nq)
    k_x = torch.zeros((w.L, w.shape.n_kv_heads, w.shape.head_dim), dtype=H.TORCH_DTYPE[dt], device="cuda")
    v_x = torch.zeros_like(k_x)
    v_x[: w.L_ctx] = H.dev(w.v_cached, dt)
    ctx.fr_rope_shift(H.dev(w.k_cached, dt), k_x, w.chunk_offsets, w.src_pos0)
    qi = np.arange(w.L_ctx, w.L)
    got, _ = run_attention(ctx, w, qi, H.host(k_x), H.host(v_x))
    k_prefix = synth.round_to_storage(orc.rope_shift(w.k_cached, w.chunk_offsets, w.src_pos0, None, w.shape.rope_base), dt)
    want = orc.offline_preprocess_attn(w.q_full[w.L_ctx:], w.k_full[w.L_ctx:], w.v_full[w.L_ctx:], k_prefix, w.v_cached)
    H.assert_close(got, want, dt, "offline preprocessing attention")
    ctx.close()


@pytest.mark.parametrize("name,seed", CASES)
def test_kv_deviation_selector(name, seed):
    """eq. 7-8: per-token squared deviation between the keys of full attention and the reused keys, then the same
    top-k.  fp32 sums of at most a few thousand exact squared differences: 1e-5 relative."""
    w = workloads()[name](seed)
    dt = w.shape.dtype
    k_ctx, _, k, _ = staged(w)
    k_fa = w.k_full[: w.L_ctx]
    ctx = H.make_ctx(w.shape, w.L, len(w.chunk_offsets) - 1, w.nq)
    dev = torch.full((w.L_ctx,), -1.0, dtype=torch.float32, device="cuda")
    ctx.fr_kv_deviation(H.dev(k_fa, dt), H.dev(k_ctx, dt), w.L_ctx, dev)
    qi = torch.full((k + w.nq,), -7, dtype=torch.int32, device="cuda")
    ctx.fr_select_topk(dev, w.L_ctx, k, w.nq, qi)
    torch.cuda.synchronize()
    want = orc.kv_deviation(k_fa, k_ctx)
    got = dev.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - want) <= 1e-5 * np.abs(want) + 1e-30)
    H.assert_index_set(qi.cpu().numpy(), want, k, w.nq, rel_tie=1e-5)
    ctx.close()


def test_kv_deviation_ragged_sizes():
    rng = np.random.default_rng(3)
    for shape in (synth.TINY_F32, BF16_D64_G2):
        ctx = H.make_ctx(shape, 4096, 4, 8)
        for n in (1, 3, 4, 5, 1023, 2050):
            a = synth.round_to_storage(rng.standard_normal((n, shape.n_kv_heads, shape.head_dim)).astype(np.float32), shape.dtype)
            b = synth.round_to_storage(rng.standard_normal((n, shape.n_kv_heads, shape.head_dim)).astype(np.float32), shape.dtype)
            out = torch.full((n + 1,), -1.0, dtype=torch.float32, device="cuda")
            ctx.fr_kv_deviation(H.dev(a, shape.dtype), H.dev(b, shape.dtype), n, out)
            torch.cuda.synchronize()
            got = out.cpu().numpy().astype(np.float64)
            want = orc.kv_deviation(a, b)
            assert got[n] == -1.0                                 # nothing written past the end
            assert np.all(np.abs(got[:n] - want) <= 1e-5 * want)
        ctx.close()


def run_attention(ctx, w, qi, k_cache, v_cache, with_new=True, want_lse=True):
    dt = w.shape.dtype
    R = len(qi)
    q_rows = H.dev(w.q_full[qi], dt)
    k_new, v_new = H.dev(w.k_full[qi], dt), H.dev(w.v_full[qi], dt)
    out = torch.zeros((R, w.shape.n_q_heads, w.shape.head_dim), dtype=H.TORCH_DTYPE[dt], device="cuda")
    lse = torch.zeros((R, w.shape.n_q_heads), dtype=torch.float32, device="cuda") if want_lse else None
    qi_d = torch.from_numpy(qi.astype(np.int32)).cuda()
    ctx.fr_sparse_prefill_attn(q_rows, qi_d, R, H.dev(k_cache, dt), H.dev(v_cache, dt), w.L,
                               k_new if with_new else None, v_new if with_new else None, out, lse)
    torch.cuda.synchronize()
    return H.host(out), (lse.cpu().numpy().astype(np.float64) if want_lse else None)


@pytest.mark.parametrize("name,seed", CASES)
def test_sparse_prefill_attn(name, seed):
    w = workloads()[name](seed)
    dt = w.shape.dtype
    k_ctx, _, k, qi = staged(w)
    k_cache, v_cache = assembled_cache(w, k_ctx)
    ctx = H.make_ctx(w.shape, w.L, w.n_chunks, w.nq)
    got, lse = run_attention(ctx, w, qi, k_cache, v_cache)
    want, want_lse = orc.sparse_prefill_attn(w.q_full[qi], qi, k_cache, v_cache, w.k_full[qi], w.v_full[qi])
    H.assert_close(got, want, dt, "attention output")
    assert np.max(np.abs(lse - want_lse)) <= (1e-4 if dt == "f32" else 2e-3), "lse"
    # fresh rows already scattered into the cache + NULL k_new: same result
    k_eff, v_eff = orc.kv_scatter(qi, w.k_full[qi], w.v_full[qi], k_cache, v_cache)
    got2, _ = run_attention(ctx, w, qi, k_eff, v_eff, with_new=False, want_lse=False)
    H.assert_close(got2, want, dt, "attention over scattered cache")
    ctx.close()


@pytest.mark.parametrize("split", [B.FR_ATTN_SPLIT_OFF, B.FR_ATTN_SPLIT_ON])
@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (4, 2), (16, 2)])
def test_sparse_prefill_attn_tiled_kernel_group_sizes(Hq, Hkv, split):
    """The matrix-core attention kernels (bf16, head_dim 128) at group sizes 1, 2 and 8 (a row tile holds 64, 32 or 8
    tokens), with and without the key-range split, fused write-back included."""
    shape = synth.LayerShape(n_q_heads=Hq, n_kv_heads=Hkv, head_dim=128, dtype="bf16", rope_base=500000.0)
    w = synth.config_small_bf16(seed=Hq, ratio=0.2, chunk_lens=(130, 0, 333, 61), nq=37, shape=shape)
    dt = "bf16"
    k_ctx, _, k, qi = staged(w)
    k_cache, v_cache = assembled_cache(w, k_ctx)
    ctx = H.make_ctx(shape, w.L, w.n_chunks, w.nq)
    ctx.fr_set_option(B.FR_OPT_ATTN_SPLIT, split)
    got, lse = run_attention(ctx, w, qi, k_cache, v_cache)
    want, want_lse = orc.sparse_prefill_attn(w.q_full[qi], qi, k_cache, v_cache, w.k_full[qi], w.v_full[qi])
    H.assert_close(got, want, dt, "attention output")
    assert np.max(np.abs(lse - want_lse)) <= 2e-3, "lse"
    # write-back fused into the call: same output, and the caches end up as after the scatter
    R = len(qi)
    kc, vc = H.dev(k_cache, dt), H.dev(v_cache, dt)
    out = torch.zeros((R, Hq, 128), dtype=torch.bfloat16, device="cuda")
    ctx.fr_sparse_prefill_attn_writeback(H.dev(w.q_full[qi], dt), torch.from_numpy(qi.astype(np.int32)).cuda(), R, kc, vc, w.L,
                                         H.dev(w.k_full[qi], dt), H.dev(w.v_full[qi], dt), out)
    torch.cuda.synchronize()
    H.assert_close(H.host(out), want, dt, "attention output with write-back")
    k_eff, v_eff = orc.kv_scatter(qi, w.k_full[qi], w.v_full[qi], k_cache, v_cache)
    assert np.array_equal(H.host(kc), k_eff) and np.array_equal(H.host(vc), v_eff)
    ctx.close()


@pytest.mark.parametrize("name", ["tiny_f32", "small_bf16"])
@pytest.mark.parametrize("ratio", [0.0, 0.05, 0.30, 1.0])
def test_ratio_extremes(name, ratio):
    w = workloads()[name](2)
    dt = w.shape.dtype
    k_ctx, scores, _, _ = staged(w)
    k = orc.topk_count(w.L_ctx, ratio)
    qi = orc.select_q_index(scores, k, w.nq)
    k_cache, v_cache = assembled_cache(w, k_ctx)
    ctx = H.make_ctx(w.shape, w.L, w.n_chunks, w.nq)
    got, _ = run_attention(ctx, w, qi, k_cache, v_cache)
    if ratio == 1.0:      # recomputing everything is full causal prefill, whatever the stale cache holds
        want = orc.full_causal_attention(w.q_full, w.k_full, w.v_full)
    else:
        want, _ = orc.sparse_prefill_attn(w.q_full[qi], qi, k_cache, v_cache, w.k_full[qi], w.v_full[qi])
    H.assert_close(got, want, dt, f"ratio {ratio}")
    ctx.close()


@pytest.mark.parametrize("name,seed", CASES)
def test_kv_scatter_bit_exact(name, seed):
    w = workloads()[name](seed)
    dt = w.shape.dtype
    k_ctx, _, _, qi = staged(w)
    k_cache, v_cache = assembled_cache(w, k_ctx)
    ctx = H.make_ctx(w.shape, w.L, w.n_chunks, w.nq)
    kc, vc = H.dev(k_cache, dt), H.dev(v_cache, dt)
    k_new, v_new = H.dev(w.k_full[qi], dt), H.dev(w.v_full[qi], dt)
    qi_d = torch.from_numpy(qi.astype(np.int32)).cuda()
    ctx.fr_kv_scatter(k_new, v_new, qi_d, len(qi), kc, vc, w.L)
    torch.cuda.synchronize()
    want_k, want_v = orc.kv_scatter(qi, w.k_full[qi], w.v_full[qi], k_cache, v_cache)
    assert np.array_equal(H.host(kc), want_k.astype(np.float64)) and np.array_equal(H.host(vc), want_v.astype(np.float64))
    before_k = kc.clone()
    ctx.fr_kv_scatter(k_new, v_new, qi_d, len(qi), kc, vc, w.L)   # idempotent
    torch.cuda.synchronize()
    assert torch.equal(kc, before_k)
    ctx.close()


def test_kv_scatter_ignores_positions_outside_the_cache():
    """A Q index entry outside [0, L) breaks the caller's contract; the kernel's own bounds check drops that row
    instead of writing outside the cache, and every other row is written as usual."""
    w = workloads()["tiny_f32"](0)
    dt = w.shape.dtype
    k_ctx, _, _, qi = staged(w)
    k_cache, v_cache = assembled_cache(w, k_ctx)
    ctx = H.make_ctx(w.shape, w.L, w.n_chunks, w.nq)
    bad = qi.copy()
    bad[0], bad[-1] = -3, w.L + 5
    kc, vc = H.dev(k_cache, dt), H.dev(v_cache, dt)
    ctx.fr_kv_scatter(H.dev(w.k_full[qi], dt), H.dev(w.v_full[qi], dt), torch.from_numpy(bad.astype(np.int32)).cuda(),
                      len(qi), kc, vc, w.L)
    torch.cuda.synchronize()
    want_k, want_v = orc.kv_scatter(qi[1:-1], w.k_full[qi[1:-1]], w.v_full[qi[1:-1]], k_cache, v_cache)
    assert np.array_equal(H.host(kc), want_k.astype(np.float64)) and np.array_equal(H.host(vc), want_v.astype(np.float64))
    ctx.close()


@pytest.mark.parametrize("name,seed", CASES)
def test_chained_layer(name, seed):
    """The four calls back to back on one stream, no host work in between, against the oracle chain."""
    w = workloads()[name](seed)
    dt = w.shape.dtype
    tdt = H.TORCH_DTYPE[dt]
    Hq, Hkv, d = w.shape.n_q_heads, w.shape.n_kv_heads, w.shape.head_dim
    k_ctx_o, scores_o, k, qi_o = staged(w)
    R = k + w.nq
    ctx = H.make_ctx(w.shape, w.L, w.n_chunks, w.nq)
    k_cache = torch.zeros((w.L, Hkv, d), dtype=tdt, device="cuda")
    v_cache = torch.zeros((w.L, Hkv, d), dtype=tdt, device="cuda")
    v_cache[: w.L_ctx] = H.dev(w.v_cached, dt)
    qi = torch.empty(R, dtype=torch.int32, device="cuda")
    # the harness stands in for the model's QKV projection of the chosen rows: gather from the full tensors
    q_full, k_full, v_full = H.dev(w.q_full, dt), H.dev(w.k_full, dt), H.dev(w.v_full, dt)
    ctx.fr_rope_shift(H.dev(w.k_cached, dt), k_cache, w.chunk_offsets, w.src_pos0)
    ctx.fr_score_select(q_full[w.L_ctx:].contiguous(), w.nq, k_cache, w.chunk_offsets, k, B.FR_NORM_PER_CHUNK, None, qi)
    idx = qi.long()
    q_rows, k_new, v_new = q_full[idx].contiguous(), k_full[idx].contiguous(), v_full[idx].contiguous()
    out = torch.empty((R, Hq, d), dtype=tdt, device="cuda")
    ctx.fr_sparse_prefill_attn(q_rows, qi, R, k_cache, v_cache, w.L, k_new, v_new, out)
    ctx.fr_kv_scatter(k_new, v_new, qi, R, k_cache, v_cache, w.L)
    torch.cuda.synchronize()
    qi_g = qi.cpu().numpy().astype(np.int64)
    H.assert_index_set(qi_g, scores_o, k, w.nq)
    # attention and cache are compared on the index set the GPU chose (identical to the oracle's apart from ties)
    kc_o, vc_o = np.zeros((w.L, Hkv, d)), np.zeros((w.L, Hkv, d))
    kc_o[: w.L_ctx], vc_o[: w.L_ctx] = k_ctx_o, w.v_cached
    want, _ = orc.sparse_prefill_attn(w.q_full[qi_g], qi_g, kc_o, vc_o, w.k_full[qi_g], w.v_full[qi_g])
    H.assert_close(H.host(out), want, dt, "chained attention")
    want_k, want_v = orc.kv_scatter(qi_g, w.k_full[qi_g], w.v_full[qi_g], kc_o, vc_o)
    H.assert_close(H.host(k_cache), want_k, dt, "chained K cache")
    assert np.array_equal(H.host(v_cache), want_v)
    ctx.close()


def test_layer_under_hip_graph():
    """The four calls captured once into a HIP graph and replayed with different cache contents, the program's own eager
    work and synchronisations between the replays: every replay equals the eager calls on the same inputs bit for bit
    (the calls allocate nothing, synchronise nothing and clear their scratch with kernels, so they can be captured)."""
    w = workloads()["small_bf16"](2)
    dt, tdt = w.shape.dtype, H.TORCH_DTYPE[w.shape.dtype]
    Hq, Hkv, d = w.shape.n_q_heads, w.shape.n_kv_heads, w.shape.head_dim
    _, _, k, _ = staged(w)
    R = k + w.nq
    ctx = H.make_ctx(w.shape, w.L, w.n_chunks, w.nq)
    rng = np.random.default_rng(4)
    variants = [(H.dev(w.k_cached, dt), H.dev(w.v_cached, dt))]
    for _ in range(2):   # two more stale caches of the same prompt
        noise = lambda a: synth.round_to_storage((a + 0.2 * rng.standard_normal(a.shape) * a.std()).astype(np.float32), dt)
        variants.append((H.dev(noise(w.k_cached), dt), H.dev(noise(w.v_cached), dt)))
    q_question = H.dev(w.q_question, dt)
    q_full, k_full, v_full = H.dev(w.q_full, dt), H.dev(w.k_full, dt), H.dev(w.v_full, dt)
    # static buffers of the captured step
    k_in = torch.empty_like(variants[0][0])
    k_cache = torch.zeros((w.L, Hkv, d), dtype=tdt, device="cuda")
    v_cache = torch.zeros((w.L, Hkv, d), dtype=tdt, device="cuda")
    qi = torch.empty(R, dtype=torch.int32, device="cuda")
    q_rows = torch.empty((R, Hq, d), dtype=tdt, device="cuda")
    k_new = torch.empty((R, Hkv, d), dtype=tdt, device="cuda")
    v_new = torch.empty((R, Hkv, d), dtype=tdt, device="cuda")
    out = torch.empty((R, Hq, d), dtype=tdt, device="cuda")

    def step():
        ctx.fr_rope_shift(k_in, k_cache, w.chunk_offsets, w.src_pos0)
        ctx.fr_score_select(q_question, w.nq, k_cache, w.chunk_offsets, k, B.FR_NORM_PER_CHUNK, None, qi)
        idx = qi.long()                                   # the harness's stand-in for the QKV projection of the chosen rows
        q_rows.copy_(q_full[idx]); k_new.copy_(k_full[idx]); v_new.copy_(v_full[idx])
        ctx.fr_sparse_prefill_attn(q_rows, qi, R, k_cache, v_cache, w.L, k_new, v_new, out)
        ctx.fr_kv_scatter(k_new, v_new, qi, R, k_cache, v_cache, w.L)

    def load(i):
        k_in.copy_(variants[i][0])
        v_cache.zero_()
        v_cache[: w.L_ctx] = variants[i][1]

    eager = []
    for i in range(3):
        load(i)
        step()
        torch.cuda.synchronize()
        eager.append((qi.clone(), out.clone(), k_cache.clone(), v_cache.clone()))
    graph = torch.cuda.CUDAGraph()
    load(0)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        step()
    for i in (1, 0, 2, 1):
        load(i)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        want = eager[i]
        assert torch.equal(qi, want[0]) and torch.equal(out, want[1])
        assert torch.equal(k_cache, want[2]) and torch.equal(v_cache, want[3])
    ctx.close()


def test_attention_softmax_modes_agree():
    """The running-maximum kernel alone (forced through fr_set_option) gives the oracle's result too."""
    w = workloads()["small_bf16"](5)
    k_ctx, _, k, qi = staged(w)
    k_cache, v_cache = assembled_cache(w, k_ctx)
    ctx = H.make_ctx(w.shape, w.L, w.n_chunks, w.nq)
    want, want_lse = orc.sparse_prefill_attn(w.q_full[qi], qi, k_cache, v_cache, w.k_full[qi], w.v_full[qi])
    ctx.fr_set_option(B.FR_OPT_ATTN_SOFTMAX, B.FR_ATTN_SOFTMAX_RUNNING_MAX)
    got, lse = run_attention(ctx, w, qi, k_cache, v_cache)
    H.assert_close(got, want, "bf16", "running-max attention")
    assert np.max(np.abs(lse - want_lse)) <= 2e-3
    ctx.fr_set_option(B.FR_OPT_ATTN_SOFTMAX, B.FR_ATTN_SOFTMAX_AUTO)
    got2, _ = run_attention(ctx, w, qi, k_cache, v_cache)
    H.assert_close(got2, want, "bf16", "default attention")
    with pytest.raises(B.FusionRAGError):
        ctx.fr_set_option(B.FR_OPT_ATTN_SOFTMAX, 7)
    ctx.close()


def test_attention_logits_far_above_the_first_keys():
    """Degenerate case of the fixed exponent reference: logits that grow along the sequence until exp2 would
    overflow against the maximum of the first 32 keys.  The default path must still match the oracle (the
    overflowing workgroups are recomputed with a running maximum)."""
    shape = synth.LLAMA3_8B_BF16
    rng = np.random.default_rng(11)
    L_ctx, nq, d = 600, 24, shape.head_dim
    L = L_ctx + nq
    u = rng.standard_normal(d)
    u /= np.linalg.norm(u)
    ramp = np.linspace(0.0, 1.0, L)[:, None, None]                       # key j gains ramp_j * 180 * u
    k_all = rng.standard_normal((L, shape.n_kv_heads, d)) * 0.05 + ramp * 180.0 * u
    q_all = rng.standard_normal((L, shape.n_q_heads, d)) * 0.05 + 12.0 * u   # logit ~ 12*180*ramp/sqrt(128) ~ 190*ramp
    v_all = rng.standard_normal((L, shape.n_kv_heads, d))
    r = lambda a: synth.round_to_storage(a.astype(np.float32), "bf16")
    k_all, q_all, v_all = r(k_all), r(q_all), r(v_all)
    sel = np.sort(rng.choice(L_ctx, size=90, replace=False))
    qi = np.concatenate([sel, L_ctx + np.arange(nq)])
    w = synth.Workload("ramp", shape, 0, np.array([0, L_ctx], np.int32), np.zeros(1, np.int32), nq, 0.15,
                       k_all[:L_ctx], v_all[:L_ctx], q_all, k_all, v_all, np.zeros(0, np.int64))
    ctx = H.make_ctx(shape, L, 1, nq)
    got, lse = run_attention(ctx, w, qi, k_all, v_all)
    want, want_lse = orc.sparse_prefill_attn(q_all[qi], qi, k_all, v_all, k_all[qi], v_all[qi])
    H.assert_close(got, want, "bf16", "attention with runaway logits")
    assert np.max(np.abs(lse - want_lse) / np.abs(want_lse)) <= 1e-3
    ctx.close()


@pytest.mark.parametrize("ratio", [0.0, 0.15, 1.0])
@pytest.mark.parametrize("seed", [3, 4])
def test_attention_split_key_range(seed, ratio):
    """The key range of every (row tile, KV head) walked by two workgroups (forced; AUTO picks it only for long
    prompts with few rows): same oracle, same tolerance, and the unsplit launch agrees to fp32 summation order.
    Row tiles at positions < 64 have a single key tile: their second part is empty."""
    w = synth.config_small_bf16(seed=seed, ratio=ratio)
    dt = w.shape.dtype
    k_ctx, scores, _, _ = staged(w)
    k = orc.topk_count(w.L_ctx, ratio)
    qi = orc.select_q_index(scores, k, w.nq)
    k_cache, v_cache = assembled_cache(w, k_ctx)
    ctx = H.make_ctx(w.shape, w.L, w.n_chunks, w.nq)
    want, want_lse = orc.sparse_prefill_attn(w.q_full[qi], qi, k_cache, v_cache, w.k_full[qi], w.v_full[qi])
    ctx.fr_set_option(B.FR_OPT_ATTN_SPLIT, B.FR_ATTN_SPLIT_ON)
    got, lse = run_attention(ctx, w, qi, k_cache, v_cache)
    H.assert_close(got, want, dt, "split attention")
    assert np.max(np.abs(lse - want_lse)) <= 2e-3
    ctx.fr_set_option(B.FR_OPT_ATTN_SPLIT, B.FR_ATTN_SPLIT_OFF)
    got1, lse1 = run_attention(ctx, w, qi, k_cache, v_cache)
    assert H.max_rel_err(got, got1) <= 2.0 ** -7          # at most one bf16 rounding step apart
    assert np.max(np.abs(lse - lse1)) <= 1e-5
    with pytest.raises(B.FusionRAGError):
        ctx.fr_set_option(B.FR_OPT_ATTN_SPLIT, 9)
    ctx.close()


@pytest.mark.parametrize("name", ["tiny_f32", "small_bf16"])
def test_attention_with_fused_writeback(name):
    """fr_sparse_prefill_attn_writeback = attention + write-back in one call: output and caches equal the two-call path
    bit for bit (the tiled path fuses the copy into its packing pass, the generic path runs the scatter kernel)."""
    w = workloads()[name](6)
    dt, tdt = w.shape.dtype, H.TORCH_DTYPE[w.shape.dtype]
    k_ctx, _, _, qi = staged(w)
    k_cache, v_cache = assembled_cache(w, k_ctx)
    R = len(qi)
    ctx = H.make_ctx(w.shape, w.L, w.n_chunks, w.nq)
    q_rows, k_new, v_new = H.dev(w.q_full[qi], dt), H.dev(w.k_full[qi], dt), H.dev(w.v_full[qi], dt)
    qi_d = torch.from_numpy(qi.astype(np.int32)).cuda()
    kc1, vc1 = H.dev(k_cache, dt), H.dev(v_cache, dt)
    kc2, vc2 = kc1.clone(), vc1.clone()
    out1 = torch.zeros((R, w.shape.n_q_heads, w.shape.head_dim), dtype=tdt, device="cuda")
    out2 = torch.zeros_like(out1)
    ctx.fr_sparse_prefill_attn(q_rows, qi_d, R, kc1, vc1, w.L, k_new, v_new, out1)
    ctx.fr_kv_scatter(k_new, v_new, qi_d, R, kc1, vc1, w.L)
    ctx.fr_sparse_prefill_attn_writeback(q_rows, qi_d, R, kc2, vc2, w.L, k_new, v_new, out2)
    torch.cuda.synchronize()
    assert torch.equal(out1, out2) and torch.equal(kc1, kc2) and torch.equal(vc1, vc2)
    want_k, want_v = orc.kv_scatter(qi, w.k_full[qi], w.v_full[qi], k_cache, v_cache)
    assert np.array_equal(H.host(kc2), want_k) and np.array_equal(H.host(vc2), want_v)
    with pytest.raises(B.FusionRAGError):
        ctx.fr_sparse_prefill_attn_writeback(q_rows, qi_d, R, kc2, vc2, w.L, None, None, out2)
    ctx.close()


def test_attention_kernel_timer():
    """The optional event pairs around the dominant attention kernel: one duration per launch, the most recent kept."""
    w = synth.config_small_bf16(seed=2)
    k_ctx, _, _, qi = staged(w)
    k_cache, v_cache = assembled_cache(w, k_ctx)
    ctx = H.make_ctx(w.shape, w.L, w.n_chunks, w.nq)
    assert ctx.fr_attn_kernel_times() == []
    ctx.fr_set_option(B.FR_OPT_ATTN_KERNEL_TIMER, 3)
    for _ in range(5):
        got, _ = run_attention(ctx, w, qi, k_cache, v_cache)
    ms = ctx.fr_attn_kernel_times()
    assert len(ms) == 3 and all(0.0 < t < 50.0 for t in ms)
    ctx.fr_set_option(B.FR_OPT_ATTN_KERNEL_TIMER, 0)
    got2, _ = run_attention(ctx, w, qi, k_cache, v_cache)
    assert np.array_equal(got, got2) and ctx.fr_attn_kernel_times() == []
    with pytest.raises(B.FusionRAGError):
        ctx.fr_set_option(B.FR_OPT_ATTN_KERNEL_TIMER, 1000)
    ctx.close()


def test_attention_split_with_runaway_logits():
    """Split launch + overflow of the fixed exponent reference: the combine step must flag the workgroups and the
    running-maximum kernel recompute them."""
    shape = synth.LLAMA3_8B_BF16
    rng = np.random.default_rng(12)
    L_ctx, nq, d = 500, 40, shape.head_dim
    L = L_ctx + nq
    u = rng.standard_normal(d)
    u /= np.linalg.norm(u)
    ramp = np.linspace(0.0, 1.0, L)[:, None, None]
    r = lambda a: synth.round_to_storage(a.astype(np.float32), "bf16")
    k_all = r(rng.standard_normal((L, shape.n_kv_heads, d)) * 0.05 + ramp * 180.0 * u)
    q_all = r(rng.standard_normal((L, shape.n_q_heads, d)) * 0.05 + 12.0 * u)
    v_all = r(rng.standard_normal((L, shape.n_kv_heads, d)))
    sel = np.sort(rng.choice(L_ctx, size=70, replace=False))
    qi = np.concatenate([sel, L_ctx + np.arange(nq)])
    w = synth.Workload("ramp", shape, 0, np.array([0, L_ctx], np.int32), np.zeros(1, np.int32), nq, 0.15,
                       k_all[:L_ctx], v_all[:L_ctx], q_all, k_all, v_all, np.zeros(0, np.int64))
    ctx = H.make_ctx(shape, L, 1, nq)
    ctx.fr_set_option(B.FR_OPT_ATTN_SPLIT, B.FR_ATTN_SPLIT_ON)
    got, lse = run_attention(ctx, w, qi, k_all, v_all)
    want, want_lse = orc.sparse_prefill_attn(q_all[qi], qi, k_all, v_all, k_all[qi], v_all[qi])
    H.assert_close(got, want, "bf16", "split attention with runaway logits")
    assert np.max(np.abs(lse - want_lse) / np.abs(want_lse)) <= 1e-3
    ctx.close()


@pytest.mark.parametrize("ratio", [0.05, 0.30, 1.0])
def test_full_size_ratio_sweep_sampled(ratio):
    """Config 3's sweep on config 2's prompt, in the launch configuration of `bench.py --ratio`: at 5 % there are few row
    tiles, so the default launch splits the key range; at 30 % and 100 % it does not; 100 % is full causal prefill.
    Attention output checked against the oracle on sampled rows."""
    w = synth.config_17k(seed=0, ratio=ratio)
    dt = w.shape.dtype
    rng = np.random.default_rng(0)
    k = orc.topk_count(w.L_ctx, w.ratio)
    sel = np.sort(rng.choice(w.L_ctx, size=k, replace=False))     # any index set will do for the attention call
    qi = np.concatenate([sel, w.L_ctx + np.arange(w.nq)]).astype(np.int64)
    k_cache = np.concatenate([w.k_cached, w.k_full[w.L_ctx:]])   # stale keys as they are: the call takes any cache
    v_cache = np.concatenate([w.v_cached, w.v_full[w.L_ctx:]])
    ctx = H.make_ctx(w.shape, w.L, w.n_chunks, w.nq)
    got, lse = run_attention(ctx, w, qi, k_cache, v_cache)
    rows = np.unique(np.concatenate([[0, 1, len(qi) - 1], rng.choice(len(qi), size=48, replace=False)]))
    want, want_lse = orc.sparse_prefill_attn(w.q_full[qi], qi, k_cache, v_cache, w.k_full[qi], w.v_full[qi], rows=rows)
    H.assert_close(got[rows], want, dt, "sampled rows of the split launch")
    assert np.max(np.abs(lse[rows] - want_lse)) <= 2e-3
    ctx.close()


@pytest.mark.parametrize("config_id,n_sample", [(2, 96), (4, 64)])
def test_full_size_chain_sampled(config_id, n_sample):
    """The benchmark's configurations at full size, in the launch configuration bench.py times: the whole chain
    on the GPU; the oracle checks the Q index (all of it), the shifted keys and the attention output on a
    sample of rows it can compute one by one, and the scattered cache on the sampled rows."""
    w = synth.CONFIGS[config_id](seed=0)
    dt, tdt = w.shape.dtype, H.TORCH_DTYPE[w.shape.dtype]
    Hq, Hkv, d = w.shape.n_q_heads, w.shape.n_kv_heads, w.shape.head_dim
    k = B.fr_topk_count(w.L_ctx, w.ratio)
    R = k + w.nq
    ctx = H.make_ctx(w.shape, w.L, w.n_chunks, w.nq)
    k_cache = torch.zeros((w.L, Hkv, d), dtype=tdt, device="cuda")
    v_cache = torch.zeros((w.L, Hkv, d), dtype=tdt, device="cuda")
    v_cache[: w.L_ctx] = H.dev(w.v_cached, dt)
    qi = torch.empty(R, dtype=torch.int32, device="cuda")
    scores = torch.empty(w.L_ctx, dtype=torch.float32, device="cuda")
    ctx.fr_rope_shift(H.dev(w.k_cached, dt), k_cache, w.chunk_offsets, w.src_pos0)
    k_ctx_gpu = H.host(k_cache[: w.L_ctx])
    ctx.fr_score_select(H.dev(w.q_question, dt), w.nq, k_cache, w.chunk_offsets, k, B.FR_NORM_PER_CHUNK, scores, qi)
    idx = qi.long()
    q_rows = H.dev(w.q_full, dt)[idx].contiguous()
    k_new, v_new = H.dev(w.k_full, dt)[idx].contiguous(), H.dev(w.v_full, dt)[idx].contiguous()
    out = torch.empty((R, Hq, d), dtype=tdt, device="cuda")
    ctx.fr_sparse_prefill_attn(q_rows, qi, R, k_cache, v_cache, w.L, k_new, v_new, out)
    ctx.fr_kv_scatter(k_new, v_new, qi, R, k_cache, v_cache, w.L)
    torch.cuda.synchronize()

    k_ctx_o = orc.rope_shift(w.k_cached, w.chunk_offsets, w.src_pos0, None, w.shape.rope_base)
    H.assert_close(k_ctx_gpu, k_ctx_o, dt, "shifted keys")
    k_ctx_r = synth.round_to_storage(k_ctx_o, dt)
    scores_o = orc.critical_scores(w.q_question, k_ctx_r, w.chunk_offsets)
    assert H.max_rel_err(scores.cpu().numpy().astype(np.float64), scores_o) <= 2e-3   # the GPU scored its own shifted keys
    qi_g = qi.cpu().numpy().astype(np.int64)
    H.assert_index_set(qi_g, scores_o, k, w.nq)
    kc = np.zeros((w.L, Hkv, d), np.float32)
    vc = np.zeros((w.L, Hkv, d), np.float32)
    kc[: w.L_ctx], vc[: w.L_ctx] = k_ctx_r, w.v_cached
    rows = np.unique(np.linspace(0, R - 1, n_sample).round().astype(np.int64))
    want, _ = orc.sparse_prefill_attn(w.q_full[qi_g], qi_g, kc, vc, w.k_full[qi_g], w.v_full[qi_g], rows=rows)
    H.assert_close(H.host(out[torch.from_numpy(rows).cuda()]), want, dt, "sampled attention rows")
    pos = qi_g[rows]
    assert np.array_equal(H.host(k_cache[torch.from_numpy(pos).cuda()]), w.k_full[pos].astype(np.float64))
    assert np.array_equal(H.host(v_cache[torch.from_numpy(pos).cuda()]), w.v_full[pos].astype(np.float64))
    ctx.close()

"""GPU parity of the model steps around the path (RMSNorm, projections with fused epilogues) against the oracle."""
import numpy as np
import pytest
import torch

from oracle import fusionrag_oracle as orc
from paper_2601_12904_amd import binding as B
from paper_2601_12904_amd import synth
from tests import harness as H

pytestmark = pytest.mark.gpu
SHAPE = synth.LLAMA3_8B_BF16


def bf(x):
    return synth.round_to_storage(np.asarray(x, dtype=np.float32), "bf16")


@pytest.fixture()
def ctx():
    c = H.make_ctx(SHAPE, 4096, 4, 64)
    yield c
    c.close()


@pytest.mark.parametrize("M,N,K", [(1, 128, 64), (130, 256, 192), (300, 384, 1024), (257, 128, 4096)])
def test_linear(ctx, M, N, K):
    rng = np.random.default_rng(M + N + K)
    a, w, r = bf(rng.standard_normal((M, K))), bf(rng.standard_normal((N, K)) * 0.05), bf(rng.standard_normal((M, N)))
    out = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
    ctx.fr_linear(H.dev(a, "bf16"), H.dev(w, "bf16"), M, N, K, None, out)
    torch.cuda.synchronize()
    H.assert_close(H.host(out), orc.linear(a, w), "bf16", "linear")
    res = H.dev(r, "bf16")
    ctx.fr_linear(H.dev(a, "bf16"), H.dev(w, "bf16"), M, N, K, res, res)       # in place on the residual
    torch.cuda.synchronize()
    H.assert_close(H.host(res), orc.linear(a, w, r), "bf16", "linear + residual")


@pytest.mark.parametrize("tile", [128, 256])
@pytest.mark.parametrize("M,N,K", [(130, 256, 192), (300, 384, 1024), (129, 512, 4096)])
def test_linear_both_tilings(ctx, M, N, K, tile):
    """Both workgroup tilings forced (the default picks by feature count); N = 384 with 256-feature workgroups has a
    half-empty last feature tile."""
    rng = np.random.default_rng(M + N + K + tile)
    a, w = bf(rng.standard_normal((M, K))), bf(rng.standard_normal((N, K)) * 0.05)
    out = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
    ctx.fr_set_option(B.FR_OPT_GEMM_TILE, tile)
    try:
        ctx.fr_linear(H.dev(a, "bf16"), H.dev(w, "bf16"), M, N, K, None, out)
        torch.cuda.synchronize()
    finally:
        ctx.fr_set_option(B.FR_OPT_GEMM_TILE, 0)
    H.assert_close(H.host(out), orc.linear(a, w), "bf16", f"linear, {tile}-feature workgroups")
    with pytest.raises(B.FusionRAGError):
        ctx.fr_set_option(B.FR_OPT_GEMM_TILE, 64)


@pytest.mark.parametrize("split", [0, 1])
@pytest.mark.parametrize("tile", [128, 256])
@pytest.mark.parametrize("K", [2 * 16 * 64, 2 * 96 * 64])   # two parts of 16 K tiles: the shortest split the launcher makes
def test_epilogues_with_and_without_tail_split(ctx, tile, split, K):
    """Few output tiles and a long K: every tile belongs to the launch's last round and is computed by several
    workgroups along K, whose partial sums a second kernel adds before the epilogue (residual, SwiGLU, rotary Q/K/V).
    Forced off for comparison: same oracle, same tolerance."""
    rng = np.random.default_rng(40 + tile + split + K)
    Hq, Hkv, d = SHAPE.n_q_heads, SHAPE.n_kv_heads, SHAPE.head_dim
    M = 300
    a = bf(rng.standard_normal((M, K)))
    ctx.fr_set_option(B.FR_OPT_GEMM_TILE, tile)
    ctx.fr_set_option(B.FR_OPT_GEMM_TAIL_SPLIT, split)
    try:
        w, r = bf(rng.standard_normal((384, K)) * 0.05), bf(rng.standard_normal((M, 384)))
        res = H.dev(r, "bf16")
        ctx.fr_linear(H.dev(a, "bf16"), H.dev(w, "bf16"), M, 384, K, res, res)
        wg = bf(rng.standard_normal((2 * 192, K)) * 0.05)
        sw = torch.zeros((M, 192), dtype=torch.bfloat16, device="cuda")
        ctx.fr_linear_swiglu(H.dev(a, "bf16"), H.dev(wg, "bf16"), M, 192, K, sw)
        wq = bf(rng.standard_normal(((Hq + 2 * Hkv) * d, K)) * 0.05)
        pos = np.sort(rng.choice(4000, size=M, replace=False)).astype(np.int32)
        q = torch.zeros((M, Hq, d), dtype=torch.bfloat16, device="cuda")
        k = torch.zeros((M, Hkv, d), dtype=torch.bfloat16, device="cuda")
        v = torch.zeros((M, Hkv, d), dtype=torch.bfloat16, device="cuda")
        ctx.fr_qkv_rope(H.dev(a, "bf16"), H.dev(wq, "bf16"), M, K, torch.from_numpy(pos).cuda(), q, k, v)
        torch.cuda.synchronize()
    finally:
        ctx.fr_set_option(B.FR_OPT_GEMM_TILE, 0)
        ctx.fr_set_option(B.FR_OPT_GEMM_TAIL_SPLIT, 1)
    H.assert_close(H.host(res), orc.linear(a, w, r), "bf16", "linear + residual")
    H.assert_close(H.host(sw), orc.linear_swiglu(a, wg), "bf16", "swiglu")
    qo, ko, vo = orc.qkv_rope(a, wq, pos, Hq, Hkv, d, SHAPE.rope_base)
    H.assert_close(H.host(q), qo, "bf16", "q")
    H.assert_close(H.host(k), ko, "bf16", "k")
    H.assert_close(H.host(v), vo, "bf16", "v")
    with pytest.raises(B.FusionRAGError):
        ctx.fr_set_option(B.FR_OPT_GEMM_TAIL_SPLIT, 2)


@pytest.mark.parametrize("M,F,K", [(70, 64, 128), (300, 192, 320)])
def test_linear_swiglu(ctx, M, F, K):
    rng = np.random.default_rng(M + F)
    a, w = bf(rng.standard_normal((M, K))), bf(rng.standard_normal((2 * F, K)) * 0.1)
    out = torch.zeros((M, F), dtype=torch.bfloat16, device="cuda")
    ctx.fr_linear_swiglu(H.dev(a, "bf16"), H.dev(w, "bf16"), M, F, K, out)
    torch.cuda.synchronize()
    H.assert_close(H.host(out), orc.linear_swiglu(a, w), "bf16", "swiglu")


@pytest.mark.parametrize("M,K", [(5, 64), (333, 256)])
def test_qkv_rope(ctx, M, K):
    rng = np.random.default_rng(M)
    Hq, Hkv, d = SHAPE.n_q_heads, SHAPE.n_kv_heads, SHAPE.head_dim
    a, w = bf(rng.standard_normal((M, K))), bf(rng.standard_normal(((Hq + 2 * Hkv) * d, K)) * 0.1)
    pos = np.sort(rng.choice(4000, size=M, replace=False)).astype(np.int32)
    q = torch.zeros((M, Hq, d), dtype=torch.bfloat16, device="cuda")
    k = torch.zeros((M, Hkv, d), dtype=torch.bfloat16, device="cuda")
    v = torch.zeros((M, Hkv, d), dtype=torch.bfloat16, device="cuda")
    ctx.fr_qkv_rope(H.dev(a, "bf16"), H.dev(w, "bf16"), M, K, torch.from_numpy(pos).cuda(), q, k, v)
    torch.cuda.synchronize()
    qo, ko, vo = orc.qkv_rope(a, w, pos, Hq, Hkv, d, SHAPE.rope_base)
    H.assert_close(H.host(q), qo, "bf16", "q")
    H.assert_close(H.host(k), ko, "bf16", "k")
    H.assert_close(H.host(v), vo, "bf16", "v")


@pytest.mark.parametrize("R,hidden", [(1, 64), (37, 4096), (130, 520)])
def test_rmsnorm(ctx, R, hidden):
    rng = np.random.default_rng(R)
    x, g = bf(rng.standard_normal((R, hidden)) * 3), bf(1 + 0.1 * rng.standard_normal(hidden))
    out = torch.zeros((R, hidden), dtype=torch.bfloat16, device="cuda")
    ctx.fr_rmsnorm(H.dev(x, "bf16"), H.dev(g, "bf16"), R, hidden, 1e-5, out)
    torch.cuda.synchronize()
    H.assert_close(H.host(out), orc.rmsnorm(x, g, 1e-5), "bf16", "rmsnorm")


def test_two_layer_stack_against_oracle():
    """A small Llama-shaped stack (real head geometry, reduced widths) end to end: every layer's output rows,
    fresh K/V and written-back cache against the oracle, which follows the pipeline store by store."""
    from paper_2601_12904_amd import stack as S
    rng = np.random.default_rng(3)
    hidden, ffn, n_layers = 256, 384, 2
    Hq, Hkv, d = SHAPE.n_q_heads, SHAPE.n_kv_heads, SHAPE.head_dim
    w = synth.config_small_bf16(seed=7, chunk_lens=(150, 90, 201), nq=24)
    k = orc.topk_count(w.L_ctx, 0.2)
    sel = np.sort(rng.choice(w.L_ctx, size=k, replace=False))
    qi = np.concatenate([sel, w.L_ctx + np.arange(w.nq)]).astype(np.int64)
    R = len(qi)
    ctx = H.make_ctx(SHAPE, w.L, w.n_chunks, w.nq)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    layers = [S.random_layer(hidden, ffn, Hq, Hkv, d, gen, std=0.08) for _ in range(n_layers)]
    st = S.SelectivePrefillStack(ctx, layers, hidden, ffn)
    h0 = bf(rng.standard_normal((R, hidden)))
    kc_src = [bf(rng.standard_normal(w.k_cached.shape) * 0.3) for _ in range(n_layers)]
    vc_src = [bf(rng.standard_normal(w.v_cached.shape)) for _ in range(n_layers)]
    k_cached = [H.dev(a, "bf16") for a in kc_src]
    k_cache = [torch.zeros((w.L, Hkv, d), dtype=torch.bfloat16, device="cuda") for _ in range(n_layers)]
    v_cache = [torch.zeros((w.L, Hkv, d), dtype=torch.bfloat16, device="cuda") for _ in range(n_layers)]
    for l in range(n_layers):
        v_cache[l][: w.L_ctx] = H.dev(vc_src[l], "bf16")
    h = H.dev(h0, "bf16")
    qi_d = torch.from_numpy(qi.astype(np.int32)).cuda()
    scratch = torch.empty(R, dtype=torch.int32, device="cuda")
    st.forward(h, qi_d, k_cached, k_cache, v_cache, w.chunk_offsets, w.src_pos0, w.nq, w.L,
               select_every_layer=True, k_select=k, q_index_scratch=scratch)
    torch.cuda.synchronize()

    rnd = lambda t: synth.round_to_storage(np.asarray(t, dtype=np.float32), "bf16").astype(np.float64)
    ho = h0.astype(np.float64)
    for l, lw in enumerate(layers):
        wd = {n: H.host(getattr(lw, n)) for n in ("g1", "w_qkv", "w_o", "g2", "w_gate_up", "w_down")}
        kc = np.zeros((w.L, Hkv, d))
        vc = np.zeros((w.L, Hkv, d))
        kc[: w.L_ctx] = rnd(orc.rope_shift(kc_src[l], w.chunk_offsets, w.src_pos0, None, SHAPE.rope_base))
        vc[: w.L_ctx] = vc_src[l]
        ho, k_new, v_new = orc.selective_prefill_layer(ho, qi, kc, vc, wd, Hq, Hkv, d, SHAPE.rope_base, 1e-5, round_fn=rnd)
        want_k, want_v = orc.kv_scatter(qi, k_new, v_new, kc, vc)
        H.assert_close(H.host(k_cache[l]), want_k, "bf16", f"layer {l} K cache")
        H.assert_close(H.host(v_cache[l]), want_v, "bf16", f"layer {l} V cache")
    H.assert_close(H.host(h), ho, "bf16", "stack output")
    ctx.close()


def test_full_size_layer_sampled():
    """One decoder layer at the benchmark's size (hidden 4096, FFN 14336, config 2's prompt: 2970 rows at 15 %), in the
    launch configuration `bench.py --config 5` times (256-feature workgroups, last round of each projection split along
    K): the fresh K/V of all rows and the layer output on sampled rows against the oracle, which follows the pipeline
    store by store (the Q/K/V projection for all rows, everything after it for the sampled ones)."""
    from paper_2601_12904_amd import stack as S
    rng = np.random.default_rng(12)
    hidden, ffn = 4096, 14336
    Hq, Hkv, d = SHAPE.n_q_heads, SHAPE.n_kv_heads, SHAPE.head_dim
    w = synth.config_17k(seed=0)
    k = orc.topk_count(w.L_ctx, w.ratio)
    sel = np.sort(rng.choice(w.L_ctx, size=k, replace=False))
    qi = np.concatenate([sel, w.L_ctx + np.arange(w.nq)]).astype(np.int64)
    R = len(qi)
    ctx = H.make_ctx(SHAPE, w.L, w.n_chunks, w.nq)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(8)
    layer = S.random_layer(hidden, ffn, Hq, Hkv, d, gen)
    st = S.SelectivePrefillStack(ctx, [layer], hidden, ffn)
    h0 = bf(rng.standard_normal((R, hidden)))
    k_cache = torch.zeros((w.L, Hkv, d), dtype=torch.bfloat16, device="cuda")
    v_cache = torch.zeros((w.L, Hkv, d), dtype=torch.bfloat16, device="cuda")
    v_cache[: w.L_ctx] = H.dev(w.v_cached, "bf16")
    h = H.dev(h0, "bf16")
    qi_d = torch.from_numpy(qi.astype(np.int32)).cuda()
    st.forward(h, qi_d, [H.dev(w.k_cached, "bf16")], [k_cache], [v_cache], w.chunk_offsets, w.src_pos0, w.nq, w.L)
    torch.cuda.synchronize()

    rnd = lambda t: synth.round_to_storage(np.asarray(t, dtype=np.float32), "bf16").astype(np.float64)
    wd = {n: H.host(getattr(layer, n)) for n in ("g1", "w_qkv", "w_o", "g2", "w_gate_up", "w_down")}
    kc = np.zeros((w.L, Hkv, d))
    vc = np.zeros((w.L, Hkv, d))
    kc[: w.L_ctx] = rnd(orc.rope_shift(w.k_cached, w.chunk_offsets, w.src_pos0, None, SHAPE.rope_base))
    vc[: w.L_ctx] = w.v_cached
    rows = np.unique(np.concatenate([[0, R - 1], rng.choice(R, size=14, replace=False)]))
    ho, k_new, v_new = orc.selective_prefill_layer(h0.astype(np.float64), qi, kc, vc, wd, Hq, Hkv, d, SHAPE.rope_base, 1e-5,
                                                   round_fn=rnd, rows=rows)
    idx = torch.from_numpy(qi).cuda()
    H.assert_close(H.host(k_cache[idx]), k_new, "bf16", "fresh K rows written back")
    H.assert_close(H.host(v_cache[idx]), v_new, "bf16", "fresh V rows written back")
    H.assert_close(H.host(h[torch.from_numpy(rows).cuda()]), ho, "bf16", "layer output, sampled rows")
    ctx.close()


@pytest.fixture(scope="module")
def full_stack_run():
    """The 32-layer stack of the full-stack configuration (hidden 4096, FFN 14336, config 2's prompt, 2970 rows) run
    once on the GPU; inputs and outputs of layers 1, 15 and 31 are kept for the teacher-forced checks below."""
    from paper_2601_12904_amd import stack as S
    hidden, ffn, n_layers = 4096, 14336, 32
    Hq, Hkv, d = SHAPE.n_q_heads, SHAPE.n_kv_heads, SHAPE.head_dim
    w = synth.config_17k(seed=0)
    rng = np.random.default_rng(21)
    k = orc.topk_count(w.L_ctx, w.ratio)
    qi = np.concatenate([np.sort(rng.choice(w.L_ctx, size=k, replace=False)), w.L_ctx + np.arange(w.nq)]).astype(np.int64)
    R = len(qi)
    ctx = H.make_ctx(SHAPE, w.L, w.n_chunks, w.nq)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(9)
    layers = [S.random_layer(hidden, ffn, Hq, Hkv, d, gen) for _ in range(n_layers)]
    st = S.SelectivePrefillStack(ctx, layers, hidden, ffn)
    sig = 1.0 / np.sqrt(d)
    bf16 = torch.bfloat16
    k_cached = [(torch.randn((w.L_ctx, Hkv, d), generator=gen, device="cuda") * sig).to(bf16) for _ in range(n_layers)]
    k_cache = [torch.zeros((w.L, Hkv, d), dtype=bf16, device="cuda") for _ in range(n_layers)]
    v_cache = [torch.zeros((w.L, Hkv, d), dtype=bf16, device="cuda") for _ in range(n_layers)]
    v_src = {}
    for l, vc in enumerate(v_cache):
        vc[: w.L_ctx] = (torch.randn((w.L_ctx, Hkv, d), generator=gen, device="cuda") * sig).to(bf16)
        if l in (1, 15, 31):
            v_src[l] = H.host(vc[: w.L_ctx])
    h = torch.randn((R, hidden), generator=gen, device="cuda").to(bf16)
    capture = {1: {}, 15: {}, 31: {}}
    st.forward(h, torch.from_numpy(qi.astype(np.int32)).cuda(), k_cached, k_cache, v_cache, w.chunk_offsets, w.src_pos0,
               w.nq, w.L, capture=capture)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(h.float()).all())
    run = dict(w=w, qi=qi, layers=layers, capture=capture, v_src=v_src,
               k_cached={l: H.host(k_cached[l]) for l in capture},
               k_cache={l: k_cache[l] for l in capture}, v_cache={l: v_cache[l] for l in capture})
    yield run
    ctx.close()


@pytest.mark.parametrize("layer", [1, 15, 31])
def test_full_size_stack_layers_teacher_forced(full_stack_run, layer):
    """Layers 1, 15 and 31 of the 32-layer run, each checked on its own: the oracle is given the rows the GPU fed into
    that layer (so errors of the layers before do not accumulate into the comparison) and follows the pipeline store
    by store; compared are the fresh K/V the layer wrote back (all rows) and its output on sampled rows."""
    r = full_stack_run
    w, qi, lw = r["w"], r["qi"], r["layers"][layer]
    Hq, Hkv, d = SHAPE.n_q_heads, SHAPE.n_kv_heads, SHAPE.head_dim
    rnd = lambda t: synth.round_to_storage(np.asarray(t, dtype=np.float32), "bf16").astype(np.float64)
    wd = {n: H.host(getattr(lw, n)) for n in ("g1", "w_qkv", "w_o", "g2", "w_gate_up", "w_down")}
    kc, vc = np.zeros((w.L, Hkv, d)), np.zeros((w.L, Hkv, d))
    kc[: w.L_ctx] = rnd(orc.rope_shift(r["k_cached"][layer], w.chunk_offsets, w.src_pos0, None, SHAPE.rope_base))
    vc[: w.L_ctx] = r["v_src"][layer]
    rng = np.random.default_rng(100 + layer)
    R = len(qi)
    rows = np.unique(np.concatenate([[0, R - 1], rng.choice(R, size=10, replace=False)]))
    h_in = H.host(r["capture"][layer]["h_in"])
    ho, k_new, v_new = orc.selective_prefill_layer(h_in, qi, kc, vc, wd, Hq, Hkv, d, SHAPE.rope_base, 1e-5, round_fn=rnd, rows=rows)
    idx = torch.from_numpy(qi).cuda()
    H.assert_close(H.host(r["k_cache"][layer][idx]), k_new, "bf16", f"layer {layer}: fresh K rows written back")
    H.assert_close(H.host(r["v_cache"][layer][idx]), v_new, "bf16", f"layer {layer}: fresh V rows written back")
    got = H.host(r["capture"][layer]["h_out"][torch.from_numpy(rows).cuda()])
    H.assert_close(got, ho, "bf16", f"layer {layer}: output rows")

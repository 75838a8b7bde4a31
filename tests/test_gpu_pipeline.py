"""The asynchronous host-to-device K/V load: overlapping the next request's copies with the current request's
layers must not change any result."""
import numpy as np
import pytest
import torch

from paper_2601_12904_amd import pipeline as P
from paper_2601_12904_amd import stack as S
from paper_2601_12904_amd import synth
from tests import harness as H

pytestmark = pytest.mark.gpu


def test_overlapped_load_equals_serial_load():
    w = synth.config_small_bf16(seed=4)
    Hq, Hkv, d = w.shape.n_q_heads, w.shape.n_kv_heads, w.shape.head_dim
    hidden, ffn, n_layers, n_req = 256, 512, 2, 5
    ctx = H.make_ctx(w.shape, w.L, w.n_chunks, w.nq)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(0)
    layers = [S.random_layer(hidden, ffn, Hq, Hkv, d, gen, std=0.05) for _ in range(n_layers)]
    st = S.SelectivePrefillStack(ctx, layers, hidden, ffn)
    rng = np.random.default_rng(0)
    k = int(0.15 * w.L_ctx + 0.5)
    qi = torch.from_numpy(np.concatenate([np.sort(rng.choice(w.L_ctx, size=k, replace=False)),
                                          w.L_ctx + np.arange(w.nq)]).astype(np.int32)).cuda()
    R = k + w.nq
    host = torch.Generator()
    host.manual_seed(1)
    def pinned():
        t = torch.empty((w.L_ctx, Hkv, d), dtype=torch.bfloat16, pin_memory=True)
        t.copy_((torch.randn((w.L_ctx, Hkv, d), generator=host) / np.sqrt(d)).to(torch.bfloat16))
        return t
    requests = [P.HostKVRequest([pinned() for _ in range(n_layers)], [pinned() for _ in range(n_layers)])
                for _ in range(n_req)]
    sets = [P.DeviceKVSet(n_layers, w.L_ctx, w.L, Hkv, d) for _ in range(2)]
    pipe = P.AsyncKVPipeline(sets)
    h0 = torch.randn((R, hidden), generator=gen, device="cuda").to(torch.bfloat16)
    results = {}

    def run(overlap):
        outs = {}
        def compute(i, kv):
            h = h0.clone()
            st.forward(h, qi, kv.k_cached, kv.k_cache, kv.v_cache, w.chunk_offsets, w.src_pos0, w.nq, w.L)
            outs[i] = (h, kv.k_cache[-1].clone(), kv.v_cache[-1].clone())
        pipe.run(requests, compute, overlap)
        torch.cuda.synchronize()
        return outs

    serial, overlapped = run(False), run(True)
    for i in range(n_req):
        for a, b in zip(serial[i], overlapped[i]):
            assert torch.equal(a, b), f"request {i}"
    assert not torch.equal(serial[0][0], serial[1][0])     # the requests really differ
    with pytest.raises(ValueError):
        P.HostKVRequest([torch.empty(4)], [torch.empty(4)])  # pageable host memory is refused
    ctx.close()


def test_overlapped_load_against_oracle():
    """Requests whose chunk K/V arrive from pinned host memory on the copy stream while the previous request computes
    (Sec. 4.2), each checked against the oracle: position shift of the loaded keys, then the decoder layers of the
    sparse prefill (eq. 9) chained over the loaded caches, following the pipeline store by store."""
    from oracle import fusionrag_oracle as orc
    shape = synth.LLAMA3_8B_BF16
    Hq, Hkv, d = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    hidden, ffn, n_layers, n_req = 256, 384, 2, 3
    w = synth.config_small_bf16(seed=9, chunk_lens=(130, 77, 200), nq=20)
    rng = np.random.default_rng(11)
    k = orc.topk_count(w.L_ctx, 0.15)
    qi = np.concatenate([np.sort(rng.choice(w.L_ctx, size=k, replace=False)), w.L_ctx + np.arange(w.nq)]).astype(np.int64)
    R = len(qi)
    ctx = H.make_ctx(shape, w.L, w.n_chunks, w.nq)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(2)
    layers = [S.random_layer(hidden, ffn, Hq, Hkv, d, gen, std=0.08) for _ in range(n_layers)]
    st = S.SelectivePrefillStack(ctx, layers, hidden, ffn)
    rnd = lambda t: synth.round_to_storage(np.asarray(t, dtype=np.float32), "bf16").astype(np.float64)
    host_k = [[rnd(rng.standard_normal((w.L_ctx, Hkv, d)) * 0.3) for _ in range(n_layers)] for _ in range(n_req)]
    host_v = [[rnd(rng.standard_normal((w.L_ctx, Hkv, d))) for _ in range(n_layers)] for _ in range(n_req)]

    def pinned(a):
        t = torch.empty(a.shape, dtype=torch.bfloat16, pin_memory=True)
        t.copy_(torch.from_numpy(a).to(torch.bfloat16))
        return t
    requests = [P.HostKVRequest([pinned(a) for a in host_k[i]], [pinned(a) for a in host_v[i]]) for i in range(n_req)]
    pipe = P.AsyncKVPipeline([P.DeviceKVSet(n_layers, w.L_ctx, w.L, Hkv, d) for _ in range(2)])
    h0 = rnd(rng.standard_normal((R, hidden)))
    qi_d = torch.from_numpy(qi.astype(np.int32)).cuda()
    got = {}

    def compute(i, kv):
        h = H.dev(h0, "bf16")
        st.forward(h, qi_d, kv.k_cached, kv.k_cache, kv.v_cache, w.chunk_offsets, w.src_pos0, w.nq, w.L)
        got[i] = (h, [t.clone() for t in kv.k_cache], [t.clone() for t in kv.v_cache])

    pipe.run(requests, compute, overlap=True)
    torch.cuda.synchronize()
    wd = [{n: H.host(getattr(lw, n)) for n in ("g1", "w_qkv", "w_o", "g2", "w_gate_up", "w_down")} for lw in layers]
    for i in range(n_req):
        ho = h0.copy()
        for l in range(n_layers):
            kc, vc = np.zeros((w.L, Hkv, d)), np.zeros((w.L, Hkv, d))
            kc[: w.L_ctx] = rnd(orc.rope_shift(host_k[i][l], w.chunk_offsets, w.src_pos0, None, shape.rope_base))
            vc[: w.L_ctx] = host_v[i][l]
            ho, k_new, v_new = orc.selective_prefill_layer(ho, qi, kc, vc, wd[l], Hq, Hkv, d, shape.rope_base, 1e-5, round_fn=rnd)
            want_k, want_v = orc.kv_scatter(qi, k_new, v_new, kc, vc)
            H.assert_close(H.host(got[i][1][l]), want_k, "bf16", f"request {i} layer {l} K cache")
            H.assert_close(H.host(got[i][2][l]), want_v, "bf16", f"request {i} layer {l} V cache")
        H.assert_close(H.host(got[i][0]), ho, "bf16", f"request {i} output rows")
    ctx.close()

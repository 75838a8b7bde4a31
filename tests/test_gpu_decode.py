"""GPU parity of the batch-decoding attention (shared chunk store + per-query exclusive pages, Sec. 4.3)
against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import fusionrag_oracle as orc
from paper_2601_12904_amd import binding as B
from paper_2601_12904_amd import synth
from tests import harness as H

pytestmark = pytest.mark.gpu

SHAPES = {
    "tiny_f32": synth.TINY_F32,
    "llama_bf16": synth.LLAMA3_8B_BF16,
    "bf16_d64_g2": synth.LayerShape(n_q_heads=4, n_kv_heads=2, head_dim=64, dtype="bf16", rope_base=10000.0),
    "f32_d128_g4": synth.LayerShape(n_q_heads=8, n_kv_heads=2, head_dim=128, dtype="f32", rope_base=500000.0),
    # the other group sizes of the matrix-core kernel (bf16, head_dim 128), and one it does not take
    "bf16_d128_g1": synth.LayerShape(n_q_heads=4, n_kv_heads=4, head_dim=128, dtype="bf16", rope_base=500000.0),
    "bf16_d128_g2": synth.LayerShape(n_q_heads=4, n_kv_heads=2, head_dim=128, dtype="bf16", rope_base=500000.0),
    "bf16_d128_g8": synth.LayerShape(n_q_heads=16, n_kv_heads=2, head_dim=128, dtype="bf16", rope_base=500000.0),
}


def make_batch(shape, seed, chunk_lens=(70, 130, 3, 257, 64), prompts=((0, 1, 3), (3, 1), (4, 2, 0, 1), ()),
               nq=(9, 17, 5, 3), n_gen=(1, 4, 2, 1), ratio=0.15, page_stride=None):
    """A chunk store cached at arbitrary positions and a batch of queries that use different chunk lists."""
    rng = np.random.default_rng(seed)
    Hq, Hkv, d, dt = shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.dtype
    rnd = lambda n, h, sig: synth.round_to_storage((rng.standard_normal((n, h, d)) * sig).astype(np.float32), dt)
    offs = np.concatenate([[0], np.cumsum(chunk_lens)]).astype(np.int64)
    N = int(offs[-1])
    src_pos0 = rng.integers(0, 3000, size=len(chunk_lens))
    k_store, v_store = rnd(N, Hkv, 1.0 / np.sqrt(d)), rnd(N, Hkv, 1.0 / np.sqrt(d))
    nb = len(prompts)
    q = rnd(nb, Hq, float(np.sqrt(d)))
    segments, stale, k_pages, v_pages = [], [], [], []
    for b, chunks in enumerate(prompts):
        pos, segs, rows = 0, [], []
        for c in chunks:
            n = int(offs[c + 1] - offs[c])
            segs.append((int(offs[c]), n, int(pos - src_pos0[c])))
            rows += list(range(int(offs[c]), int(offs[c + 1])))
            pos += n
        crit = np.sort(rng.choice(rows, size=int(ratio * len(rows) + 0.5), replace=False)) if rows else np.zeros(0, np.int64)
        P = len(crit) + nq[b] + n_gen[b]
        segments.append(segs)
        stale.append(crit)
        k_pages.append(rnd(P, Hkv, 1.0 / np.sqrt(d)))
        v_pages.append(rnd(P, Hkv, 1.0 / np.sqrt(d)))
    return dict(shape=shape, q=q, k_store=k_store, v_store=v_store, N=N, segments=segments, stale=stale, k_pages=k_pages,
                v_pages=v_pages, page_stride=page_stride or max(len(p) for p in k_pages) + 3)


def run_gpu(bt, use_mark=True, with_stale=True, generic=False):
    shape = bt["shape"]
    dt, tdt = shape.dtype, H.TORCH_DTYPE[shape.dtype]
    Hq, Hkv, d = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    nb = len(bt["segments"])
    ctx = H.make_ctx(shape, 1024, 4, 8)
    if generic:
        ctx.fr_set_option(B.FR_OPT_DECODE_KERNEL, B.FR_DECODE_KERNEL_GENERIC)
    seg_off = np.concatenate([[0], np.cumsum([len(s) for s in bt["segments"]])]).astype(np.int32)
    flat = [s for segs in bt["segments"] for s in segs]
    n_seg = len(flat)
    i32 = lambda a: torch.from_numpy(np.asarray(a, dtype=np.int32).reshape(-1)).cuda()
    row0, ln, dl = (i32([s[j] for s in flat]) if n_seg else None for j in range(3))
    words = (bt["N"] + 31) // 32
    bits = None
    if with_stale:
        bits = torch.full((nb, words), 0x5A5A5A5A, dtype=torch.int32, device="cuda")   # garbage: must be cleared
        for b in range(nb):
            if use_mark:
                rows = i32(bt["stale"][b]) if len(bt["stale"][b]) else None
                ctx.fr_mark_stale_rows(bits[b], words, rows, len(bt["stale"][b]), clear=True)
            else:
                w = np.zeros(words, dtype=np.uint32)
                for r in bt["stale"][b]:
                    w[r >> 5] |= np.uint32(1) << np.uint32(r & 31)
                bits[b] = torch.from_numpy(w.view(np.int32)).cuda()
    ps = bt["page_stride"]
    kp = torch.zeros((nb, ps, Hkv, d), dtype=tdt, device="cuda")
    vp = torch.zeros((nb, ps, Hkv, d), dtype=tdt, device="cuda")
    for b in range(nb):
        P = len(bt["k_pages"][b])
        kp[b, :P] = H.dev(bt["k_pages"][b], dt)
        vp[b, :P] = H.dev(bt["v_pages"][b], dt)
        kp[b, P:] = 1000.0          # rows past page_len must not be read
    plen = i32([len(p) for p in bt["k_pages"]])
    out = torch.zeros((nb, Hq, d), dtype=tdt, device="cuda")
    lse = torch.zeros((nb, Hq), dtype=torch.float32, device="cuda")
    ctx.fr_decode_attn(H.dev(bt["q"], dt), nb, H.dev(bt["k_store"], dt), H.dev(bt["v_store"], dt), bt["N"], i32(seg_off),
                       row0, ln, dl, n_seg, bits, words if with_stale else 0, kp, vp, ps, plen, out, lse)
    torch.cuda.synchronize()
    res = H.host(out), lse.cpu().numpy().astype(np.float64), (bits.cpu().numpy().view(np.uint32) if with_stale else None)
    ctx.close()
    return res


@pytest.mark.parametrize("name", list(SHAPES))
@pytest.mark.parametrize("seed", [0, 1])
def test_decode_attn_parity(name, seed):
    shape = SHAPES[name]
    bt = make_batch(shape, seed)
    got, lse, bits = run_gpu(bt)
    want, want_lse = orc.decode_attn(bt["q"], bt["k_store"], bt["v_store"], bt["segments"], bt["stale"], bt["k_pages"],
                                     bt["v_pages"], shape.rope_base)
    H.assert_close(got, want, shape.dtype, "decode attention")
    assert np.max(np.abs(lse - want_lse)) <= (1e-4 if shape.dtype == "f32" else 2e-3)
    # the masks fr_mark_stale_rows built are exactly the listed rows
    for b, rows in enumerate(bt["stale"]):
        w = np.zeros(bits.shape[1], dtype=np.uint32)
        for r in rows:
            w[r >> 5] |= np.uint32(1) << np.uint32(r & 31)
        assert np.array_equal(bits[b], w)


def test_decode_attn_without_mask_and_host_built_mask():
    shape = SHAPES["llama_bf16"]
    bt = make_batch(shape, 5)
    got, _, _ = run_gpu(bt, use_mark=False)
    want, _ = orc.decode_attn(bt["q"], bt["k_store"], bt["v_store"], bt["segments"], bt["stale"], bt["k_pages"],
                              bt["v_pages"], shape.rope_base)
    H.assert_close(got, want, "bf16", "decode attention, mask built on the host")
    got2, _, _ = run_gpu(bt, with_stale=False)
    want2, _ = orc.decode_attn(bt["q"], bt["k_store"], bt["v_store"], bt["segments"], [[] for _ in bt["stale"]],
                               bt["k_pages"], bt["v_pages"], shape.rope_base)
    H.assert_close(got2, want2, "bf16", "decode attention, nothing stale")


def test_decode_attn_descriptor_ranges_are_clamped():
    """Segments that reach outside the store and a page_len beyond the page: rows outside are not read and do not count."""
    shape = SHAPES["llama_bf16"]
    bt = make_batch(shape, 6, prompts=((0, 1),), nq=(4,), n_gen=(1,))
    N = bt["N"]
    good = list(bt["segments"][0])
    bt_bad = dict(bt)
    bt_bad["segments"] = [good + [(N - 10, 50, 7), (-5, 9, 3)]]     # 10 rows inside, 4 rows inside
    got, _, _ = run_gpu(bt_bad)
    bt_ref = dict(bt)
    bt_ref["segments"] = [good + [(N - 10, 10, 7), (0, 4, 3)]]
    want, _ = orc.decode_attn(bt["q"], bt["k_store"], bt["v_store"], bt_ref["segments"], bt["stale"], bt["k_pages"],
                              bt["v_pages"], shape.rope_base)
    H.assert_close(got, want, "bf16", "clamped segments")


@pytest.mark.parametrize("seed", [2, 3])
def test_decode_attn_both_kernels(seed):
    """bf16, head_dim 128: the matrix-core kernel (default) and the generic one (forced) against the oracle, on a
    batch with long ragged segments (several 32-row blocks per wave, ragged tails, unaligned mask words)."""
    shape = SHAPES["llama_bf16"]
    bt = make_batch(shape, seed, chunk_lens=(333, 1, 1025, 31, 640), prompts=((2, 0, 4), (1, 3), (4, 2, 1, 0, 3)),
                    nq=(40, 3, 11), n_gen=(2, 1, 5))
    want, want_lse = orc.decode_attn(bt["q"], bt["k_store"], bt["v_store"], bt["segments"], bt["stale"], bt["k_pages"],
                                     bt["v_pages"], shape.rope_base)
    for generic in (False, True):
        got, lse, _ = run_gpu(bt, generic=generic)
        H.assert_close(got, want, "bf16", f"decode attention (generic={generic})")
        assert np.max(np.abs(lse - want_lse)) <= 2e-3


def test_decode_attn_full_size_sampled():
    """The launch configuration `bench.py --config 7` times on its shared store: 32 queries, each over 16 of 64 cached
    1024-token chunks with 15 % of their rows stale, plus an exclusive page of 2978 rows.  Three of the queries against
    the oracle."""
    rng = np.random.default_rng(5)
    nb = 32
    prompts = tuple(tuple(int(c) for c in rng.choice(64, size=16, replace=False)) for _ in range(nb))
    bt = make_batch(SHAPES["llama_bf16"], 21, chunk_lens=(1024,) * 64, prompts=prompts, nq=(512,) * nb, n_gen=(8,) * nb)
    got, got_lse, _ = run_gpu(bt)
    for b in (0, 13, 31):
        want, want_lse = orc.decode_attn(bt["q"][[b]], bt["k_store"], bt["v_store"], [bt["segments"][b]], [bt["stale"][b]],
                                         [bt["k_pages"][b]], [bt["v_pages"][b]], bt["shape"].rope_base)
        H.assert_close(got[[b]], want, "bf16", f"decode output of query {b}")
        assert np.max(np.abs(got_lse[[b]] - want_lse)) <= 2e-3

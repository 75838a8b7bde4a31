"""Host-side checks of the C-ABI library: it loads, exports every declared symbol, and rejects bad
arguments before touching a device.  No kernel runs here."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import fusionrag_oracle as orc
from paper_2601_12904_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_exports_match_header():
    lib = B.load()
    header = open(os.path.join(ROOT, "include", "fusionrag.h")).read()
    declared = set(re.findall(r"\b(fr_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared but not exported"


def test_topk_count_matches_oracle():
    for L in (0, 1, 10, 512, 16384, 32768, 12345):
        for ratio in (0.0, 0.05, 0.10, 0.15, 0.25, 0.30, 0.5, 1.0, 1.5):
            assert B.fr_topk_count(L, ratio) == orc.topk_count(L, ratio)


def test_create_rejects_bad_descriptions():
    lib = B.load()
    def create(**kw):
        d = dict(n_q_heads=32, n_kv_heads=8, head_dim=128, dtype=B.FR_BF16, rope_base=5e5, rope_layout=0,
                 rope_index_base=0)
        d.update(kw)
        desc = B.fr_layer_desc(**d)
        h = ctypes.c_void_p()
        st = lib.fr_create(ctypes.byref(desc), 1024, 4, 16, ctypes.byref(h))
        if st == B.FR_OK:
            lib.fr_destroy(h)
        else:
            assert not h.value
        return st
    assert create() == B.FR_OK
    assert create(n_kv_heads=5) == B.FR_ERR_INVALID_ARG
    assert create(n_q_heads=0) == B.FR_ERR_INVALID_ARG
    assert create(dtype=7) == B.FR_ERR_INVALID_ARG
    assert create(rope_base=0.5) == B.FR_ERR_INVALID_ARG
    assert create(rope_layout=3) == B.FR_ERR_INVALID_ARG
    assert create(head_dim=96) == B.FR_ERR_UNSUPPORTED
    desc = B.fr_layer_desc(4, 4, 64, B.FR_F32, 1e4, 0, 0)
    h = ctypes.c_void_p()
    assert lib.fr_create(ctypes.byref(desc), 1024, B.FR_MAX_CHUNKS + 1, 16, ctypes.byref(h)) == B.FR_ERR_UNSUPPORTED
    assert lib.fr_create(ctypes.byref(desc), 0, 4, 0, ctypes.byref(h)) == B.FR_ERR_INVALID_ARG
    assert lib.fr_create(None, 1024, 4, 16, ctypes.byref(h)) == B.FR_ERR_INVALID_ARG


@pytest.fixture()
def ctx():
    c = B.Context(4, 4, 64, B.FR_F32, 1e4, max_tokens=600, max_chunks=4, max_question_tokens=32)
    yield c
    c.close()


def expect(status, fn, *a, **kw):
    with pytest.raises(B.FusionRAGError) as ei:
        fn(*a, **kw)
    assert ei.value.status == status, str(ei.value)


def test_rope_shift_argument_errors(ctx):
    P = 4096  # a fake, aligned, non-null device address: validation must fail before any launch
    expect(B.FR_ERR_INVALID_ARG, ctx.fr_rope_shift, P, P, [1, 5], [0])
    expect(B.FR_ERR_INVALID_ARG, ctx.fr_rope_shift, P, P, [0, 9, 5], [0, 0])
    expect(B.FR_ERR_WORKSPACE, ctx.fr_rope_shift, P, P, [0, 1, 2, 3, 4, 5], [0] * 5)
    expect(B.FR_ERR_WORKSPACE, ctx.fr_rope_shift, P, P, [0, 601], [0])
    expect(B.FR_ERR_INVALID_ARG, ctx.fr_rope_shift, P + 4, P, [0, 5], [0])
    expect(B.FR_ERR_INVALID_ARG, ctx.fr_rope_shift, None, P, [0, 5], [0])
    expect(B.FR_ERR_INVALID_ARG, ctx.fr_rope_shift, P, P + 256, [0, 5], [0])          # partial overlap
    expect(B.FR_ERR_INVALID_ARG, ctx.fr_rope_shift, P, P, [0, 5], [0], n_batch=2, src_batch_stride=8)
    ctx.fr_rope_shift(None, None, [0, 0], [0])                                         # nothing to do: OK


def test_score_select_argument_errors(ctx):
    P = 4096
    expect(B.FR_ERR_INVALID_ARG, ctx.fr_score_select, P, 4, P, [0, 10], 11, q_index_out=P)
    expect(B.FR_ERR_INVALID_ARG, ctx.fr_score_select, P, 4, P, [0, 10], -1, q_index_out=P)
    expect(B.FR_ERR_INVALID_ARG, ctx.fr_score_select, P, 4, P, [0, 10], 2, norm=9, q_index_out=P)
    expect(B.FR_ERR_INVALID_ARG, ctx.fr_score_select, P, 4, P, [0, 10], 2, q_index_out=None)
    expect(B.FR_ERR_WORKSPACE, ctx.fr_score_select, P, 33, P, [0, 10], 2, q_index_out=P)
    expect(B.FR_ERR_WORKSPACE, ctx.fr_score_select, P, 32, P, [0, 590], 2, q_index_out=P)   # L_ctx + nq > max_tokens
    expect(B.FR_ERR_INVALID_ARG, ctx.fr_score_select, P + 2, 4, P, [0, 10], 2, q_index_out=P)
    expect(B.FR_ERR_INVALID_ARG, ctx.fr_select_topk, P, 10, 11, 0, P)


def test_kv_deviation_argument_errors(ctx):
    P = 4096
    expect(B.FR_ERR_INVALID_ARG, ctx.fr_kv_deviation, P, P, -1, P)
    expect(B.FR_ERR_INVALID_ARG, ctx.fr_kv_deviation, None, P, 5, P)
    expect(B.FR_ERR_INVALID_ARG, ctx.fr_kv_deviation, P, P + 8, 5, P)
    expect(B.FR_ERR_INVALID_ARG, ctx.fr_kv_deviation, P, P, 5, None)
    ctx.fr_kv_deviation(None, None, 0, None)                                                  # nothing to do


def test_decode_argument_errors(ctx):
    P = 4096
    ok = (P, 2, P, P, 100, P, P, P, P, 3, P, 4, P, P, 64, P, P)
    def call(**kw):
        names = ("q", "n_queries", "k_shared", "v_shared", "n_shared_rows", "seg_offsets", "seg_row0", "seg_len", "seg_delta",
                 "n_segments", "stale_bits", "stale_words", "k_pages", "v_pages", "page_stride_rows", "page_len", "out")
        a = dict(zip(names, ok))
        a.update(kw)
        return lambda: ctx.fr_decode_attn(*[a[n] for n in names])
    expect(B.FR_ERR_INVALID_ARG, call(n_queries=-1))
    expect(B.FR_ERR_INVALID_ARG, call(q=None))
    expect(B.FR_ERR_INVALID_ARG, call(k_pages=P + 4))
    expect(B.FR_ERR_INVALID_ARG, call(seg_row0=None))
    expect(B.FR_ERR_INVALID_ARG, call(k_shared=None))
    expect(B.FR_ERR_INVALID_ARG, call(page_len=None))
    expect(B.FR_ERR_WORKSPACE, call(n_segments=4095))
    call(n_queries=0, q=None)()                                                               # nothing to do
    expect(B.FR_ERR_INVALID_ARG, ctx.fr_mark_stale_rows, None, 4, P, 3)
    expect(B.FR_ERR_INVALID_ARG, ctx.fr_mark_stale_rows, P, 4, None, 3)
    ctx.fr_mark_stale_rows(P, 0, P, 3)                                                        # no words: nothing to do
    expect(B.FR_ERR_INVALID_ARG, ctx.fr_set_option, B.FR_OPT_DECODE_KERNEL, 5)


def test_attention_and_scatter_argument_errors(ctx):
    P = 4096
    expect(B.FR_ERR_INVALID_ARG, ctx.fr_sparse_prefill_attn, P, P, 5, P, P, 4, P, P, P)      # R > L
    expect(B.FR_ERR_WORKSPACE, ctx.fr_sparse_prefill_attn, P, P, 5, P, P, 601, P, P, P)
    expect(B.FR_ERR_INVALID_ARG, ctx.fr_sparse_prefill_attn, P, P, 5, P, P, 100, P, None, P)  # only one of k_new/v_new
    expect(B.FR_ERR_INVALID_ARG, ctx.fr_sparse_prefill_attn, P, None, 5, P, P, 100, P, P, P)
    expect(B.FR_ERR_INVALID_ARG, ctx.fr_sparse_prefill_attn, P, P, 5, P + 8, P, 100, P, P, P)
    expect(B.FR_ERR_INVALID_ARG, ctx.fr_sparse_prefill_attn, P, P, -1, P, P, 100, P, P, P)
    expect(B.FR_ERR_INVALID_ARG, ctx.fr_kv_scatter, P, P, P, 5, P, P, 4)
    expect(B.FR_ERR_INVALID_ARG, ctx.fr_kv_scatter, None, P, P, 5, P, P, 100)
    ctx.fr_kv_scatter(None, None, None, 0, None, None, 100)                                   # R = 0: nothing to do
    ctx.fr_sparse_prefill_attn(None, None, 0, None, None, 100, None, None, None)


def test_valid_call_without_gpu_reports_device_error(ctx):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    P = 4096
    expect(B.FR_ERR_DEVICE, ctx.fr_rope_shift, P, P, [0, 5], [0])
    expect(B.FR_ERR_DEVICE, ctx.fr_kv_scatter, P, P, P, 5, P, P, 100)
    expect(B.FR_ERR_DEVICE, ctx.fr_kv_deviation, P, P, 5, P)
    expect(B.FR_ERR_DEVICE, ctx.fr_decode_attn, P, 2, P, P, 100, P, P, P, P, 3, P, 4, P, P, 64, P, P)
    expect(B.FR_ERR_DEVICE, ctx.fr_mark_stale_rows, P, 4, P, 3)
    assert ctx.workspace_bytes() == 0


def test_shared_batch_argument_errors():
    """fr_sparse_prefill_attn_shared_batch validates every query on the host before the first launch."""
    import torch
    c = B.Context(32, 8, 128, B.FR_BF16, 5e5, max_tokens=600, max_chunks=4, max_question_tokens=32)
    P = 4096
    q = dict(q_rows=P, q_index=P, R=5, chunk_offsets=[0, 8, 16], chunk_store_row0=[0, 8], chunk_src_pos0=[0, 0], L=20,
             k_new=P, v_new=P, out=P)
    need = c.fr_shared_batch_workspace_bytes(2, 20)
    assert need > 0 and need % 256 == 0
    assert c.fr_shared_batch_workspace_bytes(0, 20) == 0
    assert c.fr_shared_batch_workspace_bytes(40, 20) == 8 * need      # groups of 16 reuse the workspace
    c.fr_sparse_prefill_attn_shared_batch([], P, P, 100, None, 0)     # no queries: nothing to do
    expect(B.FR_ERR_WORKSPACE, c.fr_sparse_prefill_attn_shared_batch, [q, q], P, P, 100, P, 512)
    expect(B.FR_ERR_INVALID_ARG, c.fr_sparse_prefill_attn_shared_batch, [q], P, P, 100, P + 16, need)   # workspace alignment
    bad = dict(q, chunk_store_row0=[0, 96])                            # second chunk reaches past the store
    with pytest.raises(B.FusionRAGError) as ei:
        c.fr_sparse_prefill_attn_shared_batch([q, bad], P, P, 100, P, need)
    assert ei.value.status == B.FR_ERR_INVALID_ARG and "query 1" in str(ei.value)
    expect(B.FR_ERR_WORKSPACE, c.fr_sparse_prefill_attn_shared_batch, [dict(q, L=601)], P, P, 100, P, need)
    expect(B.FR_ERR_INVALID_ARG, c.fr_sparse_prefill_attn_shared_batch, [dict(q, k_new=None)], P, P, 100, P, need)
    empty = dict(q, R=0)
    c.fr_sparse_prefill_attn_shared_batch([empty, empty], P, P, 100, None, 0)   # no rows anywhere: nothing to do
    if not torch.cuda.is_available():
        expect(B.FR_ERR_DEVICE, c.fr_sparse_prefill_attn_shared_batch, [q, q], P, P, 100, P, need)
    c.close()


def test_shared_score_select_argument_errors():
    import torch
    c = B.Context(32, 8, 128, B.FR_BF16, 5e5, max_tokens=600, max_chunks=4, max_question_tokens=32)
    P = 4096
    call = lambda **kw: c.fr_score_select_shared(**{**dict(q_question=P, nq=4, k_store=P, n_store_rows=100, chunk_offsets=[0, 8, 16],
                                                        chunk_store_row0=[0, 8], chunk_src_pos0=[0, 0], k=3, norm=B.FR_NORM_PER_CHUNK,
                                                        scores_out=None, q_index_out=P), **kw})
    expect(B.FR_ERR_INVALID_ARG, call, chunk_store_row0=[0, 96])          # past the end of the store
    expect(B.FR_ERR_INVALID_ARG, call, norm=B.FR_NORM_RAW)                # softmax scopes only
    expect(B.FR_ERR_INVALID_ARG, call, k=17)                              # more than there are context tokens
    expect(B.FR_ERR_INVALID_ARG, call, q_index_out=None)
    expect(B.FR_ERR_INVALID_ARG, call, k_store=P + 4)                     # alignment
    expect(B.FR_ERR_WORKSPACE, call, nq=33)
    if not torch.cuda.is_available():
        expect(B.FR_ERR_DEVICE, call)
    c.close()
    # fp32 / head_dim 64 contexts take the same arguments (served by the generic kernels) and the same checks
    c32 = B.Context(4, 4, 64, B.FR_F32, 1e4, max_tokens=600, max_chunks=4, max_question_tokens=32)
    call32 = lambda **kw: c32.fr_score_select_shared(**{**dict(q_question=P, nq=4, k_store=P, n_store_rows=100,
                                                              chunk_offsets=[0, 8, 16], chunk_store_row0=[0, 8],
                                                              chunk_src_pos0=[0, 0], k=3, norm=B.FR_NORM_PER_CHUNK,
                                                              scores_out=None, q_index_out=P), **kw})
    expect(B.FR_ERR_INVALID_ARG, call32, chunk_store_row0=[0, 96])
    assert c32.fr_shared_batch_workspace_bytes(2, 20) == 0
    if not torch.cuda.is_available():
        expect(B.FR_ERR_DEVICE, call32)
    c32.close()


def test_bench_work_counts():
    """The two pair counts bench.py prices the attention kernel with: the pairs the method needs (sum of pos + 1) and
    the pairs the tiled kernel walks (whole 64-key tiles up to a row tile's last position, last row tile padded)."""
    import bench
    qi = np.array([0, 5, 63, 64, 200])
    assert bench.attention_pairs(qi) == 1 + 6 + 64 + 65 + 201
    # group size 4: 64 rows per tile -> one tile, padded to 64 rows, walking keys 0 .. 255 (four key tiles)
    assert bench.attention_executed_pairs(qi, 4) == 64 * 256
    # group size 8: 32 rows per tile; 40 rows -> two tiles, the first ends at position 31 (one key tile), the second at 39
    qi = np.arange(40)
    assert bench.attention_executed_pairs(qi, 8) == 32 * 64 + 32 * 64
    # a full causal block of aligned size: the overhead is what the mask removes inside the diagonal tiles
    qi = np.arange(256)
    assert bench.attention_executed_pairs(qi, 4) == sum(64 * 64 * (t + 1) for t in range(4))
    assert bench.attention_executed_pairs(qi, 4) >= bench.attention_pairs(qi)

"""ctypes binding of libfusionrag.so: the same entry points as include/fusionrag.h, argument
marshalling only.  PyTorch supplies device memory and streams; every step of the path runs in the
library's own HIP kernels.  There is no fallback: if the library is missing, loading raises."""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np
import torch  # first: the library must bind to the HIP runtime PyTorch has loaded

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libfusionrag.so")

FR_OK, FR_ERR_INVALID_ARG, FR_ERR_UNSUPPORTED, FR_ERR_WORKSPACE, FR_ERR_DEVICE = range(5)
FR_F32, FR_BF16 = 0, 1
FR_ROPE_INTERLEAVED, FR_ROPE_HALF = 0, 1
FR_NORM_PER_CHUNK, FR_NORM_GLOBAL, FR_NORM_RAW = 0, 1, 2
FR_MAX_CHUNKS = 256
FR_SELECT_STATIC_MAX_SCORES = 1 << 24
STATUS_NAMES = {0: "FR_OK", 1: "FR_ERR_INVALID_ARG", 2: "FR_ERR_UNSUPPORTED", 3: "FR_ERR_WORKSPACE",
                4: "FR_ERR_DEVICE"}
FR_OPT_ATTN_SOFTMAX = 1
FR_OPT_ATTN_SPLIT = 2
FR_OPT_DECODE_KERNEL = 3
FR_OPT_GEMM_TILE = 4
FR_OPT_GEMM_TAIL_SPLIT = 6
FR_OPT_ATTN_KERNEL_TIMER = 5
FR_DECODE_KERNEL_AUTO, FR_DECODE_KERNEL_GENERIC = 0, 1
FR_ATTN_SOFTMAX_AUTO, FR_ATTN_SOFTMAX_RUNNING_MAX = 0, 1
FR_ATTN_SPLIT_AUTO, FR_ATTN_SPLIT_OFF, FR_ATTN_SPLIT_ON = 0, 1, 2
EXPORTS = ("fr_create", "fr_destroy", "fr_last_error", "fr_workspace_bytes", "fr_set_option", "fr_attn_kernel_times", "fr_topk_count", "fr_rope_shift",
           "fr_score_select", "fr_score_select_shared", "fr_select_topk", "fr_select_topk_static", "fr_kv_deviation", "fr_sparse_prefill_attn", "fr_sparse_prefill_attn_writeback", "fr_sparse_prefill_attn_shared", "fr_shared_batch_workspace_bytes", "fr_sparse_prefill_attn_shared_batch", "fr_decode_attn", "fr_mark_stale_rows", "fr_kv_scatter", "fr_rmsnorm", "fr_linear",
           "fr_linear_swiglu", "fr_qkv_rope")


class fr_layer_desc(ctypes.Structure):
    _fields_ = [("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("rope_base", ctypes.c_double), ("rope_layout", ctypes.c_int32),
                ("rope_index_base", ctypes.c_int32)]


class fr_shared_query(ctypes.Structure):
    _fields_ = [("q_rows", ctypes.c_void_p), ("q_index", ctypes.c_void_p), ("R", ctypes.c_int32),
                ("chunk_offsets", ctypes.POINTER(ctypes.c_int32)), ("chunk_store_row0", ctypes.POINTER(ctypes.c_int32)),
                ("chunk_src_pos0", ctypes.POINTER(ctypes.c_int32)), ("n_chunks", ctypes.c_int32), ("L", ctypes.c_int64),
                ("k_new", ctypes.c_void_p), ("v_new", ctypes.c_void_p), ("out", ctypes.c_void_p),
                ("lse_out", ctypes.c_void_p)]


class FusionRAGError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


_lib = None


def load() -> ctypes.CDLL:
    """Load libfusionrag.so (built in-tree by `python -m paper_2601_12904_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2601_12904_amd.build` "
                          "(there is no fallback path)")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64, f64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_double
    pi32 = ctypes.POINTER(ctypes.c_int32)
    lib.fr_create.argtypes = [ctypes.POINTER(fr_layer_desc), i64, i32, i32, ctypes.POINTER(vp)]
    lib.fr_create.restype = i32
    lib.fr_destroy.argtypes = [vp]
    lib.fr_destroy.restype = None
    lib.fr_last_error.argtypes = [vp]
    lib.fr_last_error.restype = ctypes.c_char_p
    lib.fr_workspace_bytes.argtypes = [vp]
    lib.fr_workspace_bytes.restype = i64
    lib.fr_set_option.argtypes = [vp, i32, i64]
    lib.fr_set_option.restype = i32
    lib.fr_attn_kernel_times.argtypes = [vp, ctypes.POINTER(ctypes.c_float), i32, ctypes.POINTER(i32)]
    lib.fr_attn_kernel_times.restype = i32
    lib.fr_topk_count.argtypes = [i64, f64]
    lib.fr_topk_count.restype = i64
    lib.fr_rope_shift.argtypes = [vp, vp, vp, pi32, pi32, pi32, i32, i32, i32, i64, i64, vp]
    lib.fr_rope_shift.restype = i32
    lib.fr_score_select.argtypes = [vp, vp, i32, vp, pi32, i32, i64, i32, vp, vp, vp]
    lib.fr_score_select.restype = i32
    lib.fr_score_select_shared.argtypes = [vp, vp, i32, vp, i64, pi32, pi32, pi32, i32, i64, i32, vp, vp, vp]
    lib.fr_score_select_shared.restype = i32
    lib.fr_select_topk.argtypes = [vp, vp, i64, i64, i32, vp, vp]
    lib.fr_select_topk.restype = i32
    lib.fr_select_topk_static.argtypes = [vp, vp, i64, i64, i32, vp, vp]
    lib.fr_select_topk_static.restype = i32
    lib.fr_kv_deviation.argtypes = [vp, vp, vp, i64, vp, vp]
    lib.fr_kv_deviation.restype = i32
    lib.fr_sparse_prefill_attn.argtypes = [vp, vp, vp, i32, vp, vp, i64, vp, vp, vp, vp, vp]
    lib.fr_sparse_prefill_attn.restype = i32
    lib.fr_sparse_prefill_attn_writeback.argtypes = [vp, vp, vp, i32, vp, vp, i64, vp, vp, vp, vp, vp]
    lib.fr_sparse_prefill_attn_writeback.restype = i32
    lib.fr_sparse_prefill_attn_shared.argtypes = [vp, vp, vp, i32, vp, vp, i64, pi32, pi32, pi32, i32, i64, vp, vp, vp, vp, vp]
    lib.fr_sparse_prefill_attn_shared.restype = i32
    lib.fr_shared_batch_workspace_bytes.argtypes = [vp, i32, i64]
    lib.fr_shared_batch_workspace_bytes.restype = i64
    lib.fr_sparse_prefill_attn_shared_batch.argtypes = [vp, ctypes.POINTER(fr_shared_query), i32, vp, vp, i64, vp, i64, vp]
    lib.fr_sparse_prefill_attn_shared_batch.restype = i32
    lib.fr_decode_attn.argtypes = [vp, vp, i32, vp, vp, i64, vp, vp, vp, vp, i32, vp, i64, vp, vp, i64, vp, vp, vp, vp]
    lib.fr_decode_attn.restype = i32
    lib.fr_mark_stale_rows.argtypes = [vp, vp, i64, vp, i32, i32, vp]
    lib.fr_mark_stale_rows.restype = i32
    lib.fr_kv_scatter.argtypes = [vp, vp, vp, vp, i32, vp, vp, i64, vp]
    lib.fr_kv_scatter.restype = i32
    lib.fr_rmsnorm.argtypes = [vp, vp, vp, i32, i32, ctypes.c_float, vp, vp]
    lib.fr_rmsnorm.restype = i32
    lib.fr_linear.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp, vp]
    lib.fr_linear.restype = i32
    lib.fr_linear_swiglu.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp]
    lib.fr_linear_swiglu.restype = i32
    lib.fr_qkv_rope.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp, vp, vp]
    lib.fr_qkv_rope.restype = i32
    _lib = lib
    return lib


def _ptr(t) -> Optional[int]:
    """Device address of a tensor (or a raw integer address, or None)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("tensors handed to the library must be contiguous")
    return t.data_ptr()


def _i32_array(values: Optional[Sequence[int]]):
    if values is None:
        return None
    a = np.ascontiguousarray(np.asarray(values), dtype=np.int32)
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), a   # keep `a` alive during the call


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream() if torch.cuda.is_available() else None
    if stream is None:
        return None
    return stream if isinstance(stream, int) else stream.cuda_stream


def fr_topk_count(L_ctx: int, ratio: float) -> int:
    return int(load().fr_topk_count(int(L_ctx), float(ratio)))


def fr_select_topk_static(scores, n: int, k: int, nq: int, q_index_out, stream=None, ctx: "Context" = None):
    """fr_select_topk without a context and without any allocation (the library's static scratch); `ctx`, if given,
    only receives the error message."""
    lib = load()
    st = lib.fr_select_topk_static(ctx._h if ctx is not None else None, _ptr(scores), int(n), int(k), int(nq),
                                   _ptr(q_index_out), _stream(stream))
    if st != FR_OK:
        raise FusionRAGError(st, lib.fr_last_error(ctx._h).decode() if ctx is not None else "fr_select_topk_static failed")


class Context:
    """Owns one fr_ctx.  Methods are named after the C entry points and only marshal arguments."""

    def __init__(self, n_q_heads: int, n_kv_heads: int, head_dim: int, dtype: int, rope_base: float,
                 max_tokens: int, max_chunks: int, max_question_tokens: int,
                 rope_layout: int = FR_ROPE_INTERLEAVED, rope_index_base: int = 0):
        self._lib = load()
        self.desc = fr_layer_desc(n_q_heads, n_kv_heads, head_dim, dtype, rope_base, rope_layout, rope_index_base)
        h = ctypes.c_void_p()
        st = self._lib.fr_create(ctypes.byref(self.desc), int(max_tokens), int(max_chunks), int(max_question_tokens),
                                 ctypes.byref(h))
        if st != FR_OK:
            raise FusionRAGError(st, "fr_create rejected the layer description or could not allocate")
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            self._lib.fr_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int):
        if st != FR_OK:
            raise FusionRAGError(st, self._lib.fr_last_error(self._h).decode())

    def workspace_bytes(self) -> int:
        return int(self._lib.fr_workspace_bytes(self._h))

    def fr_attn_kernel_times(self, capacity: int = 256):
        buf = (ctypes.c_float * capacity)()
        n = ctypes.c_int32(0)
        self._check(self._lib.fr_attn_kernel_times(self._h, buf, int(capacity), ctypes.byref(n)))
        return [float(buf[i]) for i in range(n.value)]

    def fr_set_option(self, option: int, value: int):
        self._check(self._lib.fr_set_option(self._h, int(option), int(value)))

    def fr_rope_shift(self, k_src, k_dst, chunk_offsets, chunk_src_pos0, chunk_dst_pos0=None, dst_base: int = 0,
                      n_batch: int = 1, src_batch_stride: int = 0, dst_batch_stride: int = 0, stream=None):
        offs, _a = _i32_array(chunk_offsets)
        src, _b = _i32_array(chunk_src_pos0)
        dst = _i32_array(chunk_dst_pos0)
        self._check(self._lib.fr_rope_shift(self._h, _ptr(k_src), _ptr(k_dst), offs, src, dst[0] if dst else None,
                                            int(dst_base), len(_a) - 1, int(n_batch), int(src_batch_stride),
                                            int(dst_batch_stride), _stream(stream)))

    def fr_score_select(self, q_question, nq: int, k_ctx, chunk_offsets, k: int, norm: int = FR_NORM_PER_CHUNK,
                        scores_out=None, q_index_out=None, stream=None):
        offs, _a = _i32_array(chunk_offsets)
        self._check(self._lib.fr_score_select(self._h, _ptr(q_question), int(nq), _ptr(k_ctx), offs, len(_a) - 1,
                                              int(k), int(norm), _ptr(scores_out), _ptr(q_index_out),
                                              _stream(stream)))

    def fr_score_select_shared(self, q_question, nq: int, k_store, n_store_rows: int, chunk_offsets, chunk_store_row0,
                               chunk_src_pos0, k: int, norm: int = FR_NORM_PER_CHUNK, scores_out=None, q_index_out=None,
                               stream=None):
        offs, _a = _i32_array(chunk_offsets)
        row0, _b = _i32_array(chunk_store_row0)
        src, _c = _i32_array(chunk_src_pos0)
        self._check(self._lib.fr_score_select_shared(self._h, _ptr(q_question), int(nq), _ptr(k_store), int(n_store_rows),
                                                     offs, row0, src, len(_a) - 1, int(k), int(norm), _ptr(scores_out),
                                                     _ptr(q_index_out), _stream(stream)))

    def fr_select_topk(self, scores, n: int, k: int, nq: int, q_index_out, stream=None):
        self._check(self._lib.fr_select_topk(self._h, _ptr(scores), int(n), int(k), int(nq), _ptr(q_index_out),
                                             _stream(stream)))

    def fr_kv_deviation(self, kv_a, kv_b, n_tokens: int, deviation_out, stream=None):
        self._check(self._lib.fr_kv_deviation(self._h, _ptr(kv_a), _ptr(kv_b), int(n_tokens), _ptr(deviation_out),
                                              _stream(stream)))

    def fr_sparse_prefill_attn(self, q_rows, q_index, R: int, k_cache, v_cache, L: int, k_new, v_new, out,
                               lse_out=None, stream=None):
        self._check(self._lib.fr_sparse_prefill_attn(self._h, _ptr(q_rows), _ptr(q_index), int(R), _ptr(k_cache),
                                                     _ptr(v_cache), int(L), _ptr(k_new), _ptr(v_new), _ptr(out),
                                                     _ptr(lse_out), _stream(stream)))

    def fr_sparse_prefill_attn_writeback(self, q_rows, q_index, R: int, k_cache, v_cache, L: int, k_new, v_new, out,
                                         lse_out=None, stream=None):
        self._check(self._lib.fr_sparse_prefill_attn_writeback(self._h, _ptr(q_rows), _ptr(q_index), int(R),
                                                               _ptr(k_cache), _ptr(v_cache), int(L), _ptr(k_new),
                                                               _ptr(v_new), _ptr(out), _ptr(lse_out), _stream(stream)))

    def fr_sparse_prefill_attn_shared(self, q_rows, q_index, R: int, k_store, v_store, n_store_rows: int, chunk_offsets,
                                      chunk_store_row0, chunk_src_pos0, L: int, k_new, v_new, out, lse_out=None,
                                      stream=None):
        offs, _a = _i32_array(chunk_offsets)
        row0, _b = _i32_array(chunk_store_row0)
        src, _c = _i32_array(chunk_src_pos0)
        self._check(self._lib.fr_sparse_prefill_attn_shared(self._h, _ptr(q_rows), _ptr(q_index), int(R), _ptr(k_store),
                                                            _ptr(v_store), int(n_store_rows), offs, row0, src,
                                                            len(_a) - 1, int(L), _ptr(k_new), _ptr(v_new), _ptr(out),
                                                            _ptr(lse_out), _stream(stream)))

    def fr_shared_batch_workspace_bytes(self, n_queries: int, max_L: int) -> int:
        return int(self._lib.fr_shared_batch_workspace_bytes(self._h, int(n_queries), int(max_L)))

    def fr_sparse_prefill_attn_shared_batch(self, queries, k_store, v_store, n_store_rows: int, workspace,
                                            workspace_bytes: Optional[int] = None, stream=None):
        """queries: sequence of dicts with the keys q_rows, q_index, R, chunk_offsets, chunk_store_row0, chunk_src_pos0,
        L, k_new, v_new, out and optionally lse_out (the per-query arguments of fr_sparse_prefill_attn_shared)."""
        arr = (fr_shared_query * max(1, len(queries)))()
        keep = []
        for i, q in enumerate(queries):
            offs, a = _i32_array(q["chunk_offsets"])
            row0, b = _i32_array(q["chunk_store_row0"])
            src, c = _i32_array(q["chunk_src_pos0"])
            keep += [a, b, c]
            arr[i] = fr_shared_query(_ptr(q["q_rows"]), _ptr(q["q_index"]), int(q["R"]), offs, row0, src, len(a) - 1,
                                     int(q["L"]), _ptr(q["k_new"]), _ptr(q["v_new"]), _ptr(q["out"]),
                                     _ptr(q.get("lse_out")))
        if workspace_bytes is None:
            workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        self._check(self._lib.fr_sparse_prefill_attn_shared_batch(self._h, arr, len(queries), _ptr(k_store), _ptr(v_store),
                                                                  int(n_store_rows), _ptr(workspace), int(workspace_bytes),
                                                                  _stream(stream)))

    def fr_decode_attn(self, q, n_queries: int, k_shared, v_shared, n_shared_rows: int, seg_offsets, seg_row0, seg_len,
                       seg_delta, n_segments: int, stale_bits, stale_words: int, k_pages, v_pages, page_stride_rows: int,
                       page_len, out, lse_out=None, stream=None):
        self._check(self._lib.fr_decode_attn(self._h, _ptr(q), int(n_queries), _ptr(k_shared), _ptr(v_shared),
                                             int(n_shared_rows), _ptr(seg_offsets), _ptr(seg_row0), _ptr(seg_len),
                                             _ptr(seg_delta), int(n_segments), _ptr(stale_bits), int(stale_words),
                                             _ptr(k_pages), _ptr(v_pages), int(page_stride_rows), _ptr(page_len),
                                             _ptr(out), _ptr(lse_out), _stream(stream)))

    def fr_mark_stale_rows(self, stale_bits, n_words: int, rows, n_rows: int, clear: bool = True, stream=None):
        self._check(self._lib.fr_mark_stale_rows(self._h, _ptr(stale_bits), int(n_words), _ptr(rows), int(n_rows),
                                                 int(bool(clear)), _stream(stream)))

    def fr_kv_scatter(self, k_new, v_new, q_index, R: int, k_cache, v_cache, L: int, stream=None):
        self._check(self._lib.fr_kv_scatter(self._h, _ptr(k_new), _ptr(v_new), _ptr(q_index), int(R), _ptr(k_cache),
                                            _ptr(v_cache), int(L), _stream(stream)))

    def fr_rmsnorm(self, x, gain, R: int, hidden: int, eps: float, out, stream=None):
        self._check(self._lib.fr_rmsnorm(self._h, _ptr(x), _ptr(gain), int(R), int(hidden), float(eps), _ptr(out),
                                         _stream(stream)))

    def fr_linear(self, a, w, M: int, N: int, K: int, residual, out, stream=None):
        self._check(self._lib.fr_linear(self._h, _ptr(a), _ptr(w), int(M), int(N), int(K), _ptr(residual), _ptr(out),
                                        _stream(stream)))

    def fr_linear_swiglu(self, a, w_gate_up, M: int, F: int, K: int, out, stream=None):
        self._check(self._lib.fr_linear_swiglu(self._h, _ptr(a), _ptr(w_gate_up), int(M), int(F), int(K), _ptr(out),
                                               _stream(stream)))

    def fr_qkv_rope(self, a, w_qkv, M: int, K: int, positions, q_out, k_out, v_out, stream=None):
        self._check(self._lib.fr_qkv_rope(self._h, _ptr(a), _ptr(w_qkv), int(M), int(K), _ptr(positions), _ptr(q_out),
                                          _ptr(k_out), _ptr(v_out), _stream(stream)))

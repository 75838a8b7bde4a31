"""Shared helpers of the GPU parity tests: upload a synthetic workload, call the C-ABI binding,
compare with the oracle.  Comparison rules follow the stated tolerances: index sets bit-exact apart
from ties within 1e-3 relative score; floating point within max relative error (max |gpu - oracle|
over the tensor divided by max |oracle|) of 2e-2 for bf16 storage and 1e-5 for fp32."""
from __future__ import annotations

import numpy as np
import torch

from paper_2601_12904_amd import binding as B
from paper_2601_12904_amd import synth

TOL = {"f32": 1e-5, "bf16": 2e-2}
TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}
FR_DTYPE = {"f32": B.FR_F32, "bf16": B.FR_BF16}


def dev(x: np.ndarray, dtype: str) -> torch.Tensor:
    """Host fp32 array (values representable in `dtype`) -> device tensor of that dtype."""
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(TORCH_DTYPE[dtype]).cuda()


def host(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def make_ctx(shape: synth.LayerShape, max_tokens: int, max_chunks: int, max_q: int, **kw) -> B.Context:
    return B.Context(shape.n_q_heads, shape.n_kv_heads, shape.head_dim, FR_DTYPE[shape.dtype], shape.rope_base,
                     max_tokens=max_tokens, max_chunks=max_chunks, max_question_tokens=max_q, **kw)


def max_rel_err(got: np.ndarray, want: np.ndarray) -> float:
    denom = float(np.max(np.abs(want)))
    if denom == 0.0:
        return float(np.max(np.abs(got)))
    return float(np.max(np.abs(got - want)) / denom)


def assert_close(got, want, dtype: str, what: str = ""):
    err = max_rel_err(np.asarray(got, dtype=np.float64), np.asarray(want, dtype=np.float64))
    assert np.all(np.isfinite(got)), f"{what}: non-finite values"
    assert err <= TOL[dtype], f"{what}: max relative error {err:.3e} > {TOL[dtype]:.0e}"
    return err


def assert_index_set(q_index_gpu: np.ndarray, oracle_scores: np.ndarray, k: int, nq: int, rel_tie: float = 1e-3):
    """The first k entries are the chosen context tokens: strictly ascending, and equal to the oracle's
    set except for tokens whose oracle score lies within `rel_tie` (relative) of the k-th score.
    The last nq entries are the question positions.  Returns the number of tokens in the tie window."""
    L_ctx = len(oracle_scores)
    qi = np.asarray(q_index_gpu, dtype=np.int64)
    assert qi.shape == (k + nq,)
    assert np.array_equal(qi[k:], L_ctx + np.arange(nq)), "question positions wrong"
    sel = qi[:k]
    if k == 0:
        return 0
    assert np.all(np.diff(sel) > 0) and sel[0] >= 0 and sel[-1] < L_ctx, "selection not strictly ascending in range"
    order = np.lexsort((np.arange(L_ctx), -oracle_scores))
    want = np.sort(order[:k])
    if k == L_ctx:
        assert np.array_equal(sel, want)
        return 0
    kth = oracle_scores[order[k - 1]]
    in_window = np.abs(oracle_scores - kth) <= rel_tie * abs(kth)
    diff = np.setxor1d(sel, want)
    assert np.all(in_window[diff]), (f"{len(diff)} selected tokens differ from the oracle's set and "
                                     f"{int((~in_window[diff]).sum())} of them are outside the tie window")
    return int(in_window.sum())

"""Shared helpers of the GPU parity tests: upload a synthetic workload, call the C-ABI binding,
compare with the oracle.  Comparison rules follow the stated tolerances: index sets bit-exact apart
from ties within 1e-3 relative score; floating point within max relative error (max |gpu - oracle|
over the tensor divided by max |oracle|) of 2e-2 for bf16 storage and 1e-5 for fp32."""
from __future__ import annotations

import numpy as np
from paper_2601_12904_amd import binding as B  # noqa: F401
from paper_2601_12904_amd import synth  # noqa: F401

TOL = {"f32": 1e-5, "bf16": 2e-2}
# Second, element-wise figure: max over elements of |gpu - oracle| / (|oracle| + ELEMENTWISE_FLOOR * max |oracle|).
# The floor keeps elements near zero from dividing by nothing; a storage ulp of an element of average size stays
# visible.  Reported next to the tensor-normalised error; bounded by ELEMENTWISE_TOL where a test asks for it.
ELEMENTWISE_FLOOR = 1e-3
from paper_2601_12904_amd.devmem import FR_DTYPE, TORCH_DTYPE, dev, host, make_ctx  # noqa: E402,F401  (re-exported)


def max_rel_err(got: np.ndarray, want: np.ndarray) -> float:
    denom = float(np.max(np.abs(want)))
    if denom == 0.0:
        return float(np.max(np.abs(got)))
    return float(np.max(np.abs(got - want)) / denom)


def elementwise_rel_err(got: np.ndarray, want: np.ndarray) -> float:
    """max_i |got_i - want_i| / (|want_i| + ELEMENTWISE_FLOOR * max_j |want_j|)."""
    got, want = np.asarray(got, dtype=np.float64), np.asarray(want, dtype=np.float64)
    if want.size == 0:
        return 0.0
    floor = ELEMENTWISE_FLOOR * float(np.max(np.abs(want)))
    if floor == 0.0:
        return float(np.max(np.abs(got)))
    return float(np.max(np.abs(got - want) / (np.abs(want) + floor)))


class Err(float):
    """The tensor-normalised error as a float, with the element-wise figure riding along (`.elementwise`)."""
    elementwise: float = 0.0


def assert_close(got, want, dtype: str, what: str = "", elementwise_tol: float = None):
    got, want = np.asarray(got, dtype=np.float64), np.asarray(want, dtype=np.float64)
    assert np.all(np.isfinite(got)), f"{what}: non-finite values"
    err = Err(max_rel_err(got, want))
    err.elementwise = elementwise_rel_err(got, want)
    assert err <= TOL[dtype], f"{what}: max relative error {float(err):.3e} > {TOL[dtype]:.0e}"
    if elementwise_tol is not None:
        assert err.elementwise <= elementwise_tol, (f"{what}: element-wise relative error {err.elementwise:.3e} > "
                                                    f"{elementwise_tol:.0e}")
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

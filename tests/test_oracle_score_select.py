"""Pins for the oracle's Query-Guided Selection (Sec. 3.2) and Q index (Sec. 4.3)."""
import math

import numpy as np
import pytest
import scipy.special

from oracle import fusionrag_oracle as orc
from tests.conftest import read_golden_table


def brute_scores(q, k, offs, norm):
    """Triple loop over (head, question token, key) with explicit per-row normalisers."""
    nq, Hq, d = q.shape
    L, Hkv, _ = k.shape
    G = Hq // Hkv
    out = [0.0] * L
    for h in range(Hq):
        for i in range(nq):
            logit = [sum(q[i, h, t] * k[j, h // G, t] for t in range(d)) / math.sqrt(d) for j in range(L)]
            if norm == "raw":
                for j in range(L):
                    out[j] += logit[j]
                continue
            scopes = [(0, L)] if norm == "global" else [(offs[c], offs[c + 1]) for c in range(len(offs) - 1)]
            for s, e in scopes:
                z = sum(math.exp(logit[j]) for j in range(s, e))
                for j in range(s, e):
                    out[j] += math.exp(logit[j]) / z
    return np.array(out)


@pytest.mark.parametrize("norm", ["per_chunk", "global", "raw"])
def test_scores_brute_force(norm):
    rng = np.random.default_rng(0)
    q = rng.standard_normal((3, 4, 8))
    k = rng.standard_normal((11, 2, 8))
    offs = [0, 4, 5, 11]
    got = orc.critical_scores(q, k, offs, norm)
    assert np.allclose(got, brute_scores(q, k, offs, norm), rtol=1e-12, atol=1e-12)


def test_score_mass_closed_form():
    rng = np.random.default_rng(1)
    nq, Hq, Hkv, d = 5, 6, 3, 16
    q = rng.standard_normal((nq, Hq, d)) * 3
    k = rng.standard_normal((40, Hkv, d))
    offs = [0, 7, 20, 33, 40]
    s = orc.critical_scores(q, k, offs, "per_chunk")
    # every (row, head) spreads exactly one unit of attention over each chunk
    for c in range(4):
        assert math.isclose(s[offs[c]:offs[c + 1]].sum(), Hq * nq, rel_tol=1e-12)
    assert math.isclose(orc.critical_scores(q, k, offs, "global").sum(), Hq * nq, rel_tol=1e-12)


def test_single_row_single_head_is_library_softmax():
    rng = np.random.default_rng(2)
    q = rng.standard_normal((1, 1, 32))
    k = rng.standard_normal((50, 1, 32))
    logits = (k[:, 0, :] @ q[0, 0]) / math.sqrt(32)
    assert np.allclose(orc.critical_scores(q, k, [0, 50], "global"), scipy.special.softmax(logits), rtol=1e-12)
    want = np.concatenate([scipy.special.softmax(logits[:20]), scipy.special.softmax(logits[20:])])
    assert np.allclose(orc.critical_scores(q, k, [0, 20, 50], "per_chunk"), want, rtol=1e-12)


def test_raw_closed_form_and_gqa_mapping():
    # without softmax the score is linear: (sum of the group's queries) . k / sqrt(d); this also pins
    # which KV head a query head reads (contiguous groups)
    rng = np.random.default_rng(3)
    q = rng.standard_normal((4, 4, 8))
    k = rng.standard_normal((9, 2, 8))
    want = (k[:, 0, :] @ q[:, 0:2, :].sum(axis=(0, 1)) + k[:, 1, :] @ q[:, 2:4, :].sum(axis=(0, 1))) / math.sqrt(8)
    assert np.allclose(orc.critical_scores(q, k, [0, 9], "raw"), want, rtol=1e-12)


def test_scores_permute_with_tokens_inside_a_chunk():
    rng = np.random.default_rng(4)
    q = rng.standard_normal((6, 2, 8))
    k = rng.standard_normal((12, 2, 8))
    offs = [0, 5, 12]
    perm = np.concatenate([rng.permutation(5), 5 + rng.permutation(7)])
    s = orc.critical_scores(q, k, offs, "per_chunk")
    sp = orc.critical_scores(q, k[perm], offs, "per_chunk")
    assert np.allclose(sp, s[perm], rtol=1e-12)
    # per-chunk scores of a chunk do not depend on the other chunks at all
    k2 = k.copy()
    k2[5:] = rng.standard_normal((7, 2, 8))
    assert np.allclose(orc.critical_scores(q, k2, offs, "per_chunk")[:5], s[:5], rtol=1e-12)


def test_topk_count():
    assert orc.topk_count(16384, 0.15) == 2458      # 2457.6 rounds up
    assert orc.topk_count(512, 0.15) == 77          # 76.8
    assert orc.topk_count(16384, 0.05) == 819
    assert orc.topk_count(16384, 0.30) == 4915
    assert orc.topk_count(32768, 0.15) == 4915
    assert orc.topk_count(10, 0.25) == 3            # 2.5 rounds half up
    assert orc.topk_count(100, 1.0) == 100 and orc.topk_count(100, 0.0) == 0
    assert orc.topk_count(100, 1.7) == 100


def test_select_equals_full_sort_definition():
    rng = np.random.default_rng(5)
    s = rng.random(200)
    for k in (0, 1, 17, 199, 200):
        qi = orc.select_q_index(s, k, 4)
        want = np.sort(np.argsort(-s, kind="stable")[:k])
        assert np.array_equal(qi[:k], want)
        assert np.array_equal(qi[k:], 200 + np.arange(4))
        assert np.all(np.diff(qi) > 0)
    # the selected set is exactly the set of the k largest values
    qi = orc.select_q_index(s, 50, 0)
    assert s[qi].min() > np.delete(s, qi).max()


def test_select_ties_lowest_index():
    s = np.array([1.0, 3.0, 3.0, 3.0, 0.5, 3.0])
    assert list(orc.select_q_index(s, 2, 0)) == [1, 2]
    assert list(orc.select_q_index(s, 5, 1)) == [0, 1, 2, 3, 5, 6]
    assert list(orc.select_q_index(np.ones(6), 3, 0)) == [0, 1, 2]


def test_worked_q_index_example():
    rows = {r[0]: [int(v) for v in r[1:]] for r in read_golden_table("q_index_example.txt")}
    n_slots = rows["context_slots"][0]
    scores = np.zeros(n_slots)
    for rank, tok in enumerate(rows["critical"]):
        scores[tok - 1] = 10.0 - rank                       # 1-based token -> 0-based slot
    qi = orc.select_q_index(scores, len(rows["critical"]), rows["question_tokens"][0])
    assert list(qi + 1) == rows["q_index"]                   # back to the paper's 1-based slots


def test_kv_deviation_closed_form():
    a = np.zeros((3, 2, 2, 4))
    b = np.zeros((3, 2, 2, 4))
    b[1] = 0.5                                               # 16 components differ by 0.5 -> 16 * 0.25
    b[2, 0, 1, 3] = -2.0
    assert np.allclose(orc.kv_deviation(a, b), [0.0, 4.0, 4.0])


def test_kv_deviation_polarisation_identity_and_selector():
    # |a - b|^2 = |a|^2 + |b|^2 - 2 a.b, row by row (a different route to the same number) ...
    rng = np.random.default_rng(5)
    a = rng.standard_normal((40, 3, 8))
    b = a + 0.1 * rng.standard_normal((40, 3, 8))
    b[[7, 21, 30]] += 1.0                                     # three tokens deviate strongly
    a2, b2 = a.reshape(40, -1), b.reshape(40, -1)
    want = (a2 * a2).sum(1) + (b2 * b2).sum(1) - 2.0 * np.einsum("tc,tc->t", a2, b2)
    assert np.allclose(orc.kv_deviation(a, b), want, rtol=1e-10, atol=1e-12)
    # ... symmetric, zero only for equal rows, and the top-3 of it are the planted tokens (eq. 8)
    assert np.array_equal(orc.kv_deviation(a, b), orc.kv_deviation(b, a))
    assert orc.kv_deviation(a, a).max() == 0.0
    assert list(orc.select_q_index(orc.kv_deviation(a, b), 3, 2)) == [7, 21, 30, 40, 41]

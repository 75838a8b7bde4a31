"""Pins for the oracle's rotary position recovery (Appendix A of the paper)."""
import math

import numpy as np
import pytest

from oracle import fusionrag_oracle as orc
from tests.conftest import read_golden_table


def textbook_rope_complex(x, positions, base, index_base=0):
    """RoPE as the RoFormer paper states it: view each consecutive pair as a complex number and
    multiply by exp(i * s * theta_p).  Written with complex arithmetic, not the oracle's formula."""
    d = x.shape[-1]
    z = x[..., 0::2] + 1j * x[..., 1::2]
    p = np.arange(d // 2) + index_base
    theta = np.exp(-2.0 * p / d * np.log(base))
    rot = np.exp(1j * np.asarray(positions, dtype=np.float64)[:, None, None] * theta)
    z = z * rot
    out = np.empty_like(x)
    out[..., 0::2], out[..., 1::2] = z.real, z.imag
    return out


def test_closed_form_single_pair():
    # d = 2, base anything: theta_0 = 1, so k = [1, 0] moved by Delta = 3 is [cos 3, sin 3];
    # k = [0, 1] is [-sin 3, cos 3]  (rotate(k) = [-k2, k1])
    k = np.array([[[1.0, 0.0]], [[0.0, 1.0]]])
    out = orc.rope_shift(k, [0, 2], [2], [5], base=10000.0)
    assert np.allclose(out[0, 0], [math.cos(3), math.sin(3)], atol=1e-15)
    assert np.allclose(out[1, 0], [-math.sin(3), math.cos(3)], atol=1e-15)


def test_frequency_index_conventions():
    # d = 4, base 10000: usual form theta = [1, 1e-2]; the appendix's printed form (i from 1) = [1e-2, 1e-4]
    assert np.allclose(orc.rope_frequencies(4, 10000.0, 0), [1.0, 1e-2], rtol=1e-14)
    assert np.allclose(orc.rope_frequencies(4, 10000.0, 1), [1e-2, 1e-4], rtol=1e-14)
    # second pair of a d = 4 key rotates by Delta * 1e-2
    k = np.array([[[0.0, 0.0, 1.0, 0.0]]])
    out = orc.rope_shift(k, [0, 1], [0], [50], base=10000.0)
    assert np.allclose(out[0, 0], [0, 0, math.cos(0.5), math.sin(0.5)], atol=1e-15)


def test_half_layout_pairs():
    # half-split layout pairs dimension p with p + d/2
    k = np.array([[[1.0, 0.0, 0.0, 0.0]]])
    out = orc.rope_shift(k, [0, 1], [0], [2], base=10000.0, layout="half")
    assert np.allclose(out[0, 0], [math.cos(2), 0, math.sin(2), 0], atol=1e-15)


def test_worked_example_positions():
    rows = read_golden_table("appendix_a_positions.txt")
    cached = {r[0]: [int(v) for v in r[1].split(",")] for r in rows}
    after = {r[0]: [int(v) for v in r[2].split(",")] for r in rows}
    # 0-based storage: the two chunks' KV are concatenated; chunk rows 0..2 and 3..6
    offsets = [0, len(cached["C1"]), len(cached["C1"]) + len(cached["C2"])]
    src0 = [cached["C1"][0], cached["C2"][0]]
    dst0 = [after["C1"][0], after["C2"][0]]
    assert dst0[1] - src0[1] == 3 == len(cached["C1"])        # Delta of the second chunk = |C1|
    rng = np.random.default_rng(0)
    raw = rng.standard_normal((7, 2, 8))
    base = 10000.0
    cached_pos = np.array(cached["C1"] + cached["C2"])
    after_pos = np.array(after["C1"] + after["C2"])
    k_cached = textbook_rope_complex(raw, cached_pos, base)
    want = textbook_rope_complex(raw, after_pos, base)
    got = orc.rope_shift(k_cached, offsets, src0, dst0, base)
    assert np.allclose(got, want, atol=1e-13)
    # the first chunk does not move at all
    assert np.array_equal(got[:3], np.asarray(k_cached[:3]))


@pytest.mark.parametrize("layout", ["interleaved", "half"])
@pytest.mark.parametrize("index_base", [0, 1])
def test_additivity_identity_norm(layout, index_base):
    rng = np.random.default_rng(1)
    k = rng.standard_normal((37, 3, 16))
    offs = [0, 10, 11, 37]
    a = orc.rope_shift(k, offs, [0, 4, 9], [7, 100, 2000], 500000.0, layout, index_base)
    ab = orc.rope_shift(a, offs, [7, 100, 2000], [8, 3000, 1], 500000.0, layout, index_base)
    direct = orc.rope_shift(k, offs, [0, 4, 9], [8, 3000, 1], 500000.0, layout, index_base)
    assert np.allclose(ab, direct, atol=1e-12)                      # shift(shift(k,a),b) = shift(k,a+b)
    same = orc.rope_shift(k, offs, [5, 5, 5], [5, 5, 5], 500000.0, layout, index_base)
    assert np.array_equal(same, k)                                   # Delta = 0 is the identity
    pa, pb = orc._pair_views(k, layout)
    qa, qb = orc._pair_views(a, layout)
    assert np.allclose(pa ** 2 + pb ** 2, qa ** 2 + qb ** 2, atol=1e-12)   # every pair keeps its norm


def test_shift_moves_textbook_rope_between_positions():
    rng = np.random.default_rng(2)
    raw = rng.standard_normal((64, 2, 32))
    offs = [0, 20, 64]
    base = 500000.0
    local = np.concatenate([np.arange(20), np.arange(44)])          # every chunk cached from position 0
    glob = np.arange(64) + 1000                                      # lands at 1000..1063
    k_cached = textbook_rope_complex(raw, local, base)
    got = orc.rope_shift(k_cached, offs, [0, 0], None, base, dst_base=1000)
    assert np.allclose(got, textbook_rope_complex(raw, glob, base), atol=1e-12)
    assert np.allclose(orc.rope_rotate(raw, glob, base), textbook_rope_complex(raw, glob, base), atol=1e-12)


def test_inner_product_depends_on_relative_position_only():
    # the property that makes the shift meaningful: <RoPE(q,m), RoPE(k,n)> is a function of m - n
    rng = np.random.default_rng(3)
    q, k = rng.standard_normal((1, 1, 64)), rng.standard_normal((1, 1, 64))
    a = (orc.rope_rotate(q, [17], 1e4) * orc.rope_rotate(k, [5], 1e4)).sum()
    b = (orc.rope_rotate(q, [1017], 1e4) * orc.rope_rotate(k, [1005], 1e4)).sum()
    assert abs(a - b) < 1e-10

"""Host-side checks of the synthetic workload generator and of the oracle chained over it."""
import numpy as np
import torch

from oracle import fusionrag_oracle as orc
from paper_2601_12904_amd import synth


def test_deterministic_and_seed_dependent():
    a, b, c = synth.config_tiny(seed=0), synth.config_tiny(seed=0), synth.config_tiny(seed=1)
    for f in ("k_cached", "v_cached", "q_full", "k_full", "v_full", "focus"):
        assert np.array_equal(getattr(a, f), getattr(b, f))
    assert not np.array_equal(a.k_cached, c.k_cached)


def test_tiny_shapes():
    w = synth.config_tiny()
    assert w.L_ctx == 512 and w.nq == 32 and w.L == 544 and w.n_chunks == 4
    assert w.k_cached.shape == (512, 4, 64) and w.q_full.shape == (544, 4, 64)
    assert len(w.focus) == 32 and all(np.sum((w.focus >= 128 * c) & (w.focus < 128 * (c + 1))) == 8 for c in range(4))
    assert orc.topk_count(w.L_ctx, w.ratio) == 77


def test_bf16_values_are_representable():
    w = synth.config_small_bf16()
    for a in (w.k_cached, w.v_cached, w.q_full, w.k_full, w.v_full):
        t = torch.from_numpy(a)
        assert torch.equal(t.to(torch.bfloat16).to(torch.float32), t)


def test_ragged_lengths():
    lens = synth.ragged_chunk_lengths(synth._rng(0, 0), 64, 32768, 256, 1024)
    assert len(lens) == 64 and lens.sum() == 32768 and lens.min() >= 256 and lens.max() <= 1024
    assert len(set(lens.tolist())) > 20


def test_focus_tokens_are_found_by_the_oracle_chain():
    # sanity, not parity: after the position shift the planted tokens still collect the most
    # attention from the question, so Query-Guided Selection picks (nearly) all of them
    w = synth.config_tiny()
    k_ctx = orc.rope_shift(w.k_cached, w.chunk_offsets, w.src_pos0, None, w.shape.rope_base)
    s = orc.critical_scores(w.q_question, k_ctx, w.chunk_offsets)
    qi = orc.select_q_index(s, orc.topk_count(w.L_ctx, w.ratio), w.nq)
    found = np.isin(w.focus, qi).mean()
    assert found >= 0.9
    # few scores sit within the tie window of the k-th score
    kth = np.sort(s)[::-1][76]
    assert np.sum(np.abs(s - kth) <= 1e-3 * kth) <= 3

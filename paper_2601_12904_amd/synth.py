"""Seeded synthetic inputs shaped like the paper's RAG prompts.

This module draws random numbers, plants structure and rounds to the storage
dtype.  It contains none of the method's arithmetic (no rotation, no attention,
no selection): both the CPU oracle's tests and the HIP path's tests consume its
arrays, so anything computed here could not be checked by comparing the two.

What a workload holds (token-major ``[tokens, heads, head_dim]``, fp32 arrays
whose values are exactly representable in the storage dtype):

* ``k_cached, v_cached [L_ctx, Hkv, d]`` -- the stale per-chunk KV cache as it
  was stored offline: chunk ``c`` occupies rows ``chunk_offsets[c] ..
  chunk_offsets[c+1]`` and its keys carry the rotary phase of positions
  ``src_pos0[c] + t`` (Full Reuse, Sec. 2.2.1 / eq. 5-6 of the paper).
* ``q_full [L, Hq, d]``, ``k_full, v_full [L, Hkv, d]`` -- what a full prefill
  of the assembled prompt would produce at global positions ``0..L-1``; the
  harness gathers the recomputed rows from these (``X[C_idx]`` and the question
  in eq. 9).  Rows ``L_ctx..L-1`` are the question.
* ``focus`` -- context positions planted as "focus tokens": their keys (stale
  and fresh) get ``+3 sigma_K`` along a per-KV-head unit direction that the
  question queries share, which imitates the vertical stripes real attention
  shows (Sec. 3.2).  The direction lives in the lowest-frequency rotary pairs,
  whose phase moves by less than about 0.35 rad over the whole prompt, so the
  alignment survives the position shift without this module rotating anything.

The paper measures on Musique / LongBench prompts (about 17k tokens per query);
these arrays stand in for them.
"""
from __future__ import annotations

import dataclasses
from typing import Optional, Sequence

import numpy as np
import torch


@dataclasses.dataclass(frozen=True)
class LayerShape:
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str            # "f32" or "bf16": storage type of Q/K/V
    rope_base: float

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


@dataclasses.dataclass
class Workload:
    name: str
    shape: LayerShape
    seed: int
    chunk_offsets: np.ndarray      # int32 [C+1], [0] = 0, [C] = L_ctx
    src_pos0: np.ndarray           # int32 [C]: position the chunk's first token was cached at
    nq: int
    ratio: float
    k_cached: np.ndarray
    v_cached: np.ndarray
    q_full: np.ndarray
    k_full: np.ndarray
    v_full: np.ndarray
    focus: np.ndarray              # int64, sorted context positions

    @property
    def n_chunks(self) -> int:
        return len(self.chunk_offsets) - 1

    @property
    def L_ctx(self) -> int:
        return int(self.chunk_offsets[-1])

    @property
    def L(self) -> int:
        return self.L_ctx + self.nq

    @property
    def q_question(self) -> np.ndarray:
        return self.q_full[self.L_ctx:]


def round_to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp32 values to the storage dtype (nearest-even) and return them as fp32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype == "bf16":
        return torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    raise ValueError(f"unknown dtype {dtype!r}")


def _rng(seed: int, stream: int) -> np.random.Generator:
    # Philox is counter based: (seed, stream) names an independent sequence.
    return np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))


def _focus_direction(rng: np.random.Generator, n_kv_heads: int, d: int) -> np.ndarray:
    """Unit vector per KV head supported on the last d/8 head dimensions: under the paper's
    interleaved pair layout these are the d/16 lowest-frequency rotary pairs."""
    u = np.zeros((n_kv_heads, d), dtype=np.float64)
    n_pairs = max(1, d // 16)
    # members of the last n_pairs pairs under the interleaved layout: the last 2*n_pairs dims
    u[:, d - 2 * n_pairs:] = rng.standard_normal((n_kv_heads, 2 * n_pairs))
    u /= np.linalg.norm(u, axis=1, keepdims=True)
    return u


def ragged_chunk_lengths(rng: np.random.Generator, n_chunks: int, total: int,
                         lo: int, hi: int) -> np.ndarray:
    """Lengths in [lo, hi] that sum to ``total``: a uniform draw rescaled onto the fixed
    total, the rounding remainder spread one token at a time over the chunks with room."""
    if not (n_chunks * lo <= total <= n_chunks * hi):
        raise ValueError("total not reachable with these bounds")
    u = rng.integers(lo, hi + 1, size=n_chunks).astype(np.float64)
    spare = total - n_chunks * lo
    w = u - lo
    if w.sum() == 0:
        w[:] = 1.0
    lens = lo + np.floor(w * spare / w.sum()).astype(np.int64)
    lens = np.minimum(lens, hi)
    order = np.argsort(-w, kind="stable")
    i = 0
    while lens.sum() < total:
        c = order[i % n_chunks]
        if lens[c] < hi:
            lens[c] += 1
        i += 1
    assert lens.sum() == total and lens.min() >= lo and lens.max() <= hi
    return lens


def make_workload(name: str, shape: LayerShape, chunk_lens: Sequence[int], nq: int, ratio: float,
                  seed: int = 0, sigma_q: float = 1.0, sigma_kv: float = 1.0,
                  focus_per_chunk: Optional[int] = None, focus_frac: Optional[float] = None,
                  focus_zipf: bool = False, src_pos0: Optional[Sequence[int]] = None) -> Workload:
    Hq, Hkv, d = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    G = shape.group
    chunk_lens = np.asarray(chunk_lens, dtype=np.int64)
    C = len(chunk_lens)
    offsets = np.zeros(C + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(chunk_lens)
    L_ctx = int(offsets[-1])
    L = L_ctx + nq

    # ---- focus positions ------------------------------------------------------------
    r_f = _rng(seed, 1)
    if focus_per_chunk is not None:
        picks = [int(offsets[c]) + r_f.choice(int(chunk_lens[c]), size=min(focus_per_chunk, int(chunk_lens[c])),
                                              replace=False) for c in range(C)]
        focus = np.sort(np.concatenate(picks)) if picks else np.zeros(0, np.int64)
    elif focus_frac:
        n_focus = int(round(focus_frac * L_ctx))
        if focus_zipf:
            # chunk shares proportional to 1/rank over a seeded permutation of the chunks
            perm = r_f.permutation(C)
            share = np.zeros(C)
            share[perm] = 1.0 / np.arange(1, C + 1)
            share /= share.sum()
            per_chunk = np.minimum(np.floor(share * n_focus).astype(np.int64), chunk_lens)
            picks = [int(offsets[c]) + r_f.choice(int(chunk_lens[c]), size=int(per_chunk[c]), replace=False)
                     for c in range(C)]
            focus = np.sort(np.concatenate(picks))
        else:
            focus = np.sort(r_f.choice(L_ctx, size=n_focus, replace=False))
    else:
        focus = np.zeros(0, np.int64)
    focus = focus.astype(np.int64)

    u = _focus_direction(_rng(seed, 2), Hkv, d)                      # [Hkv, d]

    def gauss(stream: int, shp, sigma: float) -> np.ndarray:
        return (_rng(seed, stream).standard_normal(shp, dtype=np.float32) * np.float32(sigma))

    q_full = gauss(3, (L, Hq, d), sigma_q)
    k_full = gauss(4, (L, Hkv, d), sigma_kv)
    v_full = gauss(5, (L, Hkv, d), sigma_kv)
    k_cached = gauss(6, (L_ctx, Hkv, d), sigma_kv)
    v_cached = gauss(7, (L_ctx, Hkv, d), sigma_kv)

    # question queries share a component along u (all G query heads of a KV group use the group's u)
    u_q = np.repeat(u, G, axis=0)                                    # [Hq, d]
    q_full[L_ctx:] += (sigma_q * np.sqrt(d) * u_q).astype(np.float32)[None]
    # focus keys: +3 sigma_K along u, in the stale cache and in the fresh keys alike
    bump = (3.0 * sigma_kv * u).astype(np.float32)[None]
    k_full[focus] += bump
    k_cached[focus] += bump

    dt = shape.dtype
    if src_pos0 is None:
        src_pos0 = np.zeros(C, dtype=np.int32)
    return Workload(
        name=name, shape=shape, seed=seed, chunk_offsets=offsets,
        src_pos0=np.asarray(src_pos0, dtype=np.int32), nq=nq, ratio=ratio,
        k_cached=round_to_storage(k_cached, dt), v_cached=round_to_storage(v_cached, dt),
        q_full=round_to_storage(q_full, dt), k_full=round_to_storage(k_full, dt),
        v_full=round_to_storage(v_full, dt), focus=focus)


# ---- the named configurations -----------------------------------------------------------

TINY_F32 = LayerShape(n_q_heads=4, n_kv_heads=4, head_dim=64, dtype="f32", rope_base=10000.0)
LLAMA3_8B_BF16 = LayerShape(n_q_heads=32, n_kv_heads=8, head_dim=128, dtype="bf16", rope_base=500000.0)


def config_tiny(seed: int = 0, ratio: float = 0.15) -> Workload:
    """4 x 128 context tokens + 32 question tokens, fp32, 4/4 heads, d 64, 8 focus tokens per chunk."""
    return make_workload("tiny_f32_4x128+32", TINY_F32, [128] * 4, nq=32, ratio=ratio, seed=seed,
                         sigma_q=1.0, sigma_kv=1.0, focus_per_chunk=8)


def config_17k(seed: int = 0, ratio: float = 0.15) -> Workload:
    """16 x 1024 context tokens + 512 question tokens, bf16, 32/8 heads, d 128, 2 % focus tokens."""
    d = LLAMA3_8B_BF16.head_dim
    return make_workload("llama3_8b_layer_16x1024+512", LLAMA3_8B_BF16, [1024] * 16, nq=512, ratio=ratio,
                         seed=seed, sigma_q=float(np.sqrt(d)), sigma_kv=float(1.0 / np.sqrt(d)),
                         focus_frac=0.02)


def config_long_ragged(seed: int = 0, ratio: float = 0.15) -> Workload:
    """64 ragged chunks (256..1024, total 32768) + 1024 question tokens, bf16, Zipf focus tokens."""
    d = LLAMA3_8B_BF16.head_dim
    lens = ragged_chunk_lengths(_rng(seed, 0), 64, 32768, 256, 1024)
    return make_workload("llama3_8b_layer_64xU[256,1024]+1024", LLAMA3_8B_BF16, lens, nq=1024, ratio=ratio,
                         seed=seed, sigma_q=float(np.sqrt(d)), sigma_kv=float(1.0 / np.sqrt(d)),
                         focus_frac=0.02, focus_zipf=True)


def config_small_bf16(seed: int = 0, ratio: float = 0.15, chunk_lens: Sequence[int] = (200, 333, 91, 256),
                      nq: int = 40, shape: LayerShape = LLAMA3_8B_BF16) -> Workload:
    """A Llama-3-8B-shaped layer cut down to a few hundred tokens with ragged chunks: spans
    several kernel tiles plus ragged tails, small enough for the oracle to finish in seconds."""
    d = shape.head_dim
    return make_workload("small_bf16", shape, list(chunk_lens), nq=nq, ratio=ratio, seed=seed,
                         sigma_q=float(np.sqrt(d)), sigma_kv=float(1.0 / np.sqrt(d)), focus_frac=0.03)


CONFIGS = {1: config_tiny, 2: config_17k, 4: config_long_ragged}
RATIO_SWEEP = (0.05, 0.10, 0.15, 0.30, 1.00)

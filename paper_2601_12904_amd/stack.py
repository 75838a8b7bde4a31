"""A Llama-shaped decoder stack driven through the C-ABI binding: per layer, the model steps around the path
(RMSNorm, Q/K/V projection with RoPE, output projection, SwiGLU feed-forward) for the recomputed rows only,
with the selective-prefill calls in between.  Argument marshalling and buffer management only: every step runs
in the library's kernels.  Weights are random (there are no checkpoints here); the shapes are the model's."""
from __future__ import annotations

import dataclasses
from typing import List, Optional

import torch

from . import binding as B


@dataclasses.dataclass
class LayerWeights:
    g1: torch.Tensor          # [hidden]
    w_qkv: torch.Tensor       # [(Hq + 2 Hkv) d, hidden]: query heads, key heads, value heads
    w_o: torch.Tensor         # [hidden, Hq d]
    g2: torch.Tensor          # [hidden]
    w_gate_up: torch.Tensor   # [2 ffn, hidden]: gate and up rows interleaved
    w_down: torch.Tensor      # [hidden, ffn]


def random_layer(hidden: int, ffn: int, Hq: int, Hkv: int, d: int, gen: torch.Generator, std: float = 0.02,
                 device: str = "cuda") -> LayerWeights:
    def w(n, k):
        return (torch.randn((n, k), generator=gen, device=device, dtype=torch.float32) * std).to(torch.bfloat16)
    ones = torch.ones(hidden, dtype=torch.bfloat16, device=device)
    return LayerWeights(ones.clone(), w((Hq + 2 * Hkv) * d, hidden), w(hidden, Hq * d), ones.clone(),
                        w(2 * ffn, hidden), w(hidden, ffn))


class SelectivePrefillStack:
    """Runs `layers` decoder layers over the rows listed in a Q index.  Per layer (the order of the full-stack
    configuration): Q/K/V projection of the rows, fr_rope_shift of that layer's cached keys, optionally
    fr_score_select on the layer's own question queries (result discarded: the row set of a sparse prefill is
    fixed before the first layer), fr_sparse_prefill_attn, fr_kv_scatter, output projection and feed-forward."""

    def __init__(self, ctx: B.Context, layers: List[LayerWeights], hidden: int, ffn: int, eps: float = 1e-5):
        self.ctx, self.layers, self.hidden, self.ffn, self.eps = ctx, layers, hidden, ffn, eps
        d = ctx.desc
        self.Hq, self.Hkv, self.d = d.n_q_heads, d.n_kv_heads, d.head_dim
        self._buf = {}

    def _scratch(self, R: int):
        if self._buf.get("R") != R:
            dev, bf = "cuda", torch.bfloat16
            self._buf = dict(
                R=R, x=torch.empty((R, self.hidden), dtype=bf, device=dev),
                q=torch.empty((R, self.Hq, self.d), dtype=bf, device=dev),
                k=torch.empty((R, self.Hkv, self.d), dtype=bf, device=dev),
                v=torch.empty((R, self.Hkv, self.d), dtype=bf, device=dev),
                attn=torch.empty((R, self.Hq, self.d), dtype=bf, device=dev),
                act=torch.empty((R, self.ffn), dtype=bf, device=dev))
        return self._buf

    def forward(self, h: torch.Tensor, q_index: torch.Tensor, k_cached: List[torch.Tensor], k_cache: List[torch.Tensor],
                v_cache: List[torch.Tensor], chunk_offsets, src_pos0, nq: int, L: int, select_every_layer: bool = False,
                k_select: int = 0, q_index_scratch: Optional[torch.Tensor] = None,
                capture: Optional[dict] = None) -> torch.Tensor:
        """h [R, hidden] is updated in place and returned; k_cache / v_cache [L, Hkv, d] per layer end up holding
        the stitched cache with the recomputed rows written back.  `capture`, if given, maps layer numbers to dicts
        that receive copies of the layer's input and output rows ("h_in", "h_out"): tests feed the input to the oracle."""
        c, R = self.ctx, h.shape[0]
        s = self._scratch(R)
        for l, w in enumerate(self.layers):
            if capture is not None and l in capture:
                capture[l]["h_in"] = h.clone()
            c.fr_rmsnorm(h, w.g1, R, self.hidden, self.eps, s["x"])
            c.fr_qkv_rope(s["x"], w.w_qkv, R, self.hidden, q_index, s["q"], s["k"], s["v"])
            c.fr_rope_shift(k_cached[l], k_cache[l], chunk_offsets, src_pos0)
            if select_every_layer:
                c.fr_score_select(s["q"][R - nq:], nq, k_cache[l], chunk_offsets, k_select, B.FR_NORM_PER_CHUNK, None,
                                  q_index_scratch)
            c.fr_sparse_prefill_attn(s["q"], q_index, R, k_cache[l], v_cache[l], L, s["k"], s["v"], s["attn"])
            c.fr_kv_scatter(s["k"], s["v"], q_index, R, k_cache[l], v_cache[l], L)
            c.fr_linear(s["attn"], w.w_o, R, self.hidden, self.Hq * self.d, h, h)
            c.fr_rmsnorm(h, w.g2, R, self.hidden, self.eps, s["x"])
            c.fr_linear_swiglu(s["x"], w.w_gate_up, R, self.ffn, self.hidden, s["act"])
            c.fr_linear(s["act"], w.w_down, R, self.hidden, self.ffn, h, h)
            if capture is not None and l in capture:
                capture[l]["h_out"] = h.clone()
        return h

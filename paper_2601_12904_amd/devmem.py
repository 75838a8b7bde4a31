"""Device-memory plumbing shared by the tests, the smoke check and the benchmark: host arrays to device tensors of
the storage dtype and back, and a context for a synthetic workload's shape.  PyTorch is used for allocation and
copies only; nothing here computes."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B
from . import synth

TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}
FR_DTYPE = {"f32": B.FR_F32, "bf16": B.FR_BF16}


def dev(x: np.ndarray, dtype: str) -> torch.Tensor:
    """Host fp32 array (values representable in `dtype`) -> device tensor of that dtype."""
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(TORCH_DTYPE[dtype]).cuda()


def host(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> host float64 array (exact: every storage value is representable)."""
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def make_ctx(shape: synth.LayerShape, max_tokens: int, max_chunks: int, max_q: int, **kw) -> B.Context:
    return B.Context(shape.n_q_heads, shape.n_kv_heads, shape.head_dim, FR_DTYPE[shape.dtype], shape.rope_base,
                     max_tokens=max_tokens, max_chunks=max_chunks, max_question_tokens=max_q, **kw)

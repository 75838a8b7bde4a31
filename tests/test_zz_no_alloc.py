"""The selection entry point that allocates nothing (static scratch inside the library, no context) against the
context-based one and the oracle: two calls in a row on one GPU, the second with a smaller input, so that what the
first call left in the shared scratch must not matter."""
import numpy as np
import pytest
import torch

from oracle import fusionrag_oracle as orc
from paper_2601_12904_amd import binding as B
from paper_2601_12904_amd import synth
from tests import harness as H

pytestmark = pytest.mark.gpu


def _scores(rng, n, kind):
    if kind == "clustered":
        return (16.0 * np.exp(0.6 * rng.standard_normal(n))).astype(np.float32)
    if kind == "ties":
        return rng.integers(0, 8, size=n).astype(np.float32)
    return rng.standard_normal(n).astype(np.float32)


@pytest.mark.parametrize("kind", ["clustered", "ties", "signed"])
def test_static_scratch_selection_two_calls(kind):
    ctx = H.make_ctx(synth.TINY_F32, 4096, 4, 16)
    rng = np.random.default_rng(5)
    free_before = None
    for n, k, nq in [(700001, 105000, 7), (123457, 18519, 3), (40000, 39999, 0), (5000, 750, 2)]:   # second and later: smaller
        s = _scores(rng, n, kind)
        dev = torch.from_numpy(s).cuda()
        want_lib = torch.full((k + nq,), -7, dtype=torch.int32, device="cuda")
        got = torch.full((k + nq,), -9, dtype=torch.int32, device="cuda")
        ctx.fr_select_topk(dev, n, k, nq, want_lib)
        torch.cuda.synchronize()
        if free_before is None:
            free_before = torch.cuda.mem_get_info()[0]
        B.fr_select_topk_static(dev, n, k, nq, got)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free_before, "the call changed the amount of free device memory"
        assert torch.equal(got, want_lib), f"n = {n}: differs from fr_select_topk"
        assert np.array_equal(got.cpu().numpy(), orc.select_q_index(s, k, nq)), f"n = {n}: differs from the oracle"
        del dev, want_lib, got
        free_before = None
    # sizes beyond the static scratch are refused before anything is launched, with a message
    with pytest.raises(B.FusionRAGError) as ei:
        B.fr_select_topk_static(torch.zeros(8, device="cuda"), B.FR_SELECT_STATIC_MAX_SCORES + 1, 1, 0,
                                torch.zeros(8, dtype=torch.int32, device="cuda"), ctx=ctx)
    assert ei.value.status == B.FR_ERR_WORKSPACE and "FR_SELECT_STATIC_MAX_SCORES" in str(ei.value)
    ctx.close()

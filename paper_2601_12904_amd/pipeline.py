"""Asynchronous host-to-device load of the cached chunk K/V of the *next* request while the current request's
layers run (the asynchronous KVCache load the paper adds to its serving stack, Sec. 4.2; its share of the TTFT
saving is quoted in Sec. 5.3).  Plumbing only: pinned host buffers, one copy stream at the default priority,
events, and two device-side buffer sets that alternate between "being filled" and "being computed on".  Every
arithmetic step still runs in the library's kernels; the copies are plain asynchronous memory copies."""
from __future__ import annotations

from typing import Callable, List, Sequence

import torch


class HostKVRequest:
    """The cached K/V of one request's chunks as they sit in host memory: per layer one pinned tensor for the keys
    [L_ctx, Hkv, d] and one for the values."""

    def __init__(self, k_layers: Sequence[torch.Tensor], v_layers: Sequence[torch.Tensor]):
        assert len(k_layers) == len(v_layers)
        for t in list(k_layers) + list(v_layers):
            if not t.is_pinned():
                raise ValueError("host K/V must be allocated as pinned memory (torch.empty(..., pin_memory=True))")
        self.k_layers, self.v_layers = list(k_layers), list(v_layers)

    @property
    def nbytes(self) -> int:
        return sum(t.numel() * t.element_size() for t in self.k_layers + self.v_layers)


class DeviceKVSet:
    """Device buffers one request is loaded into: per layer the cached keys [L_ctx, Hkv, d] (input of the position
    shift) and the per-query cache pair [L, Hkv, d] whose first L_ctx value rows receive the cached values."""

    def __init__(self, n_layers: int, L_ctx: int, L: int, Hkv: int, d: int, dtype=torch.bfloat16):
        mk = lambda rows: [torch.zeros((rows, Hkv, d), dtype=dtype, device="cuda") for _ in range(n_layers)]
        self.k_cached, self.k_cache, self.v_cache = mk(L_ctx), mk(L), mk(L)
        self.L_ctx = L_ctx
        self.ready = torch.cuda.Event()      # recorded on the copy stream when the set is filled
        self.released = torch.cuda.Event()   # recorded on the compute stream when the set's request is finished
        self.released.record()


class AsyncKVPipeline:
    """Runs requests one after the other; with overlap=True the next request's K/V travel on the copy stream while
    the current request computes (two buffer sets), otherwise load and compute alternate on one stream."""

    def __init__(self, sets: List[DeviceKVSet]):
        assert len(sets) == 2
        self.sets = sets
        self.copy_stream = torch.cuda.Stream()   # default priority

    def _load(self, req: HostKVRequest, dst: DeviceKVSet):
        for l, (hk, hv) in enumerate(zip(req.k_layers, req.v_layers)):
            dst.k_cached[l].copy_(hk, non_blocking=True)
            dst.v_cache[l][: dst.L_ctx].copy_(hv, non_blocking=True)

    def run(self, requests: Sequence[HostKVRequest], compute: Callable[[int, DeviceKVSet], None], overlap: bool = True):
        """compute(i, set) enqueues request i's layers on the current stream, reading and writing `set`."""
        main = torch.cuda.current_stream()
        if not overlap:
            for i, req in enumerate(requests):
                self._load(req, self.sets[0])
                compute(i, self.sets[0])
            return
        def start_load(i):
            dst = self.sets[i % 2]
            self.copy_stream.wait_event(dst.released)      # its previous request is done with it
            with torch.cuda.stream(self.copy_stream):
                self._load(requests[i], dst)
                dst.ready.record(self.copy_stream)
        if requests:
            start_load(0)
        for i in range(len(requests)):
            if i + 1 < len(requests):
                start_load(i + 1)
            cur = self.sets[i % 2]
            main.wait_event(cur.ready)
            compute(i, cur)
            cur.released.record(main)

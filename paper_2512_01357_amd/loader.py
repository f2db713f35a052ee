"""Device memory and streams around the C ABI (PyTorch is plumbing here).

``ReusePool`` owns the slab (one torch uint8 tensor on the GPU), two streams
and the library's pool handle; every step of a load is a call into
libtangram.so through ``tangram.py``.
"""
from typing import Dict, List, Optional, Sequence, Tuple

import torch

from . import tangram as tg


class RegisteredModel:
    """A model in the CPU-side Model Cache: pinned bytes + per-tensor rows."""

    def __init__(self, model_id: int, host: torch.Tensor, offs: Sequence[int],
                 sizes: Sequence[int], fps: Sequence[int]):
        self.model_id = model_id
        self.host = host                       # keeps the pinned buffer alive
        self.offs = list(offs)
        self.sizes = list(sizes)
        self.fps = list(fps)
        self.desc = tg.ModelDesc(model_id, host.data_ptr(), host.numel(),
                                 list(zip(self.sizes, self.fps, self.offs)))

    @property
    def nbytes(self) -> int:
        return sum(self.sizes)


def fingerprint_host_buffer(host: torch.Tensor, offs: Sequence[int], sizes: Sequence[int],
                            stage_bytes: int = 2 << 30, stream=None,
                            device: str = "cuda:0") -> List[int]:
    """Fingerprints of tensors that live in a host buffer (registration time).

    The bytes are staged through a bounded device buffer in runs of
    consecutive tensors; each run is one host-to-device copy and one
    tg_fingerprint launch over the staged spans.
    """
    n = len(offs)
    fps = [0] * n
    order = sorted(range(n), key=lambda k: offs[k])
    cap = max(stage_bytes, max(sizes) if sizes else 0)
    cap = (cap + 255) // 256 * 256
    stage = torch.empty(cap + 256, dtype=torch.uint8, device=device)   # room for the phase
    i = 0
    while i < n:
        start = offs[order[i]]
        j = i
        end = start
        while j < n and offs[order[j]] + sizes[order[j]] - start <= cap:
            end = offs[order[j]] + sizes[order[j]]
            j += 1
        if j == i:
            raise ValueError("tensor larger than the staging buffer")
        # the run's first byte keeps its 16-byte phase inside the staging buffer
        phase = start % 16
        stage[phase:phase + end - start].copy_(host[start:end], non_blocking=False)
        spans = [(stage.data_ptr() + phase + offs[order[m]] - start, sizes[order[m]])
                 for m in range(i, j)]
        torch.cuda.synchronize()
        got = tg.tg_fingerprint(spans, stream)
        for m, f in zip(range(i, j), got):
            fps[order[m]] = f
        i = j
    del stage
    return fps


class ReusePool:
    """One Unified Memory Pool on one GPU, plus the streams a load runs on."""

    def __init__(self, capacity: int, align: int = 256, device: str = "cuda:0"):
        self.device = torch.device(device)
        self.capacity = capacity
        self.align = align
        self.slab = torch.empty(capacity, dtype=torch.uint8, device=self.device)
        if self.slab.data_ptr() % align:
            raise RuntimeError("slab is not aligned to %d" % align)
        self.stream_gather = torch.cuda.Stream(device=self.device)
        self.stream_h2d = torch.cuda.Stream(device=self.device)
        self.pool = tg.tg_pool_create(self.slab.data_ptr(), capacity, align)
        self.base = self.slab.data_ptr()

    def close(self) -> None:
        if self.pool is not None:
            tg.tg_pool_destroy(self.pool)
            self.pool = None
        self.slab = None

    def register(self, model_id: int, host: torch.Tensor, offs: Sequence[int],
                 sizes: Sequence[int], fps: Optional[Sequence[int]] = None,
                 stage_bytes: int = 2 << 30) -> RegisteredModel:
        if not host.is_pinned():
            raise ValueError("the Model Cache buffer must be pinned host memory")
        if fps is None:
            fps = fingerprint_host_buffer(host, offs, sizes, stage_bytes, self.stream_gather,
                                          str(self.device))
        return RegisteredModel(model_id, host, offs, sizes, fps)

    def load(self, model: RegisteredModel, confirm: bool = False, verify: bool = False
             ) -> Tuple[List[int], dict]:
        """tg_plan + tg_assemble.  Returns device addresses and the plan rows."""
        plan = tg.tg_plan(self.pool, model.desc, tg.TG_PLAN_CONFIRM if confirm else 0,
                          self.stream_gather)
        try:
            rows, reused, transfer = tg.tg_plan_ops(plan)
            ptrs = tg.tg_assemble(self.pool, plan, model.desc.n,
                                  tg.TG_ASSEMBLE_VERIFY if verify else 0,
                                  self.stream_gather, self.stream_h2d)
        finally:
            tg.tg_plan_free(plan)
        return ptrs, {"ops": rows, "reused_bytes": reused, "transfer_bytes": transfer}

    def release(self, model_id: int, evict: bool = False) -> None:
        tg.tg_release(self.pool, model_id, tg.TG_RELEASE_EVICT if evict else 0)

    def stats(self) -> dict:
        return tg.tg_pool_stats(self.pool)

    def view(self, ptr: int, nbytes: int) -> torch.Tensor:
        """The slab bytes at a returned address, as a uint8 device tensor."""
        off = ptr - self.base
        if off < 0 or off + nbytes > self.capacity:
            raise ValueError("address outside the pool")
        return self.slab[off:off + nbytes]

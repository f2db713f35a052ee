"""Runs a synthetic Workload (synth.py) through the library on one GPU."""
import time
from typing import Dict, List, Optional

import torch

from . import synth
from . import tangram as tg
from .loader import RegisteredModel, ReusePool


class WorkloadRunner:
    """Materialises a workload's models in pinned host memory (the Model
    Cache), registers them (GPU fingerprints) and replays its actions."""

    def __init__(self, w: synth.Workload, device: str = "cuda:0", gen_device: Optional[str] = None,
                 log=None):
        self.w = w
        self.device = device
        self.gen_device = gen_device or device
        self.log = log or (lambda *_: None)
        self.pool = ReusePool(w.pool_bytes, w.align, device)
        self.models: Dict[str, RegisteredModel] = {}
        self.host: Dict[str, torch.Tensor] = {}

    def materialise(self, name: str) -> RegisteredModel:
        if name in self.models:
            return self.models[name]
        spec = self.w.models[name]
        t0 = time.time()
        host = torch.empty(synth.host_bytes(spec, self.w.align), dtype=torch.uint8, pin_memory=True)
        offs = synth.fill_host(spec, host, self.gen_device, self.w.align)
        sizes = [t.nbytes for t in spec.tensors]
        reg = self.pool.register(spec.model_id, host, offs, sizes)
        self.models[name] = reg
        self.host[name] = host
        self.log("materialised %s: %d tensors, %.3f GB in %.1f s"
                 % (name, len(sizes), sum(sizes) / 1e9, time.time() - t0))
        return reg

    def drop_host(self, name: str) -> None:
        """Forget a model's host image (its resident tensors stay in the pool)."""
        self.models.pop(name, None)
        self.host.pop(name, None)

    def run_setup(self, keep_host: bool = True) -> None:
        for act in self.w.setup:
            if act[0] == "load":
                reg = self.materialise(act[1])
                self.pool.load(reg)
                self.log("setup: loaded %s" % act[1])
            else:
                _, name, evict = act
                self.pool.release(self.w.models[name].model_id, evict)
                if not keep_host:
                    self.drop_host(name)

    def load(self, name: str, confirm: bool = False, verify: bool = False):
        reg = self.materialise(name)
        return self.pool.load(reg, confirm=confirm, verify=verify)

    def release(self, name: str, evict: bool) -> None:
        self.pool.release(self.w.models[name].model_id, evict)

    def close(self) -> None:
        self.pool.close()
        self.models.clear()
        self.host.clear()

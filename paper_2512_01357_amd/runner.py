"""Runs a synthetic Workload (synth.py) through the library on one GPU."""
import contextlib
import time
from typing import Dict, List, Optional

import torch

from . import synth
from .loader import HostArena, RegisteredModel, ReusePool, refill_stream


class WorkloadRunner:
    """Materialises a workload's models in pinned host memory (the Model
    Cache), registers them (GPU fingerprints) and replays its actions.

    The measured models, and every setup model that shares tensors with them,
    live in one cache image in which equal tensors are stored once.  Other
    setup models (residents that only occupy the pool) get an image of their
    own that is freed as soon as they have been loaded.
    """

    def __init__(self, w: synth.Workload, device: str = "cuda:0", gen_device: Optional[str] = None,
                 log=None, arena_budget: int = 56 << 30, segment_bytes: int = 48 * 10**9):
        self.w = w
        self.arena_budget = arena_budget
        self.segment_bytes = segment_bytes
        self.seg_arena: Optional[HostArena] = None
        self.on_segment = None                  # hook(name, rows, arena): called whenever a segment has been filled
        self._fp_by_content: Dict[tuple, int] = {}
        self.device = device
        self.gen_device = gen_device or device
        self.log = log or (lambda *_: None)
        self.pool = ReusePool(w.pool_bytes, w.align, device)
        self.models: Dict[str, RegisteredModel] = {}
        self.arena: Optional[HostArena] = None
        self._main_names = self._pick_main()
        specs = [w.models[n] for n in self._main_names]
        if w.streamed or synth.shared_layout(specs, w.align)[0] > arena_budget:
            # too big to pin at once: every model gets a private image that
            # lives only while it is being loaded
            self._main_names = []
        self._main_offs: Dict[str, List[int]] = {}
        self._main_fps: Dict[int, int] = {}

    def _pick_main(self) -> List[str]:
        keys = set()
        for name in self.w.loads:
            keys.update(synth.content_key(t) for t in self.w.models[name].tensors if t.kind == "normal")
        names = []
        for act in self.w.setup:
            if act[0] != "load" or act[1] in names:
                continue
            if any(t.kind == "normal" and synth.content_key(t) in keys
                   for t in self.w.models[act[1]].tensors):
                names.append(act[1])
        return names + [n for n in self.w.loads if n not in names]

    def host_numpy(self, name: str):
        return self.models[name].host_tensor.numpy()

    # ------------------------------------------------------------------ models too large to pin
    def is_streamed(self, name: str) -> bool:
        """True for a model that does not fit the Model Cache: it is registered
        without a host image and loaded segment by segment."""
        return self.w.streamed and synth.host_bytes(self.w.models[name], self.w.align) > self.arena_budget

    def _segment_arena(self, need: int) -> HostArena:
        want = min(self.segment_bytes, need)
        if self.seg_arena is None or self.seg_arena.nbytes < want:
            if self.seg_arena is not None:
                self.seg_arena.free()
            t0 = time.time()
            self.seg_arena = HostArena(want)
            self.log("model cache segment: %.1f GB pinned in %.1f s" % (want / 1e9, time.time() - t0))
        return self.seg_arena

    def segments(self, name: str, parts: int = 1):
        """A generator factory for ReusePool.load_streamed: given tensor indices
        of model `name`, fills the pinned segment with as many of them as fit,
        in the given order, and yields (address, length, [(index, offset)]).
        With `parts` > 1 the segment is cut into that many equal buffers that
        are filled in turn, so that one can be filled while the copies out of
        another are still in flight."""
        spec = self.w.models[name]
        a = self.w.align

        def gen(ks):
            if not ks:
                return
            slot = [(spec.tensors[k].nbytes + a - 1) // a * a for k in ks]
            arena = self._segment_arena(max(sum(slot), a) if parts == 1 else self.segment_bytes)
            part = arena.nbytes if parts == 1 else arena.nbytes // parts // 4096 * 4096
            if max(slot) > part:
                raise RuntimeError("a tensor is larger than the Model Cache segment")
            # filling one part while another is being copied to the GPU: the tensors are made and
            # copied to the host on a stream that runs beside the load's transfer streams
            side = refill_stream(self.pool.device)[0] if parts > 1 else None
            i = n_yielded = 0
            while i < len(ks):
                base = (n_yielded % parts) * part
                rows, at = [], 0
                with torch.cuda.stream(side) if side is not None else contextlib.nullcontext():
                    while i < len(ks) and at + slot[i] <= part:
                        t = spec.tensors[ks[i]]
                        arena.tensor[base + at:base + at + t.nbytes].copy_(synth.tensor_bytes(t, self.gen_device))
                        rows.append((ks[i], at))
                        at += slot[i]
                        i += 1
                if self.on_segment is not None:
                    self.on_segment(name, [(k, base + off) for k, off in rows], arena)
                yield arena.ptr + base, at, rows
                n_yielded += 1
        return gen

    def _register_streamed(self, name: str) -> RegisteredModel:
        """Fingerprints of a model that passes through the segment piece by
        piece: each piece is fingerprinted where it lies, in pinned host memory,
        through its device mapping (tensors whose content was fingerprinted
        before -- a sibling's -- are not read again)."""
        from . import tangram as tg
        spec = self.w.models[name]
        t0 = time.time()
        fps = [self._fp_by_content.get(synth.content_key(t)) for t in spec.tensors]
        todo = [k for k, f in enumerate(fps) if f is None]
        for ptr, _n, rows in self.segments(name)(todo):
            dev = tg.tg_host_device_ptr(ptr)
            got = tg.tg_fingerprint([(dev + off, spec.tensors[k].nbytes) for k, off in rows], self.pool.stream_gather)
            for (k, _off), f in zip(rows, got):
                fps[k] = f
                self._fp_by_content[synth.content_key(spec.tensors[k])] = f
        sizes = [t.nbytes for t in spec.tensors]
        reg = RegisteredModel(spec.model_id, None, synth.layout(spec, self.w.align), sizes, fps)
        self.models[name] = reg
        self.log("registered %s: %d tensors, %.3f GB (%d fingerprinted over the host link) in %.1f s"
                 % (name, len(sizes), sum(sizes) / 1e9, len(todo), time.time() - t0))
        return reg

    def _build_main(self) -> None:
        t0 = time.time()
        specs = [self.w.models[n] for n in self._main_names]
        total, per_model, unique = synth.shared_layout(specs, self.w.align)
        self.arena = HostArena(total)
        for t, off in unique:
            self.arena.tensor[off:off + t.nbytes].copy_(synth.tensor_bytes(t, self.gen_device))
        # fingerprint every unique tensor once, then hand each model its rows
        u_offs = [off for _, off in unique]
        u_sizes = [t.nbytes for t, _ in unique]
        u_fps = self.pool.register(0, self.arena, u_offs, u_sizes).fps
        by_off = dict(zip(u_offs, u_fps))
        for spec in specs:
            offs = per_model[spec.name]
            sizes = [t.nbytes for t in spec.tensors]
            fps = [by_off[o] for o in offs]
            self.models[spec.name] = RegisteredModel(spec.model_id, self.arena, offs, sizes, fps)
        self.log("model cache: %s in one image of %.3f GB (%d unique tensors) in %.1f s"
                 % (",".join(self._main_names), total / 1e9, len(unique), time.time() - t0))

    def materialise(self, name: str) -> RegisteredModel:
        if name in self.models:
            return self.models[name]
        if name in self._main_names:
            self._build_main()
            return self.models[name]
        if self.is_streamed(name):
            return self._register_streamed(name)
        spec = self.w.models[name]
        t0 = time.time()
        host = HostArena(synth.host_bytes(spec, self.w.align))
        offs = synth.fill_host(spec, host.tensor, self.gen_device, self.w.align)
        sizes = [t.nbytes for t in spec.tensors]
        reg = self.pool.register(spec.model_id, host, offs, sizes)
        self.models[name] = reg
        self.log("materialised %s: %d tensors, %.3f GB in %.1f s"
                 % (name, len(sizes), sum(sizes) / 1e9, time.time() - t0))
        return reg

    def drop_host(self, name: str) -> None:
        """Forget a model's private host image (its tensors stay in the pool)."""
        if name in self._main_names:
            return
        if name in self.models and self.models[name].host is None:
            return                               # rows only: nothing to free
        reg = self.models.pop(name, None)
        if reg is not None and isinstance(reg.host, HostArena):
            reg.host_tensor = None
            reg.host.free()

    def run_setup(self) -> None:
        for act in self.w.setup:
            if act[0] == "load":
                self.load(act[1], details=False)
                self.log("setup: loaded %s" % act[1])
                self.drop_host(act[1])
            else:
                _, name, evict = act
                self.pool.release(self.w.models[name].model_id, evict)
        for name, (p, b, a) in self.w.costs.items():
            self.pool.set_model_cost(self.w.models[name].model_id, p, b, a)

    def load(self, name: str, confirm: bool = False, verify: bool = False, details: bool = True,
             overlap: bool = False, **flags):
        """Loads a model; plan flags default to the workload's for its measured loads.
        `overlap` (models that pass through the Model Cache in pieces): the cache is cut into
        two halves and one is refilled while the other is being copied to the GPU."""
        reg = self.materialise(name)
        if not flags and name in self.w.loads:
            flags = dict(self.w.load_flags)
        if reg.host is None:
            if confirm:
                raise ValueError("confirmation needs the model's whole host image")
            return self.pool.load_streamed(reg, self.segments(name, 2 if overlap else 1), verify=verify,
                                           details=details, overlap=overlap, **flags)
        return self.pool.load(reg, confirm=confirm, verify=verify, details=details, **flags)

    def reset_pool(self) -> None:
        """Evict everything and replay the setup (for workloads whose measured
        load moves or evicts residents)."""
        for spec in self.w.models.values():
            try:
                self.pool.release(spec.model_id, True)
            except Exception:
                pass
        self.run_setup()

    def release(self, name: str, evict: bool) -> None:
        self.pool.release(self.w.models[name].model_id, evict)

    def close(self) -> None:
        self.pool.close()
        for reg in self.models.values():
            reg.host_tensor = None
        self.models.clear()
        if self.arena is not None:
            self.arena.free()
            self.arena = None
        if self.seg_arena is not None:
            self.seg_arena.free()
            self.seg_arena = None

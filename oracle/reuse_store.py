"""Reuse Store bookkeeping as plain Python (oracle, test infrastructure).

Follows the paper's Section 3.1 (Tensor Mapping lookup, load what is missing,
update the mapping, return every tensor's address) and Section 3.2 (Region
List of free / allocated regions in physical order, best-fit allocation that
leaves a smaller free region behind).  Every decision is one linear scan over
a Python list so it can be checked against the text by eye.

Readings taken where the paper is silent (the same ones the product documents):
  * the mapping key is (fingerprint, nbytes); among several resident tensors
    with an equal key the one at the lowest pool offset is the source;
  * incoming tensors are matched against the tensors resident when planning
    starts, never against each other;
  * every incoming tensor gets a fresh slot -- a hit is copied device to
    device from the resident tensor, a miss is transferred from host memory;
  * slots are rounded up to the pool alignment; tensors are placed in order
    of descending rounded size (ties: ascending index), each into the smallest
    free region that holds it (ties: lowest offset), at the region's low end;
  * if any tensor cannot be placed the plan fails and nothing changes.
"""
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from .cbytes import bytes_equal, copy_bytes

REUSE = 0
H2D = 1


class NoSpace(Exception):
    """Best-fit could not place every tensor of the incoming model."""


class StalePlan(Exception):
    """The pool changed between planning and assembly."""


@dataclass
class Entry:
    """One row of the Tensor Mapping."""
    off: int
    nbytes: int
    fp: int
    model_id: int
    active: bool


@dataclass
class PlanOp:
    kind: int       # REUSE or H2D
    dst_off: int    # slot in the pool
    src_off: int    # REUSE: pool offset of the resident copy; H2D: host offset
    nbytes: int


@dataclass
class OraclePlan:
    model_id: int
    ops: List[PlanOp]
    fps: List[int]
    reused_bytes: int
    transfer_bytes: int
    generation: int
    regions_after: List[List] = field(default_factory=list)


def round_up(n: int, a: int) -> int:
    return (n + a - 1) // a * a


class ReuseStoreOracle:
    """Unified Memory Pool + Region List + Tensor Mapping for one GPU.

    ``image`` maps a slot's pool offset to the bytes stored there (a sparse
    picture of the pool: only tensor slots hold defined bytes).  It is kept
    only when the caller supplies host bytes; with ``host=None`` the store
    tracks metadata alone, which is all that planning needs.
    """

    def __init__(self, capacity: int, align: int = 256):
        if align < 16 or align & (align - 1):
            raise ValueError("align must be a power of two >= 16")
        if capacity <= 0 or capacity % align:
            raise ValueError("capacity must be a positive multiple of align")
        self.capacity = capacity
        self.align = align
        # Region List: [offset, length, is_free], in physical order, tiling
        # [0, capacity) exactly.
        self.regions: List[List] = [[0, capacity, True]]
        self.entries: List[Entry] = []
        self.image: Dict[int, np.ndarray] = {}
        self.generation = 0

    # ------------------------------------------------------------------ match
    def _match(self, nbytes: int, fp: int, incoming: Optional[np.ndarray],
               confirm: bool) -> Optional[int]:
        """Pool offset of the resident tensor to reuse, or None (a miss)."""
        best = None
        for e in self.entries:
            if e.fp != fp or e.nbytes != nbytes:
                continue
            if confirm:
                if incoming is None or e.off not in self.image:
                    raise ValueError("confirm needs bytes on both sides")
                if not bytes_equal(self.image[e.off], incoming):
                    continue
            if best is None or e.off < best:
                best = e.off
        return best

    # --------------------------------------------------------------- allocate
    @staticmethod
    def _best_fit(regions: List[List], need: int) -> Optional[int]:
        """Index of the smallest free region with length >= need."""
        pick = None
        for i, (off, length, free) in enumerate(regions):
            if not free or length < need:
                continue
            if pick is None or length < regions[pick][1]:
                pick = i           # strictly smaller only: ties keep low offset
        return pick

    def plan(self, model_id: int, tensors: Sequence[Tuple[int, int, int]],
             host: Optional[np.ndarray] = None, confirm: bool = False
             ) -> OraclePlan:
        """``tensors[k] = (nbytes, fp, host_off)``.  Pure: the store is not
        modified; the result records the Region List the commit will install."""
        for e in self.entries:
            if e.model_id == model_id and e.active:
                raise ValueError("model is already active in this pool")
        for nbytes, _fp, off in tensors:
            if nbytes <= 0:
                raise ValueError("zero-length tensor")
            if host is not None and off + nbytes > host.size:
                raise ValueError("tensor exceeds the host buffer")

        kinds: List[int] = []
        srcs: List[int] = []
        for nbytes, fp, off in tensors:
            incoming = None if host is None else host[off:off + nbytes]
            hit = self._match(nbytes, fp, incoming, confirm)
            if hit is None:
                kinds.append(H2D)
                srcs.append(off)
            else:
                kinds.append(REUSE)
                srcs.append(hit)

        order = sorted(range(len(tensors)),
                       key=lambda k: (-round_up(tensors[k][0], self.align), k))
        regions = [list(r) for r in self.regions]
        dsts = [0] * len(tensors)
        for k in order:
            need = round_up(tensors[k][0], self.align)
            i = self._best_fit(regions, need)
            if i is None:
                raise NoSpace("no free region of %d bytes for tensor %d"
                              % (need, k))
            off, length, _ = regions[i]
            dsts[k] = off
            taken = [off, need, False]
            if length == need:
                regions[i] = taken
            else:
                regions[i] = [off + need, length - need, True]
                regions.insert(i, taken)

        ops = [PlanOp(kinds[k], dsts[k], srcs[k], tensors[k][0])
               for k in range(len(tensors))]
        reused = sum(op.nbytes for op in ops if op.kind == REUSE)
        transfer = sum(op.nbytes for op in ops if op.kind == H2D)
        return OraclePlan(model_id, ops, [t[1] for t in tensors], reused,
                          transfer, self.generation, regions)

    # --------------------------------------------------------------- assemble
    def assemble(self, plan: OraclePlan, host: Optional[np.ndarray] = None
                 ) -> List[int]:
        """Fill every slot, then record the new tensors in the mapping and the
        Region List.  Returns the pool offset of every tensor, in index order."""
        if plan.generation != self.generation:
            raise StalePlan()
        if host is not None:
            for op in plan.ops:
                slot = np.empty(op.nbytes, dtype=np.uint8)
                if op.kind == REUSE:
                    copy_bytes(slot, self.image[op.src_off][:op.nbytes])
                else:
                    copy_bytes(slot, host[op.src_off:op.src_off + op.nbytes])
                self.image[op.dst_off] = slot
        self.regions = [list(r) for r in plan.regions_after]
        for op, fp in zip(plan.ops, plan.fps):
            self.entries.append(Entry(op.dst_off, op.nbytes, fp,
                                      plan.model_id, True))
        self.generation += 1
        return [op.dst_off for op in plan.ops]

    # ---------------------------------------------------------------- release
    def release(self, model_id: int, evict: bool = False) -> None:
        """Without ``evict`` the model's tensors stay resident and matchable
        but are marked inactive (the paper's "inactive but resident" state,
        Section 3.1); with it their regions are freed and merged with free
        neighbours."""
        mine = [e for e in self.entries if e.model_id == model_id]
        if not mine:
            raise KeyError(model_id)
        if not evict:
            for e in mine:
                e.active = False
        else:
            for e in mine:
                self._free_region(e.off)
                self.image.pop(e.off, None)
            self.entries = [e for e in self.entries if e.model_id != model_id]
        self.generation += 1

    def _free_region(self, off: int) -> None:
        for i, r in enumerate(self.regions):
            if r[0] == off and not r[2]:
                r[2] = True
                # merge with the next region, then with the previous one
                if i + 1 < len(self.regions) and self.regions[i + 1][2]:
                    r[1] += self.regions[i + 1][1]
                    del self.regions[i + 1]
                if i > 0 and self.regions[i - 1][2]:
                    self.regions[i - 1][1] += r[1]
                    del self.regions[i]
                return
        raise AssertionError("no allocated region at offset %d" % off)

    # ------------------------------------------------------------------ stats
    def stats(self) -> Dict[str, int]:
        free = [r[1] for r in self.regions if r[2]]
        return {
            "capacity": self.capacity,
            "free_bytes": sum(free),
            "largest_free": max(free) if free else 0,
            "n_regions": len(self.regions),
            "n_free_regions": len(free),
            "n_entries": len(self.entries),
            "n_active": sum(1 for e in self.entries if e.active),
        }

    def reuse_size(self, tensors: Sequence[Tuple[int, int, int]]) -> int:
        """Bytes of the model already resident (S' in the load-time estimate,
        Eq. 3 of the paper): sum of nbytes over tensors whose key is found."""
        total = 0
        for nbytes, fp, _off in tensors:
            if self._match(nbytes, fp, None, False) is not None:
                total += nbytes
        return total

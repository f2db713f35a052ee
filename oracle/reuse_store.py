"""Reuse Store bookkeeping as plain Python (oracle, test infrastructure).

Follows the paper's Section 3.1 (Tensor Mapping lookup, load what is missing,
update the mapping, return every tensor's address), Section 3.2 (Region List
of free / allocated regions in physical order, best-fit allocation; Stage 1
minimal-cost eviction, Eq. 2; Stage 2 Partitioned-Gain Packing, Algorithm 1)
and Eq. 3 (load-time estimate).  Every decision is a linear scan over Python
lists so it can be checked against the text by eye.

Readings taken where the paper is silent or at odds with itself (the same
ones the product documents):
  * the mapping key is (fingerprint, nbytes); among several resident tensors
    with an equal key the one at the lowest pool offset is the source;
  * incoming tensors are matched against the tensors resident when planning
    starts, never against each other;
  * default mode: every incoming tensor gets a fresh slot -- a hit is copied
    device to device from the resident tensor, a miss is transferred from
    host memory.  Alias mode (the paper's own design, Section 3.1): a hit is
    used where it lies, only misses get slots;
  * slots are rounded up to the pool alignment; tensors are placed in order
    of descending rounded size (ties: ascending index), each into the smallest
    free region that holds it (ties: lowest offset), at the region's low end;
  * Stage 1 runs only when the free bytes are fewer than the bytes to place;
    only tensors no running model uses, and that the plan itself does not
    read, can be evicted; ties in cost go to the lower offset; a tensor that
    several models own costs the sum of its owners' costs;
  * Stage 2 runs only when plain best fit fails.  A subspace's capacity for
    new tensors is its free bytes; the text counts allocated bytes too, which
    can hand a subspace more than it holds after merging -- that reading is
    available as ``cap_text`` and makes the plan fail when it happens.
    Partition points are tried in order of descending gain (ties: lower
    offset).  The packing test is the listing's: a tensor must be smaller than
    the smaller bin's remaining capacity, and goes to the bin with more room
    (ties: the first); the text words the test differently (the tensor only
    has to fit the bin with more room), which is available as ``pack_text``.
    Regions in use by a running model cannot move: they cut the pool into
    subspaces that cannot be merged with each other, and the tensors are dealt
    over those by the text's packing rule (largest remaining space first)
    before Algorithm 1 runs inside each.  The merge cost reported is the sum of
    the allocated bytes inside the final subspaces that were given tensors;
    the listing's running M also keeps counting regions that have dropped out
    of every subspace.  A final subspace first tries plain best fit inside
    itself and is compacted towards its low end only if that fails;
  * if the tensors cannot be placed the plan fails and nothing changes.
"""
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from .cbytes import bytes_equal, copy_bytes

REUSE = 0
H2D = 1


class NoSpace(Exception):
    """The tensors of the incoming model cannot be placed."""


class StalePlan(Exception):
    """The pool changed between planning and assembly."""


@dataclass(eq=False)
class Entry:
    """One row of the Tensor Mapping."""
    off: int
    nbytes: int
    fp: int
    owners: List[int]          # models that list this tensor, oldest first
    active_refs: int = 0       # how many running models use it

    @property
    def active(self) -> bool:
        return self.active_refs > 0

    @property
    def model_id(self) -> int:
        return self.owners[0]


@dataclass
class PlanOp:
    kind: int       # REUSE or H2D
    dst_off: int    # where the tensor will be (alias mode, hit: where it already is)
    src_off: int    # REUSE: pool offset of the resident copy at copy time; H2D: host offset
    nbytes: int


@dataclass
class OraclePlan:
    model_id: int
    ops: List[PlanOp]
    fps: List[int]
    reused_bytes: int
    transfer_bytes: int
    generation: int
    alias: bool = False
    regions_after: List[List] = field(default_factory=list)
    hits: List[Optional[Entry]] = field(default_factory=list)
    evictions: List[Entry] = field(default_factory=list)      # in eviction order
    moves: List[Tuple[Entry, int, int]] = field(default_factory=list)  # (entry, old, new), execution order
    merge_bound: int = 0       # Algorithm 1's M when Stage 2 ran, else 0
    moved_bytes: int = 0       # bytes of the tensors that really move
    evicted_bytes: int = 0


def round_up(n: int, a: int) -> int:
    return (n + a - 1) // a * a


# ------------------------------------------------------------ Region List ops
def best_fit(regions: List[List], need: int, lo: int = 0, hi: Optional[int] = None) -> Optional[int]:
    """Index of the smallest free region with length >= need among
    regions[lo:hi] (Section 3.2); ties keep the lowest offset."""
    pick = None
    hi = len(regions) if hi is None else hi
    for i in range(lo, hi):
        _off, length, free = regions[i][:3]
        if not free or length < need:
            continue
        if pick is None or length < regions[pick][1]:
            pick = i
    return pick


def carve(regions: List[List], i: int, need: int, tag=None) -> int:
    """Allocate `need` bytes at the low end of free region i; what is left
    stays free (Section 3.2).  Returns the offset."""
    off, length, _free, _tag = regions[i]
    taken = [off, need, False, tag]
    if length == need:
        regions[i] = taken
    else:
        regions[i] = [off + need, length - need, True, None]
        regions.insert(i, taken)
    return off


def free_at(regions: List[List], off: int) -> None:
    """Free the allocated region at `off` and merge it with free neighbours."""
    for i, r in enumerate(regions):
        if r[0] == off and not r[2]:
            r[2] = True
            r[3] = None
            if i + 1 < len(regions) and regions[i + 1][2]:
                r[1] += regions[i + 1][1]
                del regions[i + 1]
            if i > 0 and regions[i - 1][2]:
                regions[i - 1][1] += r[1]
                del regions[i]
            return
    raise AssertionError("no allocated region at offset %d" % off)


# --------------------------------------------------------------- Algorithm 1
def try_packing(sizes: Sequence[int], tensors: List[int], c1: int, c2: int
                ) -> Tuple[List[int], List[int]]:
    """TryPacking of Algorithm 1: tensors (already in descending size) go one
    by one to the bin with more remaining capacity; the attempt fails as soon
    as a tensor is not smaller than the smaller remaining capacity."""
    t1: List[int] = []
    t2: List[int] = []
    for k in tensors:
        if sizes[k] >= min(c1, c2):
            return [], []
        if c1 >= c2:
            t1.append(k)
            c1 -= sizes[k]
        else:
            t2.append(k)
            c2 -= sizes[k]
    return t1, t2


def try_packing_text(sizes: Sequence[int], tensors: List[int], c1: int, c2: int
                     ) -> Tuple[List[int], List[int]]:
    """TryPacking as the text of Section 3.2 words it (the listing and the text
    differ): a tensor goes to the bin with the largest remaining space (ties:
    the first) and the attempt fails only if it does not fit into that bin."""
    bins = ([], [])
    room = [c1, c2]
    for k in tensors:
        b = 0 if room[0] >= room[1] else 1
        if sizes[k] > room[b]:
            return [], []
        bins[b].append(k)
        room[b] -= sizes[k]
    return bins


def subspace(regions: List[List], lo: int, hi: int) -> Optional[Tuple[int, int]]:
    """The subspace inside regions[lo:hi]: the longest run that begins and ends
    with a free region (Section 3.2, "Partitioning subspaces"), or None."""
    free = [i for i in range(lo, hi) if regions[i][2]]
    return (free[0], free[-1] + 1) if free else None


def free_bytes(regions: List[List], sub: Tuple[int, int]) -> int:
    return sum(r[1] for r in regions[sub[0]:sub[1]] if r[2])


def allocated_bytes(regions: List[List], sub: Tuple[int, int]) -> int:
    """A subspace's maximum merge cost M: the bytes of its allocated regions."""
    return sum(r[1] for r in regions[sub[0]:sub[1]] if not r[2])


def capacity(regions: List[List], sub: Optional[Tuple[int, int]], as_printed: bool) -> int:
    """What a subspace can take of new tensors.  The text defines C as free plus
    allocated bytes (`as_printed`); the allocated regions stay where they are
    or move inside the subspace, so only the free bytes can really be handed
    out, and that is the default here."""
    if sub is None:
        return 0
    return free_bytes(regions, sub) + (allocated_bytes(regions, sub) if as_printed else 0)


def partitioned_gain_packing(regions: List[List], pairs: List[Tuple[Tuple[int, int], List[int]]],
                             sizes: Sequence[int], pack=try_packing, cap_as_printed: bool = False
                             ) -> Tuple[List[Tuple[Tuple[int, int], List[int]]], int]:
    """Algorithm 1.  `pairs` is the pending set P to start from -- (subspace,
    tensor subset) pairs, each subset in descending size; the listing starts
    with the single pair (R, T).  Returns (allocation set A in address order,
    the listing's running merge cost M: all allocated bytes of the starting
    subspaces minus the size of every partition point taken)."""
    pending = list(pairs)
    m = sum(allocated_bytes(regions, sub) for sub, _t in pending)
    done: List[Tuple[Tuple[int, int], List[int]]] = []
    while pending:
        nxt: List[Tuple[Tuple[int, int], List[int]]] = []
        for sub, tensors in pending:
            points = [i for i in range(sub[0], sub[1]) if not regions[i][2]]
            # partition gain = the point's size; the largest gain is tried first (ties: lower offset)
            points.sort(key=lambda i: (-regions[i][1], regions[i][0]))
            split_occurred = False
            for p in points:
                p1, p2 = subspace(regions, sub[0], p), subspace(regions, p + 1, sub[1])
                t1, t2 = pack(sizes, tensors, capacity(regions, p1, cap_as_printed),
                              capacity(regions, p2, cap_as_printed))
                if t1 or t2:
                    split_occurred = True
                    nxt += [(p1, t1), (p2, t2)]
                    m -= regions[p][1]
                    break
            if not split_occurred:
                done.append((sub, tensors))
        pending = nxt
    done.sort(key=lambda st: st[0][0])
    return done, m


def stretches(regions: List[List], movable) -> List[Tuple[int, int]]:
    """The pool cut at every allocated region that may not move (tensors of
    running models): the subspaces between them, in address order.  Algorithm 1
    assumes every resident tensor may move; this is what is left of its
    starting subspace R when some may not."""
    out = []
    lo = 0
    for i, r in enumerate(regions + [None]):
        if r is None or (not r[2] and not movable(r)):
            sub = subspace(regions, lo, i)
            if sub is not None:
                out.append(sub)
            lo = i + 1
    return out


def deal_over_stretches(regions: List[List], subs: List[Tuple[int, int]], sizes: Sequence[int],
                        order: List[int], cap_as_printed: bool) -> Optional[List[List[int]]]:
    """The new tensors (descending size) over several subspaces that cannot be
    merged with each other: each goes to the subspace with the largest
    remaining space (ties: lowest address) -- the packing rule of Section 3.2
    with as many bins as there are subspaces -- and None if one does not fit."""
    room = [capacity(regions, sub, cap_as_printed) for sub in subs]
    subsets: List[List[int]] = [[] for _ in subs]
    for k in order:
        if not room:
            return None
        b = max(range(len(room)), key=lambda i: (room[i], -i))
        if sizes[k] > room[b]:
            return None
        subsets[b].append(k)
        room[b] -= sizes[k]
    return subsets


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
        # Region List: [offset, length, is_free, entry], in physical order,
        # tiling [0, capacity) exactly.
        self._regions: List[List] = [[0, capacity, True, None]]
        self.entries: List[Entry] = []
        # model id -> {"active", "current" (entries the running instance uses), "owned"}
        self.models: Dict[int, Dict] = {}
        self.cost_params: Dict[int, Tuple[float, float, float]] = {}
        self.image: Dict[int, np.ndarray] = {}
        self.generation = 0

    @property
    def regions(self) -> List[List]:
        """[offset, length, is_free] rows."""
        return [r[:3] for r in self._regions]

    # ------------------------------------------------------------------ cost
    def set_model_cost(self, model_id: int, miss_prob: float, load_bw: float, alpha: float = 1.0) -> None:
        if not (miss_prob >= 0.0 and load_bw > 0.0 and alpha >= 0.0):
            raise ValueError("bad cost parameters")
        self.cost_params[model_id] = (float(miss_prob), float(load_bw), float(alpha))

    def eviction_cost(self, e: Entry) -> float:
        """Eq. 2: c_j = p_m * (s'_j / b_m) * alpha_m, summed over the models
        that own the tensor (defaults p = b = alpha = 1)."""
        total = 0.0
        for m in e.owners:
            p, b, a = self.cost_params.get(m, (1.0, 1.0, 1.0))
            total += p * (float(e.nbytes) / b) * a
        return total

    # ------------------------------------------------------------------ match
    def _match(self, nbytes: int, fp: int, incoming: Optional[np.ndarray],
               confirm: bool) -> Optional[Entry]:
        """The resident tensor to reuse, or None (a miss)."""
        best = None
        for e in self.entries:
            if e.fp != fp or e.nbytes != nbytes:
                continue
            if confirm:
                if incoming is None or e.off not in self.image:
                    raise ValueError("confirm needs bytes on both sides")
                if not bytes_equal(self.image[e.off], incoming):
                    continue
            if best is None or e.off < best.off:
                best = e
        return best

    # ------------------------------------------------------------------- plan
    def plan(self, model_id: int, tensors: Sequence[Tuple[int, int, int]],
             host: Optional[np.ndarray] = None, confirm: bool = False, evict: bool = False,
             merge: bool = False, alias: bool = False, pack_text: bool = False,
             cap_text: bool = False) -> OraclePlan:
        """``tensors[k] = (nbytes, fp, host_off)``.  Pure: the store is not
        modified; the result records everything the commit will install."""
        if model_id in self.models and self.models[model_id]["active"]:
            raise ValueError("model is already active in this pool")
        if not tensors:
            raise ValueError("empty model")
        for nbytes, _fp, off in tensors:
            if nbytes <= 0:
                raise ValueError("zero-length tensor")
            if host is not None and off + nbytes > host.size:
                raise ValueError("tensor exceeds the host buffer")

        n = len(tensors)
        hits: List[Optional[Entry]] = []
        for nbytes, fp, off in tensors:
            incoming = None if host is None else host[off:off + nbytes]
            hits.append(self._match(nbytes, fp, incoming, confirm))

        sizes = [round_up(t[0], self.align) for t in tensors]
        needs_slot = [k for k in range(n) if not (alias and hits[k] is not None)]
        order = sorted(needs_slot, key=lambda k: (-sizes[k], k))
        need_total = sum(sizes[k] for k in needs_slot)
        regions = [list(r) for r in self._regions]

        # ---- Stage 1: minimal-cost eviction (Section 3.2, Eq. 2)
        evictions: List[Entry] = []
        free_now = sum(r[1] for r in regions if r[2])
        if evict and free_now < need_total:
            protected = [h for h in hits if h is not None]
            cands = [e for e in self.entries
                     if e.active_refs == 0 and not any(e is p for p in protected)]
            cands.sort(key=lambda e: (self.eviction_cost(e), e.off))   # ascending cost
            for e in cands:
                if free_now >= need_total:
                    break
                free_at(regions, e.off)
                free_now += round_up(e.nbytes, self.align)
                evictions.append(e)
        if free_now < need_total:
            raise NoSpace("free bytes %d < needed %d" % (free_now, need_total))

        # ---- best fit (Section 3.2)
        dsts: Dict[int, int] = {}
        moves: List[Tuple[Entry, int, int]] = []
        merge_bound = 0
        trial = [list(r) for r in regions]
        ok = True
        for k in order:
            i = best_fit(trial, sizes[k])
            if i is None:
                ok = False
                break
            dsts[k] = carve(trial, i, sizes[k], ("new", k))
        if ok:
            regions = trial
        elif not merge:
            raise NoSpace("fragmented: best fit cannot place every tensor")
        else:
            # ---- Stage 2: Partitioned-Gain Packing (Algorithm 1)
            dsts = {}
            subs = stretches(regions, lambda r: r[3].active_refs == 0)
            subsets = deal_over_stretches(regions, subs, sizes, order, cap_text)
            if subsets is None:
                raise NoSpace("running models' tensors separate the free space")
            final, _m_listing = partitioned_gain_packing(
                regions, list(zip(subs, subsets)), sizes,
                try_packing_text if pack_text else try_packing, cap_text)
            # Only subspaces that were given tensors can have anything merged in them.
            final = [(sub, subset) for sub, subset in final if subset]
            merge_bound = sum(allocated_bytes(regions, sub) for sub, _t in final)
            for sub, subset in final:
                if sum(sizes[k] for k in subset) > free_bytes(regions, sub):
                    # only with the capacity as printed: allocated bytes were counted as room
                    raise NoSpace("a subspace was handed more than its free bytes")
            # realise the subspaces from the high end down so list indices stay valid
            realised = []
            for (lo, hi), subset in reversed(final):
                part = [list(r) for r in regions[lo:hi]]
                sub_moves: List[Tuple[Entry, int, int]] = []
                sub_dsts: Dict[int, int] = {}
                trial = [list(r) for r in part]
                fits = True
                for k in subset:
                    i = best_fit(trial, sizes[k])
                    if i is None:
                        fits = False
                        break
                    sub_dsts[k] = carve(trial, i, sizes[k], ("new", k))
                if fits:
                    part = trial
                else:
                    # merge: slide every allocated region to the low end, in
                    # address order, then place the tensors in the free tail
                    start = part[0][0]
                    end = part[-1][0] + part[-1][1]
                    at = start
                    packed = []
                    for r in part:
                        if r[2]:
                            continue
                        if r[0] != at:
                            sub_moves.append((r[3], r[0], at))
                        packed.append([at, r[1], False, r[3]])
                        at += r[1]
                    sub_dsts = {}
                    for k in subset:
                        sub_dsts[k] = at
                        packed.append([at, sizes[k], False, ("new", k)])
                        at += sizes[k]
                    if at > end:
                        raise AssertionError("subspace over-committed")
                    if at < end:
                        packed.append([at, end - at, True, None])
                    part = packed
                regions[lo:hi] = part
                realised.append((sub_moves, sub_dsts))
            for sub_moves, sub_dsts in reversed(realised):      # address order
                moves += sub_moves
                dsts.update(sub_dsts)

        moved_to = {id(e): new for e, _old, new in moves}
        ops: List[PlanOp] = []
        for k, (nbytes, _fp, off) in enumerate(tensors):
            h = hits[k]
            if h is None:
                ops.append(PlanOp(H2D, dsts[k], off, nbytes))
            else:
                where = moved_to.get(id(h), h.off)
                ops.append(PlanOp(REUSE, where if alias else dsts[k], where, nbytes))
        reused = sum(op.nbytes for op in ops if op.kind == REUSE)
        transfer = sum(op.nbytes for op in ops if op.kind == H2D)
        return OraclePlan(model_id, ops, [t[1] for t in tensors], reused, transfer,
                          self.generation, alias, regions, hits, evictions, moves, merge_bound,
                          sum(e.nbytes for e, _o, _n in moves),
                          sum(round_up(e.nbytes, self.align) for e in evictions))

    # --------------------------------------------------------------- assemble
    def assemble(self, plan: OraclePlan, host: Optional[np.ndarray] = None) -> List[int]:
        """Evict, move, fill every slot, then record the new tensors in the
        mapping and the Region List.  Returns the pool offset of every tensor,
        in index order."""
        if plan.generation != self.generation:
            raise StalePlan()
        for e in plan.evictions:
            self._drop_entry(e)
        # tensors that move keep their bytes (moves run before any slot is filled)
        carried = {}
        for e, old, _new in plan.moves:
            if old in self.image:
                carried[id(e)] = self.image.pop(old)
        for e, _old, new in plan.moves:
            e.off = new
            if id(e) in carried:
                self.image[new] = carried[id(e)]
        if host is not None:
            for op, hit in zip(plan.ops, plan.hits):
                if plan.alias and hit is not None:
                    continue
                slot = np.empty(op.nbytes, dtype=np.uint8)
                if op.kind == REUSE:
                    copy_bytes(slot, self.image[op.src_off][:op.nbytes])
                else:
                    copy_bytes(slot, host[op.src_off:op.src_off + op.nbytes])
                self.image[op.dst_off] = slot
        self._regions = [list(r) for r in plan.regions_after]
        m = self.models.setdefault(plan.model_id, {"active": False, "current": [], "owned": []})
        m["active"] = True
        for op, fp, hit in zip(plan.ops, plan.fps, plan.hits):
            if plan.alias and hit is not None:
                e = hit
                if plan.model_id not in e.owners:
                    e.owners.append(plan.model_id)
            else:
                e = Entry(op.dst_off, op.nbytes, fp, [plan.model_id])
                self.entries.append(e)
                for r in self._regions:
                    if r[0] == op.dst_off:
                        r[3] = e
            if not any(e is c for c in m["current"]):
                m["current"].append(e)
                e.active_refs += 1
            if not any(e is c for c in m["owned"]):
                m["owned"].append(e)
        self.generation += 1
        return [op.dst_off for op in plan.ops]

    def _drop_entry(self, e: Entry) -> None:
        """Remove a tensor from the mapping and free its region."""
        free_at(self._regions, e.off)
        self.image.pop(e.off, None)
        self.entries = [x for x in self.entries if x is not e]
        for mid in list(e.owners):
            m = self.models[mid]
            m["owned"] = [x for x in m["owned"] if x is not e]
            m["current"] = [x for x in m["current"] if x is not e]
            if not m["owned"]:
                del self.models[mid]
        e.owners = []

    # ---------------------------------------------------------------- release
    def release(self, model_id: int, evict: bool = False) -> None:
        """The model instance ends.  Without ``evict`` its tensors stay
        resident and matchable but no longer count as in use (Section 3.1:
        a model that has stopped running keeps its tensors in the pool until
        they are evicted); with it the model gives
        up its tensors, and those no other model owns are freed, their regions
        merged with free neighbours."""
        if model_id not in self.models:
            raise KeyError(model_id)
        m = self.models[model_id]
        for e in m["current"]:
            e.active_refs -= 1
        m["current"] = []
        m["active"] = False
        if evict:
            for e in list(m["owned"]):
                e.owners = [o for o in e.owners if o != model_id]
                if not e.owners:
                    if e.active_refs != 0:
                        raise AssertionError("unowned tensor in use")
                    free_at(self._regions, e.off)
                    self.image.pop(e.off, None)
                    self.entries = [x for x in self.entries if x is not e]
            del self.models[model_id]
        self.generation += 1

    # ------------------------------------------------------------------ stats
    def stats(self) -> Dict[str, int]:
        free = [r[1] for r in self._regions if r[2]]
        return {
            "capacity": self.capacity,
            "free_bytes": sum(free),
            "largest_free": max(free) if free else 0,
            "n_regions": len(self._regions),
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

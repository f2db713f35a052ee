"""Pins for the oracle's Stage 1 eviction (Eq. 2), Stage 2 Partitioned-Gain
Packing (Algorithm 1), alias mode (Section 3.1's in-place reuse) -- CPU only.

Expected values are hand-derived from the paper's formulas and from the
facts its text states about the packing example (initial C = 12, M = 4, two
partition points with gains 1 and 3, the larger tried first and succeeding,
M dropping to 1, the left subspace failing to split further, the right one
having nothing left to split at, final cost 1), plus invariants that hold
for any history: the Region List tiles the pool, every tensor of every
running model holds its source bytes at its returned address, a plan that
fails changes nothing.
"""
import random

import numpy as np
import pytest

import oracle
from oracle import H2D, REUSE, NoSpace, ReuseStoreOracle
from oracle.reuse_store import (allocated_bytes, deal_over_stretches, free_bytes, partitioned_gain_packing, stretches,
                                 subspace, try_packing, try_packing_text)

U = 256


def rb(rnd, n):
    return np.frombuffer(bytes(rnd.getrandbits(8) for _ in range(n)), dtype=np.uint8).copy()


def pack(tensors, align=256):
    offs, at = [], 0
    for t in tensors:
        offs.append(at)
        at += (len(t) + align - 1) // align * align
    host = np.zeros(max(at, align), dtype=np.uint8)
    for t, o in zip(tensors, offs):
        host[o:o + len(t)] = t
    return host, offs


def rows(tensors, offs):
    return [(len(t), oracle.fingerprint(t), o) for t, o in zip(tensors, offs)]


def load(s, mid, tensors, **flags):
    host, offs = pack(tensors)
    plan = s.plan(mid, rows(tensors, offs), host, **flags)
    dsts = s.assemble(plan, host)
    return plan, dsts


def carve_layout(s, rnd, layout):
    """layout: list of (units, keep) -- loads one single-tensor model per item
    into an empty pool (they land back to back), then evicts those with
    keep=False.  Returns {index: (model id, bytes)} of the kept ones."""
    kept = {}
    for i, (units, keep) in enumerate(layout):
        t = rb(rnd, units * U)
        load(s, 100 + i, [t])
        s.release(100 + i)
        kept[i] = (100 + i, t)
    for i, (units, keep) in enumerate(layout):
        if not keep:
            s.release(100 + i, evict=True)
            del kept[i]
    return kept


# ---------------------------------------------------------------- Stage 1
def test_eviction_cost_is_eq_2():
    s = ReuseStoreOracle(1 << 20)
    rnd = random.Random(1)
    load(s, 1, [rb(rnd, 1000)])
    e = s.entries[0]
    assert s.eviction_cost(e) == 1000.0                      # defaults p = b = alpha = 1
    s.set_model_cost(1, 0.25, 4.0, 0.5)
    assert s.eviction_cost(e) == 0.25 * (1000.0 / 4.0) * 0.5  # p * (s / b) * alpha
    with pytest.raises(ValueError):
        s.set_model_cost(1, 0.5, 0.0, 1.0)


def test_hand_derived_eviction_order():
    # Pool of 16 units.  A = {1024, 512} at [0,1536), B = {768, 256} at
    # [1536,2560), C = {512} at [2560,3072); 1024 bytes free at the end.
    # Costs p*(s/b)*alpha:  A: 0.5*(s/2)*1 -> 256, 128;  B: 1*(s/1)*0.1 -> 76.8, 25.6;  C: 512.
    # A model of two 1024-byte tensors needs 2048: evict ascending cost until
    # 2048 bytes are free: B's 256 (25.6), then B's 768 (76.8) -> stop.
    rnd = random.Random(2)
    s = ReuseStoreOracle(16 * U)
    a = [rb(rnd, 1024), rb(rnd, 512)]
    b = [rb(rnd, 768), rb(rnd, 256)]
    c = [rb(rnd, 512)]
    for mid, ts in ((1, a), (2, b), (3, c)):
        load(s, mid, ts)
        s.release(mid)
    s.set_model_cost(1, 0.5, 2.0, 1.0)
    s.set_model_cost(2, 1.0, 1.0, 0.1)
    new = [rb(rnd, 1024), rb(rnd, 1024)]
    host, offs = pack(new)
    with pytest.raises(NoSpace):
        s.plan(9, rows(new, offs), host)                     # Stage 1 is opt-in
    plan = s.plan(9, rows(new, offs), host, evict=True)
    assert [(e.owners, e.nbytes) for e in plan.evictions] == [([2], 256), ([2], 768)]
    assert plan.evicted_bytes == 1024
    dsts = s.assemble(plan, host)
    assert sorted(dsts) == [1536, 3072]                      # B's hole and the old tail
    with pytest.raises(KeyError):
        s.release(2)                                         # nothing of B is left
    assert s.stats()["free_bytes"] == 0
    for t, d in zip(new, dsts):
        assert s.image[d].tobytes() == t.tobytes()
    # Second round, pool full: C now costs 0.3*(512/1)*1 = 153.6, A's tensors still 256 and 128.
    # A 512-byte tensor needs one eviction: A's 512 (128) goes -- not C's 512 (153.6), which a
    # cost that multiplied by the bandwidth would pick, and not A's 1024 (256).
    s.set_model_cost(3, 0.3, 1.0, 1.0)
    more = [rb(rnd, 512)]
    host, offs = pack(more)
    plan = s.plan(10, rows(more, offs), host, evict=True)
    assert [(e.owners, e.nbytes) for e in plan.evictions] == [([1], 512)]
    assert s.assemble(plan, host) == [1024]


def test_eviction_spares_running_models_and_the_plans_own_sources():
    rnd = random.Random(3)
    s = ReuseStoreOracle(8 * U)
    shared = rb(rnd, 512)
    load(s, 1, [shared, rb(rnd, 512)])           # stays running: untouchable
    load(s, 2, [rb(rnd, 256), shared])
    s.release(2)
    # 1 unit free.  The new model reuses `shared` (lowest offset: model 1's copy, which
    # is running and is the plan's source) and needs 2 + 2 fresh units: the other 3
    # can only come from model 2: its 256-byte tensor (cost 256), then its copy of
    # `shared` (cost 512).  Model 1's tensors are never candidates.
    new = [shared, rb(rnd, 512)]
    host, offs = pack(new)
    plan = s.plan(3, rows(new, offs), host, evict=True)
    assert [(e.owners, e.nbytes) for e in plan.evictions] == [([2], 256), ([2], 512)]
    assert plan.ops[0].kind == REUSE and plan.ops[0].src_off == 0
    # asking for more than the evictable bytes fails and changes nothing
    big = [rb(rnd, 5 * U)]
    host2, offs2 = pack(big)
    before = (s.regions, [(e.off, e.nbytes) for e in s.entries])
    with pytest.raises(NoSpace):
        s.plan(4, rows(big, offs2), host2, evict=True)
    assert (s.regions, [(e.off, e.nbytes) for e in s.entries]) == before


@pytest.mark.parametrize("seed", range(5))
def test_eviction_takes_a_minimal_prefix_of_the_cost_order(seed):
    rnd = random.Random(40 + seed)
    s = ReuseStoreOracle(64 * U)
    for mid in range(1, 9):
        load(s, mid, [rb(rnd, rnd.choice([256, 512, 768, 1024])) for _ in range(rnd.randrange(1, 4))])
        s.release(mid)
        s.set_model_cost(mid, rnd.choice([0.1, 0.5, 1.0]), rnd.choice([1.0, 2.0, 8.0]), rnd.choice([1.0, 0.3]))
    free = s.stats()["free_bytes"]
    want = free + rnd.randrange(1, 12) * U
    new = [rb(rnd, want)]
    host, offs = pack(new)
    try:
        plan = s.plan(99, rows(new, offs), host, evict=True, merge=True)
    except NoSpace:
        return
    order = sorted(s.entries, key=lambda e: (s.eviction_cost(e), e.off))
    k = len(plan.evictions)
    assert [id(e) for e in plan.evictions] == [id(e) for e in order[:k]]
    freed = [(-(-e.nbytes // U)) * U for e in plan.evictions]
    assert free + sum(freed) >= want > free + sum(freed[:-1])


# ---------------------------------------------------------------- Algorithm 1
def test_try_packing_follows_the_listing():
    sizes = [6, 1, 3, 3, 4, 5]
    assert try_packing(sizes, [0, 1], 8, 8) == ([0], [1])   # 6 -> bin 1 (tie: first), 1 -> bin 2 (more room)
    assert try_packing(sizes, [2, 3], 4, 4) == ([], [])     # second 3 is not smaller than min(1, 4)
    assert try_packing(sizes, [4], 4, 9) == ([], [])        # not strictly smaller than the smaller bin
    assert try_packing(sizes, [0, 5], 8, 12) == ([5], [0])  # 6 -> bin 2, then 5 < min(8, 6) -> bin 1
    assert try_packing(sizes, [], 8, 8) == ([], [])


def test_try_packing_as_the_text_words_it():
    sizes = [6, 1, 3, 3, 4, 5]
    assert try_packing_text(sizes, [2, 3], 4, 4) == ([2], [3])   # each fits the bin with more room
    assert try_packing_text(sizes, [4], 4, 9) == ([], [4])
    assert try_packing_text(sizes, [4], 4, 3) == ([4], [])       # exact fit is a fit
    assert try_packing_text(sizes, [0, 5], 5, 5) == ([], [])     # 6 fits neither
    # four equal tensors over two equal halves: the listing's test gives up at the
    # fourth, the text's places two on each side
    s4 = [1000] * 4
    assert try_packing(s4, [0, 1, 2, 3], 2560, 2560) == ([], [])
    assert try_packing_text(s4, [0, 1, 2, 3], 2560, 2560) == ([0, 2], [1, 3])


def regions_of(units):
    """units: list of (length, is_free) -> Region List rows [off, len, free, tag]."""
    out, at = [], 0
    for length, free in units:
        out.append([at, length * U, free, None if free else ("t", at)])
        at += length * U
    return out


@pytest.mark.parametrize("cap_as_printed", [False, True])
def test_packing_example_of_the_paper(cap_as_printed):
    # One unit of the paper's example = 2 * 256 bytes here.  Free 2, A (gain 1),
    # free 2, B (gain 3), free 4:  C = 12, M = 4.
    regs = regions_of([(4, True), (2, False), (4, True), (6, False), (8, True)])
    whole = subspace(regs, 0, len(regs))
    assert whole == (0, 5)
    assert free_bytes(regs, whole) + allocated_bytes(regs, whole) == 12 * 2 * U      # C
    assert allocated_bytes(regs, whole) == 4 * 2 * U                                # M
    sizes = [6 * U, 1 * U]
    seen = []

    def watched(sz, tensors, c1, c2):
        seen.append((c1 // U, c2 // U))
        return try_packing(sz, tensors, c1, c2)
    final, m = partitioned_gain_packing(regs, [(whole, [0, 1])], sizes, watched, cap_as_printed)
    # the point with gain 3 is tried first and succeeds: M = 4 -> 1; the left
    # subspace keeps its tensor and cannot be split at the gain-1 point (6 is
    # not smaller than 4); the right one has no allocated region left
    assert m == 1 * 2 * U
    assert final == [((0, 3), [0]), ((4, 5), [1])]
    # what reached the packing test: first the two sides of the gain-3 point, then those of the
    # gain-1 point.  With the capacity as the text defines it the sides of the first point and the
    # point itself make up C = 12 (paper units); by free bytes alone they make up C - M = 8.
    if cap_as_printed:
        assert seen == [(10, 8), (4, 4)] and seen[0][0] + seen[0][1] + 6 == 12 * 2
    else:
        assert seen == [(8, 8), (4, 4)] and seen[0][0] + seen[0][1] == (12 - 4) * 2
    # had the gain-1 point been tried first it would have failed:
    assert try_packing(sizes, [0, 1], 4 * U, 12 * U) == ([], [])


def test_capacity_as_printed_can_hand_a_subspace_more_than_it_holds():
    # Units of 256 B:  F2 A10 F2 b1 F6  (21 units, 10 free).  Incoming 5 and 4 (9 <= 10 free), text's
    # packing test.  Best fit fails (after 5 -> F6 no hole holds 4).
    # By free bytes: at A (gain 10) the sides hold 2 and 8: 5 -> right (3 left), 4 fits neither: no.
    #   At b (gain 1) they hold 4 and 6: 5 -> right, 4 -> left: split.  Left {4}: A slides 2 -> 0, the
    #   4 lands behind it at 10; right {5} goes straight into F6 at 15.  M = 10 (A may move).
    # By the printed capacity (free + allocated): at A the sides "hold" 2 and 2 + 1 + 6 = 9: 5 -> right
    #   (4 left), 4 -> right: accepted -- but the right side has 8 free bytes for 9 bytes of tensors,
    #   and splitting it at b cannot help (5 -> F6, 4 > 2).  No placement exists inside it.
    rnd = random.Random(11)

    def fresh():
        s = ReuseStoreOracle(21 * U)
        carve_layout(s, rnd, [(2, False), (10, True), (2, False), (1, True), (6, False)])
        assert [(r[1] // U, r[2]) for r in s.regions] == [(2, True), (10, False), (2, True), (1, False), (6, True)]
        return s
    new = [rb(rnd, 5 * U), rb(rnd, 4 * U)]
    host, offs = pack(new)
    s = fresh()
    with pytest.raises(NoSpace):
        s.plan(9, rows(new, offs), host)
    plan = s.plan(9, rows(new, offs), host, merge=True, pack_text=True)
    assert [(o // U, n // U) for _e, o, n in plan.moves] == [(2, 0)]
    assert [op.dst_off // U for op in plan.ops] == [15, 10]
    assert plan.merge_bound == 10 * U and plan.moved_bytes == 10 * U
    with pytest.raises(NoSpace):
        fresh().plan(9, rows(new, offs), host, merge=True, pack_text=True, cap_text=True)
    # where nothing is over-committed the two capacities plan alike: the hand-derived merge example
    layout = [(4, False), (2, True), (4, False), (6, True), (4, False), (1, True), (4, False), (1, True), (4, False)]
    new = [rb(rnd, 6 * U), rb(rnd, 5 * U - 7)]
    host, offs = pack(new)
    plans = []
    for cap_text in (False, True):
        s = ReuseStoreOracle(30 * U)
        carve_layout(s, rnd, layout)
        plans.append(s.plan(9, rows(new, offs), host, merge=True, cap_text=cap_text))
    assert [op.dst_off for op in plans[0].ops] == [op.dst_off for op in plans[1].ops]
    assert [(o, n) for _e, o, n in plans[0].moves] == [(o, n) for _e, o, n in plans[1].moves]


def test_regions_that_cannot_move_cut_the_pool_into_subspaces():
    # F3 w1 F2 a1 F4 w1 w1 F5 a2 (w: running, cannot move; a: retained)
    regs = regions_of([(3, True), (1, False), (2, True), (1, False), (4, True), (1, False), (1, False), (5, True),
                       (2, False)])
    walls = {1, 5, 6}
    for i in walls:
        regs[i][3] = "wall"
    subs = stretches(regs, lambda r: r[3] != "wall")
    assert subs == [(0, 1), (2, 5), (7, 8)]           # the trailing retained tensor is outside every subspace
    assert [free_bytes(regs, x) // U for x in subs] == [3, 6, 5]
    sizes = [u * U for u in (5, 4, 3, 1, 1)]
    # each tensor to the subspace with the most room left (ties: lowest address):
    # 5 -> middle (6 -> 1); 4 -> last (5 -> 1); 3 -> first (3 -> 0); 1 -> middle (tie 1 = 1: lower address); 1 -> last
    assert deal_over_stretches(regs, subs, sizes, [0, 1, 2, 3, 4], False) == [[2], [0, 3], [1, 4]]
    assert deal_over_stretches(regs, subs, [6 * U, 6 * U], [0, 1], False) is None       # the second 6 fits nowhere
    assert deal_over_stretches(regs, [], sizes, [0], False) is None
    # by the printed capacity the middle subspace counts its retained tensor as room: 7
    assert deal_over_stretches(regs, subs, [7 * U], [0], True) == [[], [0], []]


# An independent statement of the two packing tests, for the checks below: written as a search for
# the first tensor that breaks the rule rather than as the listing's loop.
def packs(sizes, tensors, c1, c2, text):
    room = [c1, c2]
    sides = ([], [])
    for k in tensors:
        b = 0 if room[0] >= room[1] else 1
        ok = sizes[k] <= room[b] if text else sizes[k] < min(room)
        if not ok:
            return None
        sides[b].append(k)
        room[b] -= sizes[k]
    return sides if (sides[0] or sides[1]) else None


def consistent_tree(regs, finals, sizes, text):
    """True if the final subspaces `finals` (address order, those of one starting subspace) can have
    come from splitting their union at allocated regions, each split passing the packing test with
    exactly the tensor subsets found on its two sides."""
    if len(finals) == 1:
        return True
    lo, hi = finals[0][0][0], finals[-1][0][1]
    order = sorted((k for _s, t in finals for k in t), key=lambda k: (-sizes[k], k))
    for cut in range(1, len(finals)):
        left, right = finals[:cut], finals[cut:]
        between = [i for i in range(left[-1][0][1], right[0][0][0]) if not regs[i][2]]
        for p in between:
            p1, p2 = subspace(regs, lo, p), subspace(regs, p + 1, hi)
            if p1 != (lo, left[-1][0][1]) or p2 != (right[0][0][0], hi):
                continue
            got = packs(sizes, order, free_bytes(regs, p1), free_bytes(regs, p2), text)
            want = (sorted(k for _s, t in left for k in t), sorted(k for _s, t in right for k in t))
            if got is not None and (sorted(got[0]), sorted(got[1])) == want:
                if consistent_tree(regs, left, sizes, text) and consistent_tree(regs, right, sizes, text):
                    return True
    return False


@pytest.mark.parametrize("seed", range(40))
def test_algorithm_1_on_random_small_pools_structure_independent_checks(seed):
    """What must hold of Algorithm 1's result whatever the code that produced it looks like."""
    rnd = random.Random(7000 + seed)
    text = seed % 2 == 1
    units = []
    for _ in range(rnd.randrange(5, 16)):
        units.append((rnd.randrange(1, 6), True))
        for _ in range(rnd.randrange(1, 3)):                # sometimes two residents back to back
            units.append((rnd.randrange(1, 7), False))
    units.append((rnd.randrange(1, 6), True))
    regs = regions_of(units)
    whole = subspace(regs, 0, len(regs))
    total_free = free_bytes(regs, whole)
    sizes, left = [], total_free
    while left >= U and len(sizes) < 8:
        n = rnd.randrange(1, max(2, left // U // 2 + 1)) * U
        sizes.append(n)
        left -= n
    order = sorted(range(len(sizes)), key=lambda k: (-sizes[k], k))
    final, m_listing = partitioned_gain_packing(regs, [(whole, order)], sizes,
                                                try_packing_text if text else try_packing)
    # the allocation set covers every tensor once, its subspaces lie in address order, do not overlap,
    # and each begins and ends with a free region
    assert sorted(k for _s, t in final for k in t) == list(range(len(sizes)))
    for (a, _ta), (b, _tb) in zip(final, final[1:]):
        assert a[1] <= b[0]
    for sub, subset in final:
        assert regs[sub[0]][2] and regs[sub[1] - 1][2]
        assert subset == sorted(subset, key=lambda k: (-sizes[k], k))      # sorted once, order kept
        # every subset fits the free bytes of its subspace
        assert sum(sizes[k] for k in subset) <= free_bytes(regs, sub)
    # the bound: what can move at all lies inside the subspaces that were given tensors; the listing's
    # running M never falls below that, and never exceeds merging everything
    inside = sum(allocated_bytes(regs, sub) for sub, subset in final if subset)
    assert inside <= m_listing <= allocated_bytes(regs, whole)
    gone = sum(r[1] for i, r in enumerate(regs) if not r[2] and not any(s[0] <= i < s[1] for s, _t in final))
    empty = sum(allocated_bytes(regs, sub) for sub, subset in final if not subset)
    taken = allocated_bytes(regs, whole) - m_listing                        # sizes of the points taken
    assert m_listing - inside == empty + (gone - taken)
    # every split that led here passes the packing test with exactly these subsets ...
    assert consistent_tree(regs, final, sizes, text)
    # ... and no final subspace that holds tensors can be split any further
    for sub, subset in final:
        for p in range(sub[0], sub[1]):
            if subset and not regs[p][2]:
                p1, p2 = subspace(regs, sub[0], p), subspace(regs, p + 1, sub[1])
                assert packs(sizes, subset, free_bytes(regs, p1), free_bytes(regs, p2), text) is None


@pytest.mark.parametrize("seed", range(30))
def test_merge_plans_on_random_small_pools_keep_their_promises(seed):
    """Whole plans: moved bytes <= merge bound <= merge-all; moves only shift towards lower
    addresses and never cross a running tensor; residents that do not move stay where they were."""
    rnd = random.Random(9000 + seed)
    s = ReuseStoreOracle(64 * U)
    layout = []
    for _ in range(rnd.randrange(4, 12)):
        layout.append((rnd.randrange(1, 5), False))
        layout.append((rnd.randrange(1, 5), True))
    total = sum(u for u, _k in layout)
    if total > 60:
        pytest.skip("layout does not fit")
    layout.append((64 - total, False))
    kept = carve_layout(s, rnd, layout)
    running = []
    for i, (mid, t) in sorted(kept.items()):
        if rnd.random() < 0.25:                    # some residents are running: they cannot move
            host_w, offs_w = pack([t])
            s.assemble(s.plan(mid, rows([t], offs_w), host_w, alias=True), host_w)
            running.append(next(e for e in s.entries if e.owners == [mid]))
    free = s.stats()["free_bytes"]
    new = []
    while free >= 4 * U and len(new) < 5:
        n = rnd.randrange(1, max(2, free // U // 2)) * U
        new.append(rb(rnd, n - rnd.randrange(0, 9)))
        free -= n
    if not new:
        pytest.skip("pool is full")
    host, offs = pack(new)
    flags = dict(merge=True, pack_text=seed % 2 == 0)
    before = [list(r) for r in s._regions]
    try:
        plan = s.plan(9, rows(new, offs), host, **flags)
    except NoSpace:
        return
    merge_all = sum(r[1] for r in before if not r[2])
    assert plan.moved_bytes <= sum(-(-e.nbytes // U) * U for e, _o, _n in plan.moves) <= plan.merge_bound <= merge_all
    walls = sorted(e.off for e in running)
    for e, old, to in plan.moves:
        assert e.active_refs == 0 and to < old
        assert not any(to < w < old for w in walls)
    # nothing outside the stretch of addresses between two running tensors that a move touches has changed
    after = {r[0]: r for r in plan.regions_after if not r[2] and r[3] is not None and not isinstance(r[3], tuple)}
    moved_ids = {id(e) for e, _o, _n in plan.moves}
    for r in before:
        if not r[2] and id(r[3]) not in moved_ids and not any(e is r[3] for e in plan.evictions):
            assert r[0] in after and after[r[0]][3] is r[3]
    dsts = s.assemble(plan, host)
    for t, d in zip(new, dsts):
        assert s.image[d][:len(t)].tobytes() == t.tobytes()
    for mid, t in kept.values():
        es = [e for e in s.entries if mid in e.owners]
        assert len(es) == 1 and s.image[es[0].off][:len(t)].tobytes() == t.tobytes()


def test_hand_derived_merge_plan():
    # Units of 256 B:  F4 a2 F4 B6 F4 c1 F4 d1 F4  (30 units; free 20 in five holes of 4).
    # Incoming 6 and 5: plain best fit fails (no hole >= 6).  Algorithm 1:
    # M = 10; split at B (gain 6): bins 8 and 12 -> 6 goes right (12 > 8), 5 < min(8, 6)
    # goes left; M = 4.  Left {5} cannot split at a (5 >= 4); right {6} cannot
    # split at c or d (6 >= 4).  Realisation: left: a slides 4 -> 0, the 5 lands at 2;
    # right (starts at unit 16): c slides 20 -> 16, d slides 25 -> 17, the 6 lands at 18.
    rnd = random.Random(5)
    s = ReuseStoreOracle(30 * U)
    layout = [(4, False), (2, True), (4, False), (6, True), (4, False), (1, True), (4, False),
              (1, True), (4, False)]
    kept = carve_layout(s, rnd, layout)
    assert [r[1] // U for r in s.regions] == [4, 2, 4, 6, 4, 1, 4, 1, 4]
    new = [rb(rnd, 6 * U), rb(rnd, 5 * U - 7)]
    host, offs = pack(new)
    with pytest.raises(NoSpace):
        s.plan(9, rows(new, offs), host)
    plan = s.plan(9, rows(new, offs), host, merge=True)
    assert plan.merge_bound == 4 * U
    assert [(old // U, to // U) for _e, old, to in plan.moves] == [(4, 0), (20, 16), (25, 17)]
    assert plan.moved_bytes == 4 * U
    assert [op.dst_off // U for op in plan.ops] == [18, 2]
    dsts = s.assemble(plan, host)
    for t, d in zip(new, dsts):
        assert s.image[d].tobytes() == t.tobytes()
    for mid, t in kept.values():                       # residents kept their bytes
        e = next(e for e in s.entries if e.owners == [mid])
        assert s.image[e.off].tobytes() == t.tobytes()
    assert [(r[0] // U, r[1] // U, r[2]) for r in s.regions] == [
        (0, 2, False), (2, 5, False), (7, 3, True), (10, 6, False), (16, 1, False), (17, 1, False),
        (18, 6, False), (24, 6, True)]


def test_a_subspace_begins_and_ends_with_a_free_region():
    # Section 3.2, "Partitioning subspaces": a subspace starts and ends with a free region, so an
    # allocated region at either end of a stretch is outside it: it is not part of the merge cost
    # and it never moves.  Units: a2 F3 b1 F3 c2, one incoming tensor of 5.
    rnd = random.Random(8)
    s = ReuseStoreOracle(11 * U)
    kept = carve_layout(s, rnd, [(2, True), (3, False), (1, True), (3, False), (2, True)])
    assert [(r[1] // U, r[2]) for r in s.regions] == [(2, False), (3, True), (1, False), (3, True), (2, False)]
    assert subspace(s.regions, 0, 5) == (1, 4) and subspace(s.regions, 0, 1) is None
    assert subspace(s.regions, 2, 5) == (3, 4)
    new = [rb(rnd, 5 * U)]
    host, offs = pack(new)
    with pytest.raises(NoSpace):
        s.plan(9, rows(new, offs), host)
    plan = s.plan(9, rows(new, offs), host, merge=True)
    assert plan.merge_bound == 1 * U                              # b alone: a and c are outside
    assert [(o // U, n // U) for _e, o, n in plan.moves] == [(5, 2)]
    assert [op.dst_off // U for op in plan.ops] == [3]
    s.assemble(plan, host)
    assert [(r[0] // U, r[1] // U, r[2]) for r in s.regions] == [
        (0, 2, False), (2, 1, False), (3, 5, False), (8, 1, True), (9, 2, False)]
    for mid, t in kept.values():
        e = next(e for e in s.entries if e.owners == [mid])
        assert s.image[e.off].tobytes() == t.tobytes()


def test_running_tensors_are_walls():
    rnd = random.Random(6)
    s = ReuseStoreOracle(20 * U)
    # F4 w2 F4 a1 F5, with w running
    kept = carve_layout(s, rnd, [(4, False), (2, True), (4, False), (1, True), (9, False)])
    wall_id, wall_bytes = kept[1]
    host_w, offs_w = pack([wall_bytes])
    s.release(wall_id)  # already released; make it running again by loading it in alias mode
    plan = s.plan(wall_id, rows([wall_bytes], offs_w), host_w, alias=True)
    s.assemble(plan, host_w)
    assert s.stats()["n_active"] == 1
    # 7 units do not fit anywhere, and merging across the running tensor is not allowed,
    # but right of it free 4 + 9 with a1 in between can be merged
    new = [rb(rnd, 10 * U), rb(rnd, 3 * U)]
    host, offs = pack(new)
    plan = s.plan(9, rows(new, offs), host, merge=True)
    assert all(e.active_refs == 0 for e, _o, _n in plan.moves)
    assert [(o // U, n // U) for _e, o, n in plan.moves] == [(10, 6)]
    assert [op.dst_off // U for op in plan.ops] == [7, 0]
    # a tensor larger than either side of the wall cannot be placed
    huge = [rb(rnd, 15 * U)]
    host, offs = pack(huge)
    with pytest.raises(NoSpace):
        s.plan(10, rows(huge, offs), host, merge=True)


# ---------------------------------------------------------------- alias mode
def test_alias_mode_reuses_in_place_and_shares_ownership():
    rnd = random.Random(7)
    s = ReuseStoreOracle(32 * U)
    a = [rb(rnd, 1024), rb(rnd, 512), rb(rnd, 300)]
    _, a_dst = load(s, 1, a)
    s.release(1)
    b = [a[0], rb(rnd, 700), a[2]]
    host, offs = pack(b)
    free_before = s.stats()["free_bytes"]
    plan = s.plan(2, rows(b, offs), host, alias=True)
    assert [op.kind for op in plan.ops] == [REUSE, H2D, REUSE]
    assert plan.ops[0].dst_off == plan.ops[0].src_off == a_dst[0]
    assert plan.ops[2].dst_off == a_dst[2]
    dsts = s.assemble(plan, host)
    assert s.stats()["free_bytes"] == free_before - 768          # only the miss took space
    assert s.stats()["n_entries"] == 4 and s.stats()["n_active"] == 3
    for t, d in zip(b, dsts):
        assert s.image[d][:len(t)].tobytes() == t.tobytes()
    shared = next(e for e in s.entries if e.off == a_dst[0])
    assert shared.owners == [1, 2] and shared.active_refs == 1
    # model 1 comes back while 2 runs: everything of it is resident
    host_a, offs_a = pack(a)
    plan = s.plan(1, rows(a, offs_a), host_a, alias=True)
    assert plan.transfer_bytes == 0 and [op.dst_off for op in plan.ops] == a_dst
    s.assemble(plan, host_a)
    assert shared.active_refs == 2
    # evicting model 2 keeps what model 1 also owns
    s.release(2, evict=True)
    assert shared.owners == [1] and shared.active_refs == 1
    assert s.stats()["n_entries"] == 3
    s.release(1, evict=True)
    assert s.regions == [[0, 32 * U, True]]


def test_alias_hit_that_moves_reports_its_new_address():
    rnd = random.Random(8)
    s = ReuseStoreOracle(12 * U)
    kept = carve_layout(s, rnd, [(3, False), (2, True), (3, False), (1, True), (3, False)])
    mid, t = kept[1]
    new = [t, rb(rnd, 5 * U)]
    host, offs = pack(new)
    plan = s.plan(9, rows(new, offs), host, merge=True, alias=True)
    moved = {old: to for _e, old, to in plan.moves}
    assert moved.get(3 * U) == 0
    assert plan.ops[0].kind == REUSE and plan.ops[0].dst_off == 0 and plan.ops[0].src_off == 0
    dsts = s.assemble(plan, host)
    for x, d in zip(new, dsts):
        assert s.image[d][:len(x)].tobytes() == x.tobytes()


# ------------------------------------------------------------ any history
def check_invariants(s, running):
    at, prev_free = 0, False
    for off, length, free in s.regions:
        assert off == at and length > 0 and off % s.align == 0
        assert not (free and prev_free)
        prev_free, at = free, at + length
    assert at == s.capacity
    assert sorted(r[0] for r in s.regions if not r[2]) == sorted(e.off for e in s.entries)
    for e in s.entries:
        assert e.owners and e.active_refs >= 0
        assert e.active_refs == sum(1 for m in s.models.values() if any(x is e for x in m["current"]))
    # every tensor of every running model holds its source bytes where the caller was told
    for mid, (tensors, dsts) in running.items():
        for t, d in zip(tensors, dsts):
            cur = s.image[d]
            assert cur[:len(t)].tobytes() == t.tobytes(), (mid, d)


@pytest.mark.parametrize("seed", range(12))
def test_random_histories_with_every_flag(seed):
    rnd = random.Random(300 + seed)
    s = ReuseStoreOracle(96 * U)
    library = [rb(rnd, rnd.choice([40, 256, 300, 512, 1000, 1024, 2048, 3000])) for _ in range(24)]
    running, retained, next_id = {}, set(), 1
    for step in range(120):
        r = rnd.random()
        if r < 0.5 or not (running or retained):
            tensors = [library[rnd.randrange(24)] for _ in range(rnd.randrange(1, 7))]
            flags = dict(evict=rnd.random() < 0.7, merge=rnd.random() < 0.7, alias=rnd.random() < 0.5,
                         pack_text=rnd.random() < 0.5)
            mid = next_id
            if retained and rnd.random() < 0.2:
                mid = rnd.choice(sorted(retained))
            host, offs = pack(tensors)
            snapshot = (s.regions, [(e.off, e.nbytes, tuple(e.owners), e.active_refs) for e in s.entries])
            try:
                plan = s.plan(mid, rows(tensors, offs), host, **flags)
            except NoSpace:
                assert snapshot == (s.regions, [(e.off, e.nbytes, tuple(e.owners), e.active_refs) for e in s.entries])
                continue
            assert snapshot == (s.regions, [(e.off, e.nbytes, tuple(e.owners), e.active_refs) for e in s.entries])
            assert plan.reused_bytes + plan.transfer_bytes == sum(len(t) for t in tensors)
            assert plan.moved_bytes <= plan.merge_bound or not plan.moves
            moved = {id(e): new for e, _o, new in plan.moves}
            dsts = s.assemble(plan, host)
            # tensors of running models may not have moved or vanished
            running[mid] = (tensors, dsts)
            retained.discard(mid)
            for e in plan.evictions:
                for m in list(retained):
                    if m not in s.models:
                        retained.discard(m)
            if mid == next_id:
                next_id += 1
        else:
            if running and (not retained or rnd.random() < 0.6):
                mid = rnd.choice(sorted(running))
                evict = rnd.random() < 0.4
                s.release(mid, evict=evict)
                del running[mid]
                if not evict:
                    retained.add(mid)
            else:
                mid = rnd.choice(sorted(retained))
                if mid in s.models:
                    s.release(mid, evict=True)
                retained.discard(mid)
        retained = {m for m in retained if m in s.models}
        check_invariants(s, running)

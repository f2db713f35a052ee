"""Pins for the oracle's Reuse Store bookkeeping (CPU only).

Lookup, best-fit allocation and assembly follow the paper's Sections 3.1 and
3.2.  Expected values come from a hand-derived allocation example, from
brute force (all-pairs byte comparison, exhaustive scan of free regions
written a different way) and from invariants the text states: regions tile
the pool in physical order, each is free or allocated, an allocation leaves a
smaller free region, every new tensor is placed, tensors stay contiguous.
"""
import random

import numpy as np
import pytest

import oracle
from oracle import H2D, REUSE, NoSpace, ReuseStoreOracle, StalePlan


def rand_bytes(rnd, n):
    return np.frombuffer(bytes(rnd.getrandbits(8) for _ in range(n)), dtype=np.uint8).copy()


def pack(tensors, align=256):
    """Host buffer holding the tensors back to back on align boundaries."""
    offs, at = [], 0
    for t in tensors:
        offs.append(at)
        at += (len(t) + align - 1) // align * align
    host = np.zeros(max(at, align), dtype=np.uint8)
    for t, o in zip(tensors, offs):
        host[o:o + len(t)] = t
    return host, offs


def descs(tensors, offs):
    return [(len(t), oracle.fingerprint(t), o) for t, o in zip(tensors, offs)]


def load(store, model_id, tensors, confirm=False):
    host, offs = pack(tensors)
    plan = store.plan(model_id, descs(tensors, offs), host, confirm)
    dsts = store.assemble(plan, host)
    return plan, dsts


def check_region_invariants(store):
    at = 0
    prev_free = False
    for off, length, free in store.regions:
        assert off == at and length > 0
        assert off % store.align == 0 and length % store.align == 0
        assert not (free and prev_free), "adjacent free regions must be merged"
        prev_free = free
        at += length
    assert at == store.capacity
    allocated = sorted(r[0] for r in store.regions if not r[2])
    assert allocated == sorted(e.off for e in store.entries)
    for e in store.entries:
        r = next(r for r in store.regions if r[0] == e.off)
        assert r[1] == (e.nbytes + store.align - 1) // store.align * store.align


def test_hand_derived_best_fit_example():
    # Pool of 3072 B, alignment 256.  X and Y are resident; the free regions
    # are [0,1024), [1536,2048) and [2304,3072).  Incoming sizes 700, 256, 500
    # round to 768, 256, 512 and are placed largest first:
    #   768 -> smallest free region >= 768 is [2304,3072) (768 long): exact fit
    #   512 -> [1536,2048) exact fit
    #   256 -> only [0,1024) is left; placed at its low end
    # leaving the single free region [256,1024).
    rnd = random.Random(1)
    s = ReuseStoreOracle(3072, 256)
    for mid, n in ((1, 1024), (2, 512), (3, 512), (4, 256), (5, 768)):
        load(s, mid, [rand_bytes(rnd, n)])
    assert [e.off for e in s.entries] == [0, 1024, 1536, 2048, 2304]
    for mid in (1, 3, 5):
        s.release(mid, evict=True)
    assert s.regions == [[0, 1024, True], [1024, 512, False], [1536, 512, True],
                         [2048, 256, False], [2304, 768, True]]
    plan, dsts = load(s, 9, [rand_bytes(rnd, 700), rand_bytes(rnd, 256), rand_bytes(rnd, 500)])
    assert dsts == [2304, 0, 1536]
    assert [r for r in s.regions if r[2]] == [[256, 768, True]]
    assert plan.reused_bytes == 0 and plan.transfer_bytes == 1456
    check_region_invariants(s)


def test_ties_take_the_lowest_offset_and_equal_sizes_go_in_index_order():
    rnd = random.Random(2)
    s = ReuseStoreOracle(4096, 256)
    # carve: [0,512) free, [512,768) used, [768,1280) free, [1280,1536) used, rest free
    for mid, n in ((1, 512), (2, 256), (3, 512), (4, 256)):
        load(s, mid, [rand_bytes(rnd, n)])
    s.release(1, evict=True)
    s.release(3, evict=True)
    plan, dsts = load(s, 9, [rand_bytes(rnd, 512), rand_bytes(rnd, 300)])
    # two free regions of 512 tie: tensor 0 -> offset 0, tensor 1 (512 rounded) -> 768
    assert dsts == [0, 768]


def brute_force_sources(resident, incoming):
    """All-pairs byte comparison: lowest-offset byte-identical resident copy."""
    out = []
    for t in incoming:
        hits = [off for off, r in resident if len(r) == len(t) and r.tobytes() == t.tobytes()]
        out.append(min(hits) if hits else None)
    return out


@pytest.mark.parametrize("seed", range(6))
def test_match_equals_all_pairs_byte_comparison(seed):
    rnd = random.Random(100 + seed)
    s = ReuseStoreOracle(1 << 20, 256)
    pool_of_tensors = [rand_bytes(rnd, rnd.choice([16, 48, 256, 300, 1000, 4096]))
                       for _ in range(12)]
    # resident model A holds some tensors, several of them twice
    a = [pool_of_tensors[rnd.randrange(12)] for _ in range(14)]
    _, a_dst = load(s, 1, a)
    s.release(1)
    resident = list(zip(a_dst, a))
    b = [pool_of_tensors[rnd.randrange(12)] for _ in range(10)] + [rand_bytes(rnd, 256)]
    # same length as a resident tensor but different bytes: must miss
    b.append(rand_bytes(rnd, len(a[0])))
    want = brute_force_sources(resident, b)
    host, offs = pack(b)
    plan = s.plan(2, descs(b, offs), host)
    for op, src, off in zip(plan.ops, want, offs):
        if src is None:
            assert op.kind == H2D and op.src_off == off
        else:
            assert op.kind == REUSE and op.src_off == src
    assert plan.reused_bytes + plan.transfer_bytes == sum(len(t) for t in b)
    # confirm on gives the same answer when there are no collisions
    plan_c = s.plan(2, descs(b, offs), host, confirm=True)
    assert [(o.kind, o.src_off) for o in plan_c.ops] == [(o.kind, o.src_off) for o in plan.ops]


def replay_best_fit(regions_before, ops, align):
    """Independent replay: keep free space as a dict offset->length, and for
    each tensor (largest rounded size first, then index) check that the
    chosen offset is the start of the smallest adequate free region."""
    free = {r[0]: r[1] for r in regions_before if r[2]}
    order = sorted(range(len(ops)), key=lambda k: (-((ops[k].nbytes + align - 1) // align * align), k))
    for k in order:
        need = (ops[k].nbytes + align - 1) // align * align
        fits = sorted((length, off) for off, length in free.items() if length >= need)
        assert fits, "oracle placed a tensor where nothing fits"
        length, off = fits[0]
        assert ops[k].dst_off == off
        del free[off]
        if length > need:
            free[off + need] = length - need
    return free


@pytest.mark.parametrize("seed", range(8))
def test_random_histories_keep_every_invariant(seed):
    rnd = random.Random(200 + seed)
    cap = 256 * 400
    s = ReuseStoreOracle(cap, 256)
    library = [rand_bytes(rnd, rnd.choice([8, 100, 256, 257, 512, 700, 1024, 3000, 5000]))
               for _ in range(20)]
    live = {}
    next_id = 1
    for step in range(60):
        action = rnd.random()
        if action < 0.55 or not live:
            tensors = [library[rnd.randrange(20)] for _ in range(rnd.randrange(1, 7))]
            host, offs = pack(tensors)
            before = [list(r) for r in s.regions]
            entries_before = [(e.off, e.nbytes, e.fp, e.model_id, e.active) for e in s.entries]
            try:
                plan = s.plan(next_id, descs(tensors, offs), host)
            except NoSpace:
                assert s.regions == before
                assert [(e.off, e.nbytes, e.fp, e.model_id, e.active) for e in s.entries] == entries_before
                continue
            assert s.regions == before, "planning must not change the pool"
            replay_best_fit(before, plan.ops, 256)
            # destinations: aligned, pairwise disjoint, inside formerly free space,
            # disjoint from every source
            spans = sorted((op.dst_off, op.dst_off + (op.nbytes + 255) // 256 * 256) for op in plan.ops)
            for (a0, a1), (b0, b1) in zip(spans, spans[1:]):
                assert a1 <= b0
            for lo, hi in spans:
                assert lo % 256 == 0
                assert any(r[2] and r[0] <= lo and hi <= r[0] + r[1] for r in before)
            dsts = s.assemble(plan, host)
            for t, d in zip(tensors, dsts):
                assert s.image[d].tobytes() == t.tobytes()
            live[next_id] = True
            next_id += 1
        else:
            mid = rnd.choice(list(live))
            evict = rnd.random() < 0.6
            s.release(mid, evict=evict)
            if evict:
                del live[mid]
        check_region_invariants(s)
        st = s.stats()
        assert st["free_bytes"] + sum((e.nbytes + 255) // 256 * 256 for e in s.entries) == cap


def test_assembled_model_equals_source_and_bytes_add_up():
    rnd = random.Random(3)
    s = ReuseStoreOracle(1 << 20, 256)
    a = [rand_bytes(rnd, n) for n in (4096, 512, 512, 10000, 24)]
    load(s, 1, a)
    s.release(1)
    b = [a[0], rand_bytes(rnd, 512), a[3], a[4], rand_bytes(rnd, 24)]
    host, offs = pack(b)
    plan = s.plan(2, descs(b, offs), host)
    dsts = s.assemble(plan, host)
    assert [op.kind for op in plan.ops] == [REUSE, H2D, REUSE, REUSE, H2D]
    assert plan.reused_bytes == 4096 + 10000 + 24
    assert plan.transfer_bytes == 512 + 24
    assert plan.reused_bytes + plan.transfer_bytes == sum(len(t) for t in b)
    for t, d, o in zip(b, dsts, offs):
        assert s.image[d].tobytes() == host[o:o + len(t)].tobytes() == t.tobytes()
    # the resident copies are untouched
    for e, t in zip(s.entries[:5], a):
        assert s.image[e.off].tobytes() == t.tobytes()


def test_duplicates_inside_one_model_and_across_models():
    ones = np.frombuffer(b"\x80\x3f" * 256, dtype=np.uint8).copy()
    rnd = random.Random(4)
    s = ReuseStoreOracle(1 << 16, 256)
    # a fresh pool: identical incoming tensors do not feed each other
    plan, dsts = load(s, 1, [ones, ones, rand_bytes(rnd, 512), ones])
    assert [op.kind for op in plan.ops] == [H2D] * 4
    s.release(1)
    # now three resident copies: the lowest offset is the source for all hits
    plan2, _ = load(s, 2, [ones, ones])
    lowest = min(d for d, op in zip(dsts, plan.ops) if op.nbytes == 512 and d in (dsts[0], dsts[1], dsts[3]))
    assert [op.kind for op in plan2.ops] == [REUSE, REUSE]
    assert {op.src_off for op in plan2.ops} == {lowest}


def test_same_bytes_different_length_do_not_match():
    s = ReuseStoreOracle(1 << 16, 256)
    six = np.frombuffer(b"\x01\x02\x03\x04\x05\x06", dtype=np.uint8).copy()
    eight = np.frombuffer(b"\x01\x02\x03\x04\x05\x06\x00\x00", dtype=np.uint8).copy()
    assert oracle.fingerprint(six) == oracle.fingerprint(eight)
    load(s, 1, [six])
    s.release(1)
    plan, _ = load(s, 2, [eight])
    assert plan.ops[0].kind == H2D


def test_confirm_demotes_a_constructed_collision():
    from test_oracle_fingerprint import colliding_pair
    a, b = colliding_pair(seed=21, words=8)
    a = np.frombuffer(a, dtype=np.uint8).copy()
    b = np.frombuffer(b, dtype=np.uint8).copy()
    s = ReuseStoreOracle(1 << 16, 256)
    load(s, 1, [a])
    s.release(1)
    host, offs = pack([b])
    trusting = s.plan(2, descs([b], offs), host, confirm=False)
    careful = s.plan(2, descs([b], offs), host, confirm=True)
    assert trusting.ops[0].kind == REUSE       # fingerprint alone is fooled
    assert careful.ops[0].kind == H2D          # bytes differ: transferred


def test_release_keeps_tensors_matchable_until_evicted():
    rnd = random.Random(5)
    s = ReuseStoreOracle(1 << 16, 256)
    t = rand_bytes(rnd, 2048)
    load(s, 1, [t])
    with pytest.raises(ValueError):
        load(s, 1, [t])                        # model 1 is still active
    s.release(1)
    assert all(not e.active for e in s.entries)
    plan, _ = load(s, 2, [t])
    assert plan.ops[0].kind == REUSE
    s.release(2, evict=True)
    s.release(1, evict=True)
    assert s.regions == [[0, 1 << 16, True]]
    plan, _ = load(s, 3, [t])
    assert plan.ops[0].kind == H2D
    with pytest.raises(KeyError):
        s.release(77)


def test_no_space_and_stale_plan():
    rnd = random.Random(6)
    s = ReuseStoreOracle(2048, 256)
    load(s, 1, [rand_bytes(rnd, 512)])
    load(s, 2, [rand_bytes(rnd, 512)])
    load(s, 3, [rand_bytes(rnd, 512)])
    s.release(2, evict=True)                   # free: [512,1024) and [1536,2048)
    big = [rand_bytes(rnd, 1000)]              # 1024 free in total, but split
    host, offs = pack(big)
    before = [list(r) for r in s.regions]
    with pytest.raises(NoSpace):
        s.plan(4, descs(big, offs), host)
    assert s.regions == before
    ok = [rand_bytes(rnd, 400)]
    host, offs = pack(ok)
    plan = s.plan(4, descs(ok, offs), host)
    s.release(1)                               # pool changes after planning
    with pytest.raises(StalePlan):
        s.assemble(plan, host)


def test_reuse_size_counts_resident_bytes():
    rnd = random.Random(7)
    s = ReuseStoreOracle(1 << 16, 256)
    a = [rand_bytes(rnd, 1000), rand_bytes(rnd, 2000)]
    load(s, 1, a)
    s.release(1)
    b = [a[1], rand_bytes(rnd, 300)]
    host, offs = pack(b)
    assert s.reuse_size(descs(b, offs)) == 2000

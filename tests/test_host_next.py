"""Host logic of eviction, packing and alias mode through the C ABI (CPU).

Every plan the library makes is compared with the oracle's: rows, evicted
offsets in order, moves in order, totals; then both sides commit and their
pool statistics must agree.  tg_commit installs the metadata (no device).
"""
import random

import pytest

from oracle import NoSpace, ReuseStoreOracle
from paper_2512_01357_amd import tangram as tg

FAKE_BASE = 1 << 40
FAKE_HOST = 1 << 41
U = 256


def flags_of(evict=False, merge=False, alias=False, pack_text=False, cap_text=False):
    return (tg.TG_PLAN_EVICT if evict else 0) | (tg.TG_PLAN_MERGE if merge else 0) | \
        (tg.TG_PLAN_ALIAS if alias else 0) | (tg.TG_PLAN_PACK_TEXT if pack_text else 0) | \
        (tg.TG_PLAN_CAP_TEXT if cap_text else 0)


def plan_both(pool, store, mid, tensors, host_bytes, **fl):
    desc = tg.ModelDesc(mid, FAKE_HOST, host_bytes, tensors)
    try:
        oplan = store.plan(mid, tensors, **fl)
    except NoSpace:
        oplan = None
    try:
        lplan = tg.tg_plan(pool, desc, flags_of(**fl))
    except tg.TgError as e:
        assert e.status == tg.TG_ERR_NOSPACE
        lplan = None
    assert (lplan is None) == (oplan is None), "one side found space, the other did not"
    if lplan is None:
        return None, None
    rows, reused, transfer = tg.tg_plan_ops(lplan)
    assert rows == [(op.kind, op.dst_off, op.src_off, op.nbytes) for op in oplan.ops]
    info = tg.tg_plan_info(lplan)
    assert info["reused_bytes"] == reused == oplan.reused_bytes
    assert info["transfer_bytes"] == transfer == oplan.transfer_bytes
    assert tg.tg_plan_evictions(lplan) == [e.off for e in oplan.evictions]
    assert tg.tg_plan_moves(lplan) == [(old, new, e.nbytes) for e, old, new in oplan.moves]
    assert info["n_evictions"] == len(oplan.evictions) and info["evicted_bytes"] == oplan.evicted_bytes
    assert info["n_moves"] == len(oplan.moves) and info["moved_bytes"] == oplan.moved_bytes
    assert info["merge_bound"] == oplan.merge_bound
    assert info["alias"] == (1 if fl.get("alias") else 0)
    assert info["copy_bytes"] == (0 if fl.get("alias") else oplan.reused_bytes)
    return lplan, oplan


def same_stats(pool, store):
    """Counters, the whole Region List and the whole Tensor Mapping, row by row."""
    a, b = tg.tg_pool_stats(pool), store.stats()
    for k, v in b.items():
        assert a[k] == v, k
    assert tg.tg_pool_regions(pool) == [(off, length, bool(free)) for off, length, free in store.regions]
    assert tg.tg_pool_entries(pool) == sorted((e.off, e.nbytes, e.fp, len(e.owners), e.active_refs)
                                              for e in store.entries)


def layout_rows(sizes, contents):
    rows, at = [], 0
    for n, c in zip(sizes, contents):
        rows.append((n, random.Random("c%s" % (c,)).getrandbits(64), at))
        at += (n + 255) // 256 * 256
    return rows, max(at, 256)


def test_hand_derived_eviction_and_merge_examples():
    # the eviction example of the oracle's pins, through the library
    pool = tg.tg_pool_create(FAKE_BASE, 16 * U, 256)
    store = ReuseStoreOracle(16 * U)
    for mid, sizes in ((1, [1024, 512]), (2, [768, 256]), (3, [512])):
        rows, hb = layout_rows(sizes, [(mid, i) for i in range(len(sizes))])
        lp, op = plan_both(pool, store, mid, rows, hb)
        tg.tg_commit(pool, lp, len(rows))
        store.assemble(op)
        tg.tg_plan_free(lp)
        tg.tg_release(pool, mid, 0)
        store.release(mid)
    for side in (lambda m, p, b, a: tg.tg_set_model_cost(pool, m, p, b, a), store.set_model_cost):
        side(1, 0.5, 2.0, 1.0)
        side(2, 1.0, 1.0, 0.1)
    rows, hb = layout_rows([1024, 1024], ["n0", "n1"])
    lp, op = plan_both(pool, store, 9, rows, hb, evict=True)
    assert tg.tg_plan_evictions(lp) == [2304, 1536]
    tg.tg_commit(pool, lp, 2)
    store.assemble(op)
    tg.tg_plan_free(lp)
    same_stats(pool, store)
    # second round of the same example: model 3 now costs 153.6, model 1's tensors 256 and 128
    tg.tg_set_model_cost(pool, 3, 0.3, 1.0, 1.0)
    store.set_model_cost(3, 0.3, 1.0, 1.0)
    rows, hb = layout_rows([512], ["n2"])
    lp, op = plan_both(pool, store, 10, rows, hb, evict=True)
    assert tg.tg_plan_evictions(lp) == [1024] and tg.tg_plan_ops(lp)[0][0][1] == 1024
    tg.tg_commit(pool, lp, 1)
    store.assemble(op)
    tg.tg_plan_free(lp)
    same_stats(pool, store)
    with pytest.raises(tg.TgError) as e:
        tg.tg_release(pool, 2, 0)
    assert e.value.status == tg.TG_ERR_NOTFOUND
    with pytest.raises(tg.TgError) as e:
        tg.tg_set_model_cost(pool, 1, 0.5, 0.0, 1.0)
    assert e.value.status == tg.TG_ERR_INVALID
    tg.tg_pool_destroy(pool)

    # the merge example: F4 a2 F4 B6 F4 c1 F4 d1 F4
    pool = tg.tg_pool_create(FAKE_BASE, 30 * U, 256)
    store = ReuseStoreOracle(30 * U)
    layout = [(4, False), (2, True), (4, False), (6, True), (4, False), (1, True), (4, False),
              (1, True), (4, False)]
    for i, (units, keep) in enumerate(layout):
        rows, hb = layout_rows([units * U], [("L", i)])
        lp, op = plan_both(pool, store, 100 + i, rows, hb)
        tg.tg_commit(pool, lp, 1)
        store.assemble(op)
        tg.tg_plan_free(lp)
        tg.tg_release(pool, 100 + i, 0)
        store.release(100 + i)
    for i, (units, keep) in enumerate(layout):
        if not keep:
            tg.tg_release(pool, 100 + i, tg.TG_RELEASE_EVICT)
            store.release(100 + i, evict=True)
    rows, hb = layout_rows([6 * U, 5 * U - 7], ["m0", "m1"])
    lp, op = plan_both(pool, store, 9, rows, hb, merge=True)
    assert tg.tg_plan_moves(lp) == [(4 * U, 0, 2 * U), (20 * U, 16 * U, U), (25 * U, 17 * U, U)]
    assert tg.tg_plan_info(lp)["merge_bound"] == 4 * U
    assert [r[1] // U for r in tg.tg_plan_ops(lp)[0]] == [18, 2]
    tg.tg_commit(pool, lp, 2)
    store.assemble(op)
    tg.tg_plan_free(lp)
    same_stats(pool, store)
    tg.tg_pool_destroy(pool)

    # a subspace begins and ends with a free region: a2 F3 b1 F3 c2 and a tensor of 5 move b only
    pool = tg.tg_pool_create(FAKE_BASE, 11 * U, 256)
    store = ReuseStoreOracle(11 * U)
    layout = [(2, True), (3, False), (1, True), (3, False), (2, True)]
    for i, (units, keep) in enumerate(layout):
        rows, hb = layout_rows([units * U], [("S", i)])
        lp, op = plan_both(pool, store, 100 + i, rows, hb)
        tg.tg_commit(pool, lp, 1)
        store.assemble(op)
        tg.tg_plan_free(lp)
        tg.tg_release(pool, 100 + i, 0)
        store.release(100 + i)
    for i, (units, keep) in enumerate(layout):
        if not keep:
            tg.tg_release(pool, 100 + i, tg.TG_RELEASE_EVICT)
            store.release(100 + i, evict=True)
    rows, hb = layout_rows([5 * U], ["s0"])
    lp, op = plan_both(pool, store, 9, rows, hb, merge=True)
    assert tg.tg_plan_moves(lp) == [(5 * U, 2 * U, U)]
    assert tg.tg_plan_info(lp)["merge_bound"] == U
    assert [r[1] // U for r in tg.tg_plan_ops(lp)[0]] == [3]
    tg.tg_commit(pool, lp, 1)
    store.assemble(op)
    tg.tg_plan_free(lp)
    same_stats(pool, store)
    tg.tg_pool_destroy(pool)


def test_abandoned_plan_keeps_its_evictions_and_moves_only():
    # F4 a2 F4 B6 F4 c1 F4 d1 F4 again: the merge happens, the model does not arrive
    pool = tg.tg_pool_create(FAKE_BASE, 30 * U, 256)
    layout = [(4, False), (2, True), (4, False), (6, True), (4, False), (1, True), (4, False),
              (1, True), (4, False)]
    kept = {}
    for i, (units, keep) in enumerate(layout):
        rows, hb = layout_rows([units * U], [("L", i)])
        lp = tg.tg_plan(pool, tg.ModelDesc(100 + i, FAKE_HOST, hb, rows), 0)
        tg.tg_commit(pool, lp, 1)
        tg.tg_plan_free(lp)
        tg.tg_release(pool, 100 + i, 0)
        if keep:
            kept[100 + i] = (rows, hb)
    for i, (units, keep) in enumerate(layout):
        if not keep:
            tg.tg_release(pool, 100 + i, tg.TG_RELEASE_EVICT)
    rows, hb = layout_rows([6 * U, 5 * U - 7], ["m0", "m1"])
    lp = tg.tg_plan(pool, tg.ModelDesc(9, FAKE_HOST, hb, rows), tg.TG_PLAN_MERGE)
    stale = tg.tg_plan(pool, tg.ModelDesc(10, FAKE_HOST, hb, rows), tg.TG_PLAN_MERGE)
    assert tg.tg_plan_moves(lp) == [(4 * U, 0, 2 * U), (20 * U, 16 * U, U), (25 * U, 17 * U, U)]
    before = tg.tg_pool_stats(pool)
    tg.tg_abandon(pool, lp)
    after = tg.tg_pool_stats(pool)
    assert after["free_bytes"] == before["free_bytes"] and after["n_entries"] == before["n_entries"] == 4
    assert after["generation"] == before["generation"] + 1 and after["n_active"] == 0
    # regions now: a2 F8 B6 c1 d1 F12
    assert after["n_free_regions"] == 2 and after["largest_free"] == 12 * U
    with pytest.raises(tg.TgError) as e:
        tg.tg_abandon(pool, lp)
    assert e.value.status == tg.TG_ERR_INVALID
    with pytest.raises(tg.TgError) as e:
        tg.tg_abandon(pool, stale)
    assert e.value.status == tg.TG_ERR_STALE
    tg.tg_plan_free(lp)
    tg.tg_plan_free(stale)
    with pytest.raises(tg.TgError) as e:
        tg.tg_release(pool, 9, 0)
    assert e.value.status == tg.TG_ERR_NOTFOUND
    # the survivors are found where the moves put them
    want = {101: 0, 103: 10 * U, 105: 16 * U, 107: 17 * U}
    for mid, (r, h) in kept.items():
        lp = tg.tg_plan(pool, tg.ModelDesc(mid, FAKE_HOST, h, r), tg.TG_PLAN_ALIAS)
        assert tg.tg_plan_ops(lp)[0] == [(tg.TG_OP_REUSE, want[mid], want[mid], r[0][0])]
        tg.tg_plan_free(lp)
    tg.tg_pool_destroy(pool)


def test_unknown_flag_bits_are_refused():
    pool = tg.tg_pool_create(FAKE_BASE, 4096, 256)
    with pytest.raises(tg.TgError) as e:
        tg.tg_plan(pool, tg.ModelDesc(1, FAKE_HOST, 4096, [(512, 1, 0)]), 64)
    assert e.value.status == tg.TG_ERR_INVALID
    tg.tg_pool_destroy(pool)


def history(seed):
    rnd = random.Random(500 + seed)
    align = [256, 256, 16, 4096][seed % 4]
    cap = align * rnd.choice([96, 160, 400]) * (256 // min(align, 256))
    pool = tg.tg_pool_create(FAKE_BASE, cap, align)
    store = ReuseStoreOracle(cap, align)
    contents = [(rnd.choice([40, 256, 300, 512, 1000, 1024, 2048, 3000, 6000]), i) for i in range(30)]
    running, retained, next_id = [], [], 1
    n_evict = n_move = n_alias = 0
    for _ in range(220):
        r = rnd.random()
        if r < 0.5 or not (running or retained):
            picks = [contents[rnd.randrange(30)] for _ in range(rnd.randrange(1, 8))]
            rows, hb = layout_rows([p[0] for p in picks], [p[1] for p in picks])
            fl = dict(evict=rnd.random() < 0.7, merge=rnd.random() < 0.7, alias=rnd.random() < 0.5,
                      pack_text=rnd.random() < 0.5, cap_text=rnd.random() < 0.3)
            mid = next_id
            if retained and rnd.random() < 0.25:
                mid = rnd.choice(retained)
            if rnd.random() < 0.3:
                cost = (rnd.choice([0.1, 0.5, 1.0]), rnd.choice([1.0, 3.0, 57e9]), rnd.choice([1.0, 0.3]))
                tg.tg_set_model_cost(pool, mid, *cost)
                store.set_model_cost(mid, *cost)
            lp, op = plan_both(pool, store, mid, rows, hb, **fl)
            if lp is None:
                same_stats(pool, store)
                continue
            n_evict += len(op.evictions)
            n_move += len(op.moves)
            n_alias += sum(1 for h in op.hits if h is not None) if fl["alias"] else 0
            if rnd.random() < 0.1:
                tg.tg_plan_free(lp)
            elif mid == next_id and rnd.random() < 0.12:
                # giving a plan up == carrying it out and evicting the (new) model at once
                tg.tg_abandon(pool, lp)
                store.assemble(op)
                store.release(mid, True)
                with pytest.raises(tg.TgError) as e:
                    tg.tg_commit(pool, lp, len(rows))
                assert e.value.status == tg.TG_ERR_INVALID
                tg.tg_plan_free(lp)
                next_id += 1
            else:
                ptrs = tg.tg_commit(pool, lp, len(rows))
                dsts = store.assemble(op)
                assert ptrs == [FAKE_BASE + d for d in dsts]
                tg.tg_plan_free(lp)
                running.append(mid)
                if mid in retained:
                    retained.remove(mid)
                if mid == next_id:
                    next_id += 1
        else:
            if running and (not retained or rnd.random() < 0.6):
                mid = rnd.choice(running)
                evict = rnd.random() < 0.4
                tg.tg_release(pool, mid, tg.TG_RELEASE_EVICT if evict else 0)
                store.release(mid, evict)
                running.remove(mid)
                if not evict:
                    retained.append(mid)
            else:
                mid = rnd.choice(retained)
                if mid in store.models:
                    tg.tg_release(pool, mid, tg.TG_RELEASE_EVICT)
                    store.release(mid, True)
                else:
                    with pytest.raises(tg.TgError) as e:
                        tg.tg_release(pool, mid, tg.TG_RELEASE_EVICT)
                    assert e.value.status == tg.TG_ERR_NOTFOUND
                retained.remove(mid)
        retained = [m for m in retained if m in store.models]
        same_stats(pool, store)
    tg.tg_pool_destroy(pool)
    return n_evict, n_move, n_alias


@pytest.mark.parametrize("seed", range(16))
def test_random_histories_with_every_flag_match_the_oracle(seed):
    history(seed)


def test_the_random_histories_exercise_every_stage():
    totals = [0, 0, 0]
    for seed in range(16, 40):
        for i, v in enumerate(history(seed)):
            totals[i] += v
    assert all(t > 20 for t in totals), totals

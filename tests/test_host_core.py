"""Host logic of the library through the C ABI, on the CPU (no kernel runs).

Plans of the library are compared row by row with the oracle's on random
histories and on all five workload shapes; error paths are forced from the
host.  The pool base is a made-up aligned address: nothing here touches
device memory.
"""
import os
import random
import re

import pytest

from oracle import NoSpace, ReuseStoreOracle
from paper_2512_01357_amd import synth
from paper_2512_01357_amd import tangram as tg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE_BASE = 1 << 40
FAKE_HOST = 1 << 41


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "tangram.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(tg_[a-z_0-9]+)\s*\(", header))
    assert declared, "no declarations found"
    lib = tg.lib()
    for name in sorted(declared):
        assert hasattr(lib, name), name
    assert declared == set(tg.EXPORTS)


def test_strerror_names_every_status():
    names = {tg.tg_strerror(s) for s in range(0, -8, -1)}
    assert len(names) == 8
    assert tg.tg_strerror(-99) == "unknown status"


def test_pool_create_argument_checks():
    for base, cap, align in [(0, 4096, 256), (FAKE_BASE, 0, 256), (FAKE_BASE, 4096, 8),
                             (FAKE_BASE, 4096, 48), (FAKE_BASE + 16, 4096, 256),
                             (FAKE_BASE, 4096 + 16, 256)]:
        with pytest.raises(tg.TgError) as e:
            tg.tg_pool_create(base, cap, align)
        assert e.value.status == tg.TG_ERR_INVALID
    p = tg.tg_pool_create(FAKE_BASE, 4096, 16)
    st = tg.tg_pool_stats(p)
    assert st["capacity"] == 4096 and st["free_bytes"] == 4096 and st["n_regions"] == 1
    tg.tg_pool_destroy(p)


def fake_fp(key) -> int:
    # stands in for a content fingerprint in metadata-only tests: equal
    # content keys <=> equal values
    return random.Random(repr(key)).getrandbits(64)


def rows_of(plan):
    rows, reused, transfer = tg.tg_plan_ops(plan)
    return rows, reused, transfer


def both_plan(pool, store, model_id, tensors, host_bytes):
    """Plan on both sides; returns (library plan handle or None, oracle plan or None)."""
    desc = tg.ModelDesc(model_id, FAKE_HOST, host_bytes, tensors)
    try:
        oplan = store.plan(model_id, tensors)
    except NoSpace:
        oplan = None
    try:
        lplan = tg.tg_plan(pool, desc)
    except tg.TgError as e:
        assert e.status == tg.TG_ERR_NOSPACE
        lplan = None
    assert (lplan is None) == (oplan is None)
    return lplan, oplan, desc


def assert_same_plan(lplan, oplan):
    rows, reused, transfer = rows_of(lplan)
    assert rows == [(op.kind, op.dst_off, op.src_off, op.nbytes) for op in oplan.ops]
    assert reused == oplan.reused_bytes and transfer == oplan.transfer_bytes


def assert_same_stats(pool, store):
    """Counters, the whole Region List and the whole Tensor Mapping, row by row."""
    a, b = tg.tg_pool_stats(pool), store.stats()
    for k, v in b.items():
        assert a[k] == v, k
    assert tg.tg_pool_regions(pool) == [(off, length, bool(free)) for off, length, free in store.regions]
    assert tg.tg_pool_entries(pool) == sorted((e.off, e.nbytes, e.fp, len(e.owners), e.active_refs)
                                              for e in store.entries)


@pytest.mark.parametrize("seed", range(10))
def test_random_histories_match_the_oracle(seed):
    rnd = random.Random(seed)
    cap = 256 * rnd.choice([64, 200, 1000])
    pool = tg.tg_pool_create(FAKE_BASE, cap, 256)
    store = ReuseStoreOracle(cap, 256)
    contents = [(rnd.choice([8, 100, 256, 257, 512, 700, 1024, 3000, 5000, 20000]), i) for i in range(25)]
    live, next_id = [], 1
    for _ in range(150):
        r = rnd.random()
        if r < 0.5 or not live:
            picks = [contents[rnd.randrange(25)] for _ in range(rnd.randrange(1, 9))]
            tensors, at = [], 0
            for nbytes, cid in picks:
                tensors.append((nbytes, fake_fp(("c", cid)), at))
                at += (nbytes + 255) // 256 * 256
            lplan, oplan, _ = both_plan(pool, store, next_id, tensors, at)
            if lplan is None:
                assert_same_stats(pool, store)
                continue
            assert_same_plan(lplan, oplan)
            if rnd.random() < 0.15:
                tg.tg_plan_free(lplan)          # planned but never carried out
            else:
                ptrs = tg.tg_commit(pool, lplan, len(tensors))
                dsts = store.assemble(oplan)
                assert ptrs == [FAKE_BASE + d for d in dsts]
                tg.tg_plan_free(lplan)
                live.append(next_id)
            next_id += 1
        else:
            mid = rnd.choice(live)
            evict = rnd.random() < 0.6
            tg.tg_release(pool, mid, tg.TG_RELEASE_EVICT if evict else 0)
            store.release(mid, evict)
            if evict:
                live.remove(mid)
        assert_same_stats(pool, store)
    tg.tg_pool_destroy(pool)


def workload_descs(w, name):
    spec = w.models[name]
    offs = synth.layout(spec, w.align)
    return [(t.nbytes, fake_fp(synth.content_key(t)), o) for t, o in zip(spec.tensors, offs)], \
        synth.host_bytes(spec, w.align)


def replay(w):
    pool = tg.tg_pool_create(FAKE_BASE, w.pool_bytes, w.align)
    store = ReuseStoreOracle(w.pool_bytes, w.align)
    out = {}

    def load(name):
        tensors, hb = workload_descs(w, name)
        mid = w.models[name].model_id
        lplan, oplan, _ = both_plan(pool, store, mid, tensors, hb)
        assert lplan is not None, "workload must fit its pool"
        assert_same_plan(lplan, oplan)
        tg.tg_commit(pool, lplan, len(tensors))
        store.assemble(oplan)
        tg.tg_plan_free(lplan)
        return oplan

    for act in w.setup:
        if act[0] == "load":
            load(act[1])
        else:
            tg.tg_release(pool, w.models[act[1]].model_id, tg.TG_RELEASE_EVICT if act[2] else 0)
            store.release(w.models[act[1]].model_id, act[2])
        assert_same_stats(pool, store)
    out["stats_before"] = store.stats()

    def evict(name):
        mid = w.models[name].model_id
        tg.tg_release(pool, mid, tg.TG_RELEASE_EVICT)
        store.release(mid, True)

    if w.streamed:
        # the parts of one model are loaded one after the other, then all released
        for name in w.loads:
            out[name] = load(name)
            assert_same_stats(pool, store)
        for name in w.loads:
            evict(name)
        assert store.stats() == out["stats_before"]
        assert_same_stats(pool, store)
    else:
        for name in w.loads:
            out[name] = load(name)
            assert_same_stats(pool, store)
            evict(name)
            assert store.stats() == out["stats_before"]
            assert_same_stats(pool, store)
    tg.tg_pool_destroy(pool)
    return out


def test_plan_parity_tiny_and_1b():
    out = replay(synth.workload_tiny())
    plan = out["B"]
    assert sum(1 for op in plan.ops if op.kind == 0) == 39
    out = replay(synth.workload_gpt1b())
    plan = out["M"]
    n_reuse = sum(1 for op in plan.ops if op.kind == 0)
    # designated 146 shared tensors, plus the norm gains (all ones) of the odd layers
    assert n_reuse == 146 + 12 * 2 + 1
    assert plan.reused_bytes + plan.transfer_bytes == synth.workload_gpt1b().models["M"].nbytes


def test_plan_parity_llama7b_family():
    w = synth.workload_llama7b()
    out = replay(w)
    for v in ("v1", "v2", "v3"):
        plan = out[v]
        assert plan.reused_bytes + plan.transfer_bytes == w.models[v].nbytes
        shared_bytes = sum(t.nbytes for t, b in zip(w.models[v].tensors, w.models["base"].tensors)
                           if synth.content_key(t) == synth.content_key(b))
        assert plan.reused_bytes == shared_bytes
        assert 0.5 < plan.reused_bytes / w.models[v].nbytes < 0.55


def test_plan_parity_neox20b_fragmented_pool():
    w = synth.workload_neox20b()
    out = replay(w)
    plan = out["M20"]
    st = out["stats_before"]
    assert st["n_free_regions"] >= 5, "the pool must be fragmented before the load"
    frac = sum(1 for op in plan.ops if op.kind == 0)
    assert frac >= w.designated_shared["M20"]
    assert 0.29 < w.designated_shared["M20"] / len(plan.ops) < 0.31
    # the load used more than one free region
    regions_used = set()
    holes = sorted(op.dst_off for op in plan.ops)
    assert holes[0] < st["capacity"] - st["largest_free"]


@pytest.mark.parametrize("reuse", [0.0, 0.5, 0.9])
def test_plan_parity_llama70b(reuse):
    w = synth.workload_llama70b(reuse, 272 * 10**9)
    out = replay(w)
    total = sum(w.models[n].nbytes for n in w.loads)
    reused = sum(out[n].reused_bytes for n in w.loads)
    transfer = sum(out[n].transfer_bytes for n in w.loads)
    assert len(w.loads) == 3 and sum(len(w.models[n].tensors) for n in w.loads) == 723
    assert reused + transfer == total
    assert 141.0e9 < total < 141.2e9
    # the parts hold every tensor once, fit the Model Cache, and each has its share of the transfers
    names = [t.name for n in w.loads for t in w.models[n].tensors]
    assert len(set(names)) == 723
    assert all(w.models[n].nbytes <= 50 * 10**9 for n in w.loads)
    if reuse < 1.0:
        share = [out[n].transfer_bytes / transfer for n in w.loads]
        assert min(share) > 0.2, share
    if reuse == 0.0:
        # nothing designated; later parts still find the all-ones norm gains of earlier parts
        assert reused == sum(t.nbytes for n in w.loads[1:] for t in w.models[n].tensors if t.kind == "ones")
    else:
        assert abs(reused / total - reuse) < 0.02


def test_error_paths_leave_the_pool_unchanged():
    pool = tg.tg_pool_create(FAKE_BASE, 2048, 256)
    t = [(512, 1, 0)]
    # invalid descriptors
    for tensors, hb in [([(0, 1, 0)], 4096), ([(512, 1, 4000)], 4096), ([], 4096)]:
        with pytest.raises(tg.TgError) as e:
            tg.tg_plan(pool, tg.ModelDesc(1, FAKE_HOST, hb, tensors))
        assert e.value.status == tg.TG_ERR_INVALID
    before = tg.tg_pool_stats(pool)
    # too large
    with pytest.raises(tg.TgError) as e:
        tg.tg_plan(pool, tg.ModelDesc(1, FAKE_HOST, 1 << 20, [(4096, 1, 0)]))
    assert e.value.status == tg.TG_ERR_NOSPACE
    assert tg.tg_pool_stats(pool) == before
    # stale plan
    p1 = tg.tg_plan(pool, tg.ModelDesc(1, FAKE_HOST, 4096, t))
    p2 = tg.tg_plan(pool, tg.ModelDesc(2, FAKE_HOST, 4096, t))
    tg.tg_commit(pool, p1, 1)
    with pytest.raises(tg.TgError) as e:
        tg.tg_commit(pool, p2, 1)
    assert e.value.status == tg.TG_ERR_STALE
    # a plan is carried out once
    with pytest.raises(tg.TgError) as e:
        tg.tg_commit(pool, p1, 1)
    assert e.value.status == tg.TG_ERR_INVALID
    # model 1 is active: planning it again is refused
    with pytest.raises(tg.TgError) as e:
        tg.tg_plan(pool, tg.ModelDesc(1, FAKE_HOST, 4096, t))
    assert e.value.status == tg.TG_ERR_INVALID
    # unknown model
    with pytest.raises(tg.TgError) as e:
        tg.tg_release(pool, 77, 0)
    assert e.value.status == tg.TG_ERR_NOTFOUND
    # a plan belongs to its pool
    other = tg.tg_pool_create(FAKE_BASE, 2048, 256)
    p3 = tg.tg_plan(other, tg.ModelDesc(5, FAKE_HOST, 4096, t))
    with pytest.raises(tg.TgError) as e:
        tg.tg_commit(pool, p3, 1)
    assert e.value.status == tg.TG_ERR_INVALID
    for p in (p1, p2, p3):
        tg.tg_plan_free(p)
    tg.tg_pool_destroy(other)
    tg.tg_pool_destroy(pool)


def test_reuse_size_and_load_time_estimate():
    pool = tg.tg_pool_create(FAKE_BASE, 1 << 20, 256)
    store = ReuseStoreOracle(1 << 20, 256)
    a = [(1000, 11, 0), (2000, 12, 1024), (512, 13, 4096)]
    p = tg.tg_plan(pool, tg.ModelDesc(1, FAKE_HOST, 8192, a))
    tg.tg_commit(pool, p, 3)
    tg.tg_plan_free(p)
    store.assemble(store.plan(1, a))
    tg.tg_release(pool, 1, 0)
    store.release(1)
    b = [(2000, 12, 0), (300, 14, 2048), (512, 13, 4096), (999, 11, 5000)]
    desc = tg.ModelDesc(2, FAKE_HOST, 8192, b)
    reuse, est = tg.tg_reuse_size(pool, desc, 50e9)
    assert reuse == store.reuse_size(b) == 2512
    # Eq. 3: (S - S') / B
    assert est == pytest.approx((2000 + 300 + 512 + 999 - 2512) / 50e9)
    tg.tg_pool_destroy(pool)


def test_device_calls_fail_loudly_without_a_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(tg.TgError) as e:
        tg.tg_fingerprint([(FAKE_BASE, 4096)])
    assert e.value.status in (tg.TG_ERR_HIP, tg.TG_ERR_NOMEM)
    with pytest.raises(tg.TgError) as e:
        tg.tg_fingerprint([(FAKE_BASE + 8, 4096)])
    assert e.value.status == tg.TG_ERR_INVALID
    # nothing was allocated: shutting down (twice) is harmless, and so are the host-only calls after it
    tg.tg_shutdown()
    tg.tg_shutdown()
    with pytest.raises(tg.TgError) as e:
        tg.tg_compare([(FAKE_BASE, FAKE_BASE, 64)])
    assert e.value.status in (tg.TG_ERR_HIP, tg.TG_ERR_NOMEM)
    pool = tg.tg_pool_create(FAKE_BASE, 4096, 256)
    lp = tg.tg_plan(pool, tg.ModelDesc(1, FAKE_HOST, 4096, [(512, 7, 0)]), 0)
    with pytest.raises(tg.TgError) as e:
        tg.tg_assemble(pool, lp, 1, 0, None, None)          # needs the device: refused, pool untouched
    assert e.value.status in (tg.TG_ERR_HIP, tg.TG_ERR_NOMEM)
    assert tg.tg_pool_stats(pool)["n_entries"] == 0
    tg.tg_commit(pool, lp, 1)
    tg.tg_plan_free(lp)
    tg.tg_pool_destroy(pool)

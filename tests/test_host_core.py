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
    """Plan on both sides; returns (library plan handle or None, oracle plan or None).
    host_bytes None: the model has no host image (only rows)."""
    if host_bytes is None:
        desc = tg.ModelDesc(model_id, 0, 0, tensors)
    else:
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
        lplan, oplan, _ = both_plan(pool, store, mid, tensors, None if w.streamed else hb)
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
    """Config 5 is one model of 723 tensors and one plan, made without a host image."""
    w = synth.workload_llama70b(reuse, 272 * 10**9)
    out = replay(w)
    assert w.loads == ["M70"] and len(w.models["M70"].tensors) == 723
    plan = out["M70"]
    total = w.models["M70"].nbytes
    assert plan.reused_bytes + plan.transfer_bytes == total
    assert 141.0e9 < total < 141.2e9
    n_reused = sum(1 for op in plan.ops if op.kind == 0)
    if reuse == 0.0:
        # nothing is resident, so nothing is found: incoming tensors never match each other
        assert n_reused == 0 and plan.reused_bytes == 0 and "sib" not in w.models
    else:
        assert abs(plan.reused_bytes / total - reuse) < 0.02
        # every designated tensor is found, and so are the all-ones norm gains of the other layers
        ones = sum(1 for t, (nm, _, _) in zip(w.models["M70"].tensors, synth.llama_tensors(**synth.LLAMA70B_SHAPES))
                   if t.kind == "ones")
        assert w.designated_shared["M70"] <= n_reused <= w.designated_shared["M70"] + ones


def test_plan_parity_llama70b_sweep_against_one_pool():
    """The benchmark's arrangement: one pool holding the 90 % sibling, the three reuse levels in turn."""
    w = synth.workload_llama70b_sweep(272 * 10**9)
    out = replay(w)
    for name, lo, hi in (("M70-90", 0.88, 0.92), ("M70-50", 0.48, 0.52), ("M70-0", 0.0, 0.0001)):
        plan = out[name]
        total = w.models[name].nbytes
        assert plan.reused_bytes + plan.transfer_bytes == total
        assert lo <= plan.reused_bytes / total <= hi, name


def test_plan_without_a_host_image_and_its_argument_checks():
    pool = tg.tg_pool_create(FAKE_BASE, 1 << 20, 256)
    store = ReuseStoreOracle(1 << 20, 256)
    # src_off is the caller's own reference when there is no image: any value is echoed back
    tensors = [(512, 11, 1 << 50), (700, 12, 7), (512, 11, 99)]
    lplan, oplan, _ = both_plan(pool, store, 1, tensors, None)
    assert_same_plan(lplan, oplan)
    assert [r[2] for r in rows_of(lplan)[0]] == [1 << 50, 7, 99]
    # a whole-image assemble of a plan that has no image is refused before anything happens
    with pytest.raises(tg.TgError) as e:
        tg.tg_assemble(pool, lplan, 3)
    assert e.value.status == tg.TG_ERR_INVALID
    assert_same_stats(pool, store)
    tg.tg_plan_free(lplan)
    # confirmation needs bytes to compare with
    desc = tg.ModelDesc(2, 0, 0, tensors)
    with pytest.raises(tg.TgError) as e:
        tg.tg_plan(pool, desc, tg.TG_PLAN_CONFIRM)
    assert e.value.status == tg.TG_ERR_INVALID
    # a length without a base is a mistake
    bad = tg.ModelDesc(3, 0, 4096, tensors)
    with pytest.raises(tg.TgError) as e:
        tg.tg_plan(pool, bad)
    assert e.value.status == tg.TG_ERR_INVALID
    # the calls of a load in steps need a load that has begun
    lplan = tg.tg_plan(pool, desc)
    for call in (lambda: tg.tg_assemble_wait(pool, lplan, 3), lambda: tg.tg_assemble_feed_wait(pool, lplan, 0),
                 lambda: tg.tg_assemble_feed(pool, lplan, FAKE_HOST, 4096, [(0, 0)])):
        with pytest.raises(tg.TgError) as e:
            call()
        assert e.value.status == tg.TG_ERR_INVALID
    tg.tg_plan_free(lplan)
    tg.tg_pool_destroy(pool)


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

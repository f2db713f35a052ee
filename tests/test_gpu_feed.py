"""GPU parity of the load in steps (tg_assemble_begin / _feed / _wait and
tg_assemble_async), of two pools loading at the same time, and of the kernels
reading pinned host memory in place.  Through the C ABI, against the oracle;
everything is integer or byte work and is compared bit for bit."""
import random
import sys
import threading

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

import oracle  # noqa: E402
from oracle import ReuseStoreOracle  # noqa: E402
from paper_2512_01357_amd import tangram as tg  # noqa: E402
from paper_2512_01357_amd.loader import HostArena, RegisteredModel, ReusePool  # noqa: E402
from gpu_harness import same_pool_state  # noqa: E402

DEV = "cuda:0"
TILE_COPY = 1024 * 16 * 4


def say(msg):
    print("[gpu-test] " + msg, flush=True)
    sys.stdout.flush()


def rbytes(rnd, n):
    return np.random.default_rng(rnd.getrandbits(32)).integers(0, 256, n, dtype=np.uint8)


def pack(tensors, align=256):
    """(host image, offsets) with every tensor on an `align` boundary."""
    offs, at = [], 0
    for t in tensors:
        offs.append(at)
        at += (t.size + align - 1) // align * align
    host = np.zeros(max(at, align), dtype=np.uint8)
    for t, o in zip(tensors, offs):
        host[o:o + t.size] = t
    return host, offs


class Pair:
    """A pool of the library and the oracle's store, driven side by side."""

    def __init__(self, capacity, align=256):
        self.pool = ReusePool(capacity, align, DEV)
        self.store = ReuseStoreOracle(capacity, align)
        self.keep = []

    def rows(self, tensors, offs):
        return [(t.size, oracle.fingerprint(t), o) for t, o in zip(tensors, offs)]

    def load_whole(self, model_id, tensors, verify=True):
        host, offs = pack(tensors)
        arena = HostArena(host.size)
        arena.numpy()[:] = host
        rows = self.rows(tensors, offs)
        reg = RegisteredModel(model_id, arena, offs, [t.size for t in tensors], [r[1] for r in rows])
        oplan = self.store.plan(model_id, rows, host)
        ptrs, info = self.pool.load(reg, verify=verify)
        assert info["ops"] == [(op.kind, op.dst_off, op.src_off, op.nbytes) for op in oplan.ops]
        dsts = self.store.assemble(oplan, host)
        assert ptrs == [self.pool.base + d for d in dsts]
        self.check_image()
        arena.free()
        return oplan

    def check_image(self):
        for e in self.store.entries:
            got = self.pool.slab[e.off:e.off + e.nbytes].cpu().numpy()
            assert got.tobytes() == self.store.image[e.off].tobytes(), (e.off, e.nbytes)
        same_pool_state(self.pool.pool, self.store)

    def release(self, model_id, evict=False):
        self.pool.release(model_id, evict)
        self.store.release(model_id, evict)

    def close(self):
        self.pool.close()


def stream_args(p):
    return dict(stream_gather=p.stream_gather, stream_h2d=p.stream_h2d, stream_h2d_second=p.stream_h2d_second,
                use_second_h2d_stream=p.stream_h2d_second is not None)


SIZES = [1, 7, 16, 24, 255, 256, 257, 4096, 5000, 65536, 65537, TILE_COPY - 8, TILE_COPY, TILE_COPY + 24,
         2 * TILE_COPY, (1 << 20) + 24, 3 * (1 << 20) + 1, 9 << 20, 33 << 20, 70 << 20]


@pytest.mark.parametrize("verify", [True, False])
@pytest.mark.parametrize("seg_mib", [72, 128, 256])
def test_load_in_steps_through_a_small_segment_matches_the_oracle(seg_mib, verify):
    say("begin / feed / wait: segment of %d MiB, verify=%s" % (seg_mib, verify))
    rnd = random.Random(1000 + seg_mib)
    b = Pair(512 << 20)
    a = [rbytes(rnd, n) for n in SIZES]
    b.load_whole(1, a)
    b.release(1)
    # second model: hits (copied device to device) and misses of every size class
    m2 = [a[i] if i % 3 == 0 else rbytes(rnd, SIZES[i]) for i in range(len(SIZES))]
    host, offs = pack(m2)
    rows = b.rows(m2, offs)
    oplan = b.store.plan(2, rows, host)
    # the library plans from rows alone: no host image
    desc = tg.ModelDesc(2, 0, 0, rows)
    plan = tg.tg_plan(b.pool.pool, desc)
    got_rows, reused, transfer = tg.tg_plan_ops(plan)
    assert got_rows == [(op.kind, op.dst_off, op.src_off, op.nbytes) for op in oplan.ops]
    missing = [k for k, op in enumerate(oplan.ops) if op.kind == 1]
    assert missing and len(missing) < len(rows)
    rnd.shuffle(missing)
    seg = HostArena(seg_mib << 20)
    tg.tg_assemble_begin(b.pool.pool, plan, tg.TG_ASSEMBLE_VERIFY if verify else 0, **stream_args(b.pool))
    # while the load is in flight the pool refuses what would change it
    for call in (lambda: tg.tg_release(b.pool.pool, 1, 0), lambda: tg.tg_commit(b.pool.pool, plan, len(rows))):
        with pytest.raises(tg.TgError) as e:
            call()
        assert e.value.status == tg.TG_ERR_INVALID
    feeds = 0
    i = 0
    while i < len(missing):
        seg_rows, at = [], 0
        while i < len(missing):
            k = missing[i]
            # odd phases inside the segment: some small tensors are not 16-byte aligned there
            start = at + (8 if k % 2 else 0)
            if start + SIZES[k] > seg.nbytes:
                break
            seg.numpy()[start:start + SIZES[k]] = m2[k]
            seg_rows.append((k, start))
            at = (start + SIZES[k] + 255) // 256 * 256
            i += 1
        assert seg_rows, "segment too small for a tensor"
        ticket = tg.tg_assemble_feed(b.pool.pool, plan, seg.ptr, seg.nbytes, seg_rows)
        tg.tg_assemble_feed_wait(b.pool.pool, plan, ticket)
        seg.numpy()[:at] = 0xEE                    # the segment is ours again: overwrite it
        feeds += 1
    ptrs = tg.tg_assemble_wait(b.pool.pool, plan, len(rows))
    t = tg.tg_plan_timing(plan)
    tg.tg_plan_free(plan)
    dsts = b.store.assemble(oplan, host)
    assert ptrs == [b.pool.base + d for d in dsts]
    b.check_image()
    assert t["feeds"] == feeds and (feeds >= 2 or seg_mib > 72)
    assert t["h2d_bytes"] + t["gather_bytes"] == sum(op.nbytes for op in oplan.ops)
    # a verifying load fingerprints every tensor once: inside the copy launch or by a launch of its own
    assert t["verify_bytes"] + t["fused_verify_bytes"] == (sum(op.nbytes for op in oplan.ops) if verify else 0)
    assert (t["fused_verify_bytes"] > 0) == verify
    b.release(2, evict=True)
    b.check_image()
    seg.free()
    b.close()


def test_one_half_of_the_segment_is_refilled_while_the_other_is_copied():
    say("begin / feed / wait: two halves, the next piece written while the previous one is in flight")
    rnd = random.Random(4242)
    b = Pair(768 << 20)
    sizes = [33 << 20, 9 << 20, (1 << 20) + 24, 65537, 4096, 70 << 20, 5000, 24, 40 << 20, 3 * (1 << 20) + 1,
             64 << 20, 1, 31 << 20, 65536, 17 << 20]
    a = [rbytes(rnd, n) for n in sizes]
    b.load_whole(1, a)
    b.release(1)
    m2 = [a[i] if i % 4 == 0 else rbytes(rnd, sizes[i]) for i in range(len(sizes))]
    host, offs = pack(m2)
    rows = b.rows(m2, offs)
    oplan = b.store.plan(2, rows, host)
    plan = tg.tg_plan(b.pool.pool, tg.ModelDesc(2, 0, 0, rows))
    missing = [k for k, op in enumerate(oplan.ops) if op.kind == 1]
    half = 72 << 20
    seg = HostArena(2 * half)

    def fill(part, i):
        """Writes as many of missing[i:] as fit into half `part`; returns (rows, next i)."""
        seg_rows, at = [], 0
        while i < len(missing) and at + sizes[missing[i]] <= half:
            k = missing[i]
            seg.numpy()[part * half + at:part * half + at + sizes[k]] = m2[k]
            seg_rows.append((k, at))
            at = (at + sizes[k] + 255) // 256 * 256
            i += 1
        assert seg_rows, "half too small for a tensor"
        return seg_rows, i

    piece, i = fill(0, 0)                              # the cache holds the first piece beforehand
    tg.tg_assemble_begin(b.pool.pool, plan, tg.TG_ASSEMBLE_VERIFY, **stream_args(b.pool))
    feeds = 0
    while piece:
        part = feeds % 2
        ticket = tg.tg_assemble_feed(b.pool.pool, plan, seg.ptr + part * half, half, piece)
        feeds += 1
        # the other half was waited for one turn ago: it may be overwritten while this one is read
        nxt = None
        if i < len(missing):
            seg.numpy()[(1 - part) * half:(2 - part) * half] = 0xEE
            nxt, i = fill(1 - part, i)
        tg.tg_assemble_feed_wait(b.pool.pool, plan, ticket)
        piece = nxt
    ptrs = tg.tg_assemble_wait(b.pool.pool, plan, len(rows))
    t = tg.tg_plan_timing(plan)
    tg.tg_plan_free(plan)
    assert ptrs == [b.pool.base + d for d in b.store.assemble(oplan, host)]
    b.check_image()
    assert t["feeds"] == feeds and feeds >= 4
    seg.free()
    b.close()


def test_mistakes_in_a_load_in_steps_end_it_and_leave_the_pool_as_it_was():
    say("begin / feed / wait: error paths")
    rnd = random.Random(77)
    b = Pair(64 << 20)
    a = [rbytes(rnd, n) for n in (4096, 1 << 20, 300000)]
    b.load_whole(1, a)
    b.release(1)
    m2 = [a[0], rbytes(rnd, 1 << 20), rbytes(rnd, 70000), rbytes(rnd, 512)]
    host, offs = pack(m2)
    rows = b.rows(m2, offs)
    desc = tg.ModelDesc(2, 0, 0, rows)
    seg = HostArena(host.size)
    seg.numpy()[:] = host
    args = stream_args(b.pool)

    def begin():
        plan = tg.tg_plan(b.pool.pool, desc)
        tg.tg_assemble_begin(b.pool.pool, plan, tg.TG_ASSEMBLE_VERIFY, **args)
        return plan

    bad_feeds = [
        [(0, offs[0])],                              # a tensor the plan reuses is not a transfer
        [(9, 0)],                                    # no such tensor
        [(1, seg.nbytes - 100)],                     # reaches past the segment
        [(1, offs[1]), (1, offs[1])],                # twice in one feed
    ]
    for rows_bad in bad_feeds:
        plan = begin()
        with pytest.raises(tg.TgError) as e:
            tg.tg_assemble_feed(b.pool.pool, plan, seg.ptr, seg.nbytes, rows_bad)
        assert e.value.status == tg.TG_ERR_INVALID
        # a refused feed changes nothing: the load goes on and can still be completed
        tg.tg_assemble_feed(b.pool.pool, plan, seg.ptr, seg.nbytes, [(k, offs[k]) for k in (1, 2, 3)])
        with pytest.raises(tg.TgError) as e:
            tg.tg_assemble_feed(b.pool.pool, plan, seg.ptr, seg.nbytes, [(2, offs[2])])      # fed before
        assert e.value.status == tg.TG_ERR_INVALID
        ptrs = tg.tg_assemble_wait(b.pool.pool, plan, 4)
        tg.tg_plan_free(plan)
        oplan = b.store.plan(2, rows, host)
        dsts = b.store.assemble(oplan, host)
        assert ptrs == [b.pool.base + d for d in dsts]
        b.check_image()
        b.release(2, evict=True)
    # waiting with a tensor that was never handed over: INVALID, nothing committed, pool as before
    plan = begin()
    tg.tg_assemble_feed(b.pool.pool, plan, seg.ptr, seg.nbytes, [(1, offs[1])])
    with pytest.raises(tg.TgError) as e:
        tg.tg_assemble_wait(b.pool.pool, plan, 4)
    assert e.value.status == tg.TG_ERR_INVALID
    with pytest.raises(tg.TgError) as e:             # the load has ended
        tg.tg_assemble_feed(b.pool.pool, plan, seg.ptr, seg.nbytes, [(2, offs[2])])
    assert e.value.status == tg.TG_ERR_INVALID
    tg.tg_plan_free(plan)
    b.check_image()
    # a second load cannot begin while one is in flight; freeing a plan in flight ends its load
    plan = begin()
    other = tg.tg_plan(b.pool.pool, tg.ModelDesc(3, 0, 0, rows[1:2]))
    with pytest.raises(tg.TgError) as e:
        tg.tg_assemble_begin(b.pool.pool, other, 0, **args)
    assert e.value.status == tg.TG_ERR_INVALID
    tg.tg_plan_free(plan)
    tg.tg_assemble_begin(b.pool.pool, other, tg.TG_ASSEMBLE_VERIFY, **args)
    tg.tg_assemble_feed(b.pool.pool, other, seg.ptr, seg.nbytes, [(0, offs[1])])
    tg.tg_assemble_wait(b.pool.pool, other, 1)
    tg.tg_plan_free(other)
    oplan = b.store.plan(3, rows[1:2], host)
    b.store.assemble(oplan, host)
    b.check_image()
    # a verifying load whose segment holds the wrong bytes is refused and leaves the pool alone
    b.release(3, evict=True)
    plan = begin()
    seg.numpy()[offs[2] + 5] ^= 1
    tg.tg_assemble_feed(b.pool.pool, plan, seg.ptr, seg.nbytes, [(k, offs[k]) for k in (1, 2, 3)])
    with pytest.raises(tg.TgError) as e:
        tg.tg_assemble_wait(b.pool.pool, plan, 4)
    assert e.value.status == tg.TG_ERR_CORRUPT
    tg.tg_plan_free(plan)
    b.check_image()
    seg.free()
    b.close()


def test_destroying_a_pool_or_freeing_a_plan_ends_a_load_in_flight():
    say("pool destroyed / plan freed while a load is in flight")
    rnd = random.Random(88)
    tensors = [rbytes(rnd, n) for n in (64 << 20, 4096, 1 << 20)]
    host, offs = pack(tensors)
    seg = HostArena(host.size)
    seg.numpy()[:] = host
    rows = [(t.size, oracle.fingerprint(t), o) for t, o in zip(tensors, offs)]
    for how in ("destroy", "free"):
        p = ReusePool(256 << 20, 256, DEV)
        plan = tg.tg_plan(p.pool, tg.ModelDesc(1, 0, 0, rows))
        tg.tg_assemble_begin(p.pool, plan, tg.TG_ASSEMBLE_VERIFY, **stream_args(p))
        tg.tg_assemble_feed(p.pool, plan, seg.ptr, seg.nbytes, [(0, offs[0]), (1, offs[1])])
        if how == "destroy":
            p.close()                              # waits for the streams, gives the load up, frees the tables
            tg.tg_plan_free(plan)
        else:
            tg.tg_plan_free(plan)
            st = p.stats()
            assert st["n_entries"] == 0 and st["free_bytes"] == st["capacity"]
            # the pool goes on working
            plan = tg.tg_plan(p.pool, tg.ModelDesc(1, seg.ptr, seg.nbytes, rows))
            ptrs = tg.tg_assemble(p.pool, plan, 3, tg.TG_ASSEMBLE_VERIFY, p.stream_gather, p.stream_h2d)
            tg.tg_plan_free(plan)
            for ptr, t in zip(ptrs, tensors):
                assert p.view(ptr, t.size).cpu().numpy().tobytes() == t.tobytes()
            p.close()
    torch.cuda.synchronize()
    seg.free()


def test_async_assemble_returns_before_the_transfer_and_gives_the_same_result():
    say("tg_assemble_async + tg_assemble_wait")
    import time
    rnd = random.Random(5)
    b = Pair(1 << 30)
    a = [rbytes(rnd, n) for n in (1 << 20, 4096, 96 << 20)]
    b.load_whole(1, a)
    b.release(1)
    m2 = [a[2], rbytes(rnd, 300 << 20), rbytes(rnd, 1000), a[1], rbytes(rnd, 5 << 20)]
    host, offs = pack(m2)
    arena = HostArena(host.size)
    arena.numpy()[:] = host
    rows = b.rows(m2, offs)
    desc = tg.ModelDesc(2, arena.ptr, arena.nbytes, rows)
    oplan = b.store.plan(2, rows, host)
    plan = tg.tg_plan(b.pool.pool, desc)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    tg.tg_assemble_async(b.pool.pool, plan, tg.TG_ASSEMBLE_VERIFY, **stream_args(b.pool))
    t_enqueue = time.perf_counter() - t0
    ptrs = tg.tg_assemble_wait(b.pool.pool, plan, len(rows))
    t_all = time.perf_counter() - t0
    tg.tg_plan_free(plan)
    dsts = b.store.assemble(oplan, host)
    assert ptrs == [b.pool.base + d for d in dsts]
    b.check_image()
    # 305 MB over the host link take about 5 ms; enqueueing them does not wait for that
    say("async: enqueue %.3f ms, whole load %.3f ms" % (t_enqueue * 1e3, t_all * 1e3))
    assert t_enqueue < 0.5 * t_all
    arena.free()
    b.close()


def test_two_pools_load_at_the_same_time_from_two_threads():
    say("two pools, two threads, loads at the same time")
    from paper_2512_01357_amd.loader import concurrent_stream_pair
    concurrent_stream_pair(torch.device(DEV))        # the one-off stream measurement, before the threads start
    errors = []
    ready = threading.Barrier(2)

    def worker(seed):
        try:
            rnd = random.Random(seed)
            b = Pair(768 << 20)
            b.pool.set_profiling(seed % 2 == 0)          # the two pools do not share settings
            b.pool.set_tuning(gather_unroll=4 if seed % 2 else 8)
            base = [rbytes(rnd, n) for n in (1 << 20, 24 << 20, 4096, 48 << 20, 100, 65536)]
            ready.wait(timeout=60)
            b.load_whole(1, base)
            b.release(1)
            for step in range(6):
                model = [base[i] if (i + step) % 2 else rbytes(rnd, base[i].size + 16 * step) for i in range(len(base))]
                b.load_whole(10 + step, model)
                b.release(10 + step, evict=(step % 2 == 0))
            b.check_image()
            assert (b.pool.last_timing["gather_ms"] > 0) == (seed % 2 == 0)
            b.close()
        except BaseException as exc:                     # noqa: BLE001
            errors.append((seed, repr(exc)))
            try:
                ready.abort()
            except Exception:
                pass

    threads = [threading.Thread(target=worker, args=(s,)) for s in (20, 21)]
    for th in threads:
        th.start()
    for th in threads:
        th.join(timeout=200)
    assert not any(th.is_alive() for th in threads), "a thread did not finish"
    assert not errors, errors


def test_fingerprint_and_compare_read_pinned_host_memory_in_place():
    say("tg_fingerprint / tg_compare on pinned host memory through its device mapping")
    rnd = random.Random(9)
    lengths = [0, 1, 15, 16, 17, 4095, 32768, 32769, 100003, (1 << 20) + 24, 5 * (1 << 20) + 13]
    datas = [rbytes(rnd, n) for n in lengths]
    host, offs = pack(datas)
    arena = HostArena(host.size)
    arena.numpy()[:] = host
    dev = tg.tg_host_device_ptr(arena.ptr)
    spans = [(dev + o, n) for o, n in zip(offs, lengths)]
    want = [oracle.fingerprint(d) for d in datas]
    assert tg.tg_fingerprint(spans) == want
    assert tg.tg_fingerprint_noalloc(spans) == want
    # compare: the pinned image against a device copy, with single bytes flipped on the device
    on_dev = torch.from_numpy(host).to(DEV)
    flipped = [2, 5, 8, 10]
    for i in flipped:
        on_dev[offs[i] + lengths[i] - 1] ^= 0x40
    torch.cuda.synchronize()
    pairs = [(on_dev.data_ptr() + o, dev + o, n) for o, n in zip(offs, lengths)]
    want_diff = [0 if oracle.bytes_equal(on_dev[o:o + n].cpu().numpy(), d) else 1 for o, n, d in zip(offs, lengths, datas)]
    assert want_diff == [1 if i in flipped else 0 for i in range(len(lengths))]
    assert tg.tg_compare(pairs) == want_diff
    with pytest.raises(tg.TgError) as e:
        tg.tg_host_device_ptr(0)
    assert e.value.status == tg.TG_ERR_INVALID
    arena.free()


def test_copy_grouping_threshold_changes_the_copies_not_the_result():
    say("h2d_group_bytes: adjacent missing tensors merged until a copy exceeds the threshold")
    rnd = random.Random(12)
    mib = 1 << 20
    tensors = [rbytes(rnd, mib) for _ in range(8)]       # equal slots: best fit lines them up in index order
    copies = {}
    for limit in (0, 2 * mib, 8 * mib, 1):
        b = Pair(64 * mib)
        b.pool.set_tuning(h2d_group_bytes=limit)
        b.load_whole(1, tensors)
        copies[limit] = b.pool.last_timing["h2d_copies"]
        b.close()
    # no limit: one copy; 2 MiB: a copy stops growing once it is past 2 MiB (3 + 3 + 2 tensors);
    # the paper's 8 MB: everything in one copy here; 1 byte: nothing is merged
    assert copies == {0: 1, 2 * mib: 3, 8 * mib: 1, 1: 8}


def _some_size(rnd, tile):
    r = rnd.random()
    if r < 0.25:
        return rnd.randrange(1, 300)
    if r < 0.45:
        return rnd.choice([tile, 2 * tile, 3 * tile]) + rnd.randrange(-40, 41)
    if r < 0.65:
        return rnd.randrange(1, 1 << 16)
    if r < 0.9:
        return rnd.randrange(1 << 16, 4 << 20)
    return rnd.randrange(4 << 20, 24 << 20)


@pytest.mark.parametrize("seed", range(24))
def test_random_models_under_random_launch_shapes(seed):
    rnd = random.Random(90000 + seed)
    unroll = rnd.choice([2, 4, 8, 16])
    tune = dict(gather_unroll=unroll, fingerprint_unroll=rnd.choice([2, 4, 8, 16]), gather_wgs_per_cu=rnd.choice([1, 2]),
                fingerprint_wgs_per_cu=rnd.choice([1, 2, 4, 8]), fuse_verify=rnd.randrange(4),
                h2d_kernel_max_bytes=rnd.choice([0, 4096, 65536, 1 << 20]),
                h2d_group_bytes=rnd.choice([0, 1, 1 << 20, 8 << 20]))
    align = rnd.choice([16, 256, 4096])
    say("random model %d: align %d, %s" % (seed, align, tune))
    b = Pair(512 << 20, align)
    b.pool.set_tuning(**tune)
    tile = 1024 * 16 * unroll
    n = rnd.randrange(1, 40)
    a = [rbytes(rnd, _some_size(rnd, tile)) for _ in range(n)]
    b.load_whole(1, a)
    b.release(1)
    # a second model that shares about half of the tensors, then a third made of a subset
    m2 = [a[i] if rnd.random() < 0.5 else rbytes(rnd, _some_size(rnd, tile)) for i in range(n)]
    b.load_whole(2, m2, verify=rnd.random() < 0.8)
    b.release(2, evict=rnd.random() < 0.5)
    b.load_whole(3, [m2[i] for i in rnd.sample(range(n), max(1, n // 2))])
    b.close()


@pytest.mark.parametrize("fuse", [1, 0])
@pytest.mark.parametrize("unroll", [2, 4, 8, 16])
def test_a_verifying_load_fingerprints_inside_the_copy_launch_or_after_it(fuse, unroll):
    say("verify: fuse_verify=%d, gather_unroll=%d" % (fuse, unroll))
    rnd = random.Random(40 + unroll)
    b = Pair(256 << 20)
    b.pool.set_tuning(fuse_verify=fuse, gather_unroll=unroll)
    tile = 1024 * 16 * unroll
    sizes = [1, 7, 16, 24, 255, 4096, 5000, 65536, 65537, tile - 16, tile - 8, tile, tile + 1, tile + 24, 2 * tile,
             3 * tile + 4096 + 5, (1 << 20) + 24, 3 * (1 << 20) + 1, 9 << 20]
    a = [rbytes(rnd, n) for n in sizes]
    b.load_whole(1, a)
    b.release(1)
    m2 = [a[i] if i % 3 else rbytes(rnd, sizes[i]) for i in range(len(sizes))]
    oplan = b.load_whole(2, m2)
    t = b.pool.last_timing
    through_copy_launch = sum(op.nbytes for op in oplan.ops if op.kind == 0 or op.nbytes <= 65536)
    assert t["fused_verify_bytes"] == (through_copy_launch if fuse else 0)
    assert t["verify_bytes"] + t["fused_verify_bytes"] == sum(sizes)
    b.release(2, evict=True)
    # a resident tensor is damaged in the pool; a verifying load that reuses it is refused either way
    victim = next(e for e in b.store.entries if e.nbytes == sizes[-2])
    b.pool.slab[victim.off + 12345] ^= 0x10
    torch.cuda.synchronize()
    host, offs = pack(m2)
    arena = HostArena(host.size)
    arena.numpy()[:] = host
    reg = RegisteredModel(3, arena, offs, sizes, [r[1] for r in b.rows(m2, offs)])
    with pytest.raises(tg.TgError) as e:
        b.pool.load(reg, verify=True)
    assert e.value.status == tg.TG_ERR_CORRUPT
    b.pool.slab[victim.off + 12345] ^= 0x10
    torch.cuda.synchronize()
    b.check_image()                                   # nothing was committed
    b.load_whole(3, m2)
    arena.free()
    b.close()

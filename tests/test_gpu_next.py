"""GPU parity for eviction, merge moves and alias mode: the pool's bytes after
every step against the oracle's image, bit for bit, through the C ABI."""
import random

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

import oracle  # noqa: E402
from gpu_harness import DEV, same_pool_state, say  # noqa: E402
from oracle import NoSpace, ReuseStoreOracle  # noqa: E402
from paper_2512_01357_amd import tangram as tg  # noqa: E402
from paper_2512_01357_amd.loader import HostArena, ReusePool  # noqa: E402

U = 256
MIB = 1 << 20


def rbytes(rnd, n):
    return np.random.default_rng(rnd.getrandbits(32)).integers(0, 256, n, dtype=np.uint8)


def pack(tensors, align=256):
    offs, at = [], 0
    for t in tensors:
        offs.append(at)
        at += (len(t) + align - 1) // align * align
    host = np.zeros(max(at, align), dtype=np.uint8)
    for t, o in zip(tensors, offs):
        host[o:o + len(t)] = t
    return host, offs


class Both:
    def __init__(self, capacity, align=256):
        self.align = align
        self.pool = ReusePool(capacity, align, DEV)
        self.store = ReuseStoreOracle(capacity, align)
        self.keep = []

    def load(self, mid, tensors, in_steps=0, overlap=False, **fl):
        """Loads on both sides.  in_steps > 0: the library plans without a host image and is fed
        the missing tensors in that many pieces (tg_assemble_begin / _feed / _wait)."""
        host, offs = pack(tensors, max(self.align, 16))
        arena = HostArena(host.size)
        arena.numpy()[:] = host
        self.keep.append(arena)
        sizes = [len(t) for t in tensors]
        want = [oracle.fingerprint(t) for t in tensors]
        reg = self.pool.register(mid, arena, offs, sizes)
        assert reg.fps == want
        rows = list(zip(sizes, want, offs))
        try:
            oplan = self.store.plan(mid, rows, host, **fl)
        except NoSpace:
            with pytest.raises(tg.TgError) as e:
                self.pool.load(reg, **fl)
            assert e.value.status == tg.TG_ERR_NOSPACE
            return None, None
        if in_steps:
            from paper_2512_01357_amd.loader import RegisteredModel
            bare = RegisteredModel(mid, None, offs, sizes, want)

            def pieces(missing):
                n = max(1, -(-len(missing) // in_steps))
                for i in range(0, len(missing), n):
                    yield arena.ptr, arena.nbytes, [(k, offs[k]) for k in missing[i:i + n]]
            ptrs, info = self.pool.load_streamed(bare, pieces, verify=True, overlap=overlap, **fl)
        else:
            ptrs, info = self.pool.load(reg, verify=True, **fl)
        assert info["ops"] == [(op.kind, op.dst_off, op.src_off, op.nbytes) for op in oplan.ops]
        assert info["moves"] == [(old, new, e.nbytes) for e, old, new in oplan.moves]
        assert info["evictions"] == [e.off for e in oplan.evictions]
        dsts = self.store.assemble(oplan, host)
        assert ptrs == [self.pool.base + d for d in dsts]
        self.check()
        return oplan, dsts

    def check(self):
        """Every resident tensor holds exactly the oracle's bytes."""
        for e in self.store.entries:
            got = self.pool.slab[e.off:e.off + e.nbytes].cpu().numpy()
            assert got.tobytes() == self.store.image[e.off][:e.nbytes].tobytes(), (e.off, e.nbytes)
        same_pool_state(self.pool.pool, self.store)

    def release(self, mid, evict=False):
        self.pool.release(mid, evict)
        self.store.release(mid, evict)

    def cost(self, mid, p, b, a):
        self.pool.set_model_cost(mid, p, b, a)
        self.store.set_model_cost(mid, p, b, a)

    def close(self):
        self.pool.close()
        for a in self.keep:
            a.free()


def carve(b, rnd, layout, unit):
    for i, (units, keep) in enumerate(layout):
        b.load(100 + i, [rbytes(rnd, units * unit)])
        b.release(100 + i)
    for i, (units, keep) in enumerate(layout):
        if not keep:
            b.release(100 + i, evict=True)


def test_hand_derived_merge_plan_moves_real_bytes():
    say("merge example, small shifts (staged moves)")
    rnd = random.Random(1)
    b = Both(30 * U)
    carve(b, rnd, [(4, False), (2, True), (4, False), (6, True), (4, False), (1, True), (4, False),
                   (1, True), (4, False)], U)
    plan, dsts = b.load(9, [rbytes(rnd, 6 * U), rbytes(rnd, 5 * U - 7)], merge=True)
    assert [(o // U, n // U) for _e, o, n in plan.moves] == [(4, 0), (20, 16), (25, 17)]
    b.close()


def test_failed_verification_after_moves_and_evictions_leaves_a_consistent_pool():
    say("verification fails on a plan that moves and evicts")
    rnd = random.Random(77)
    b = Both(30 * U)
    carve(b, rnd, [(4, False), (2, True), (4, False), (6, True), (4, False), (1, True), (4, False),
                   (1, True), (4, False)], U)

    def failing_load(mid, tensors, **fl):
        """A model whose last descriptor carries a wrong fingerprint: the library
        gives the plan up; the oracle carries it out and drops the model at once."""
        host, offs = pack(tensors)
        arena = HostArena(host.size)
        arena.numpy()[:] = host
        b.keep.append(arena)
        sizes = [len(t) for t in tensors]
        fps = [oracle.fingerprint(t) for t in tensors]
        fps[-1] ^= 1 << 40
        reg = b.pool.register(mid, arena, offs, sizes, fps=fps)
        oplan = b.store.plan(mid, list(zip(sizes, fps, offs)), host, **fl)
        gen = b.pool.stats()["generation"]
        with pytest.raises(tg.TgError) as e:
            b.pool.load(reg, verify=True, **fl)
        assert e.value.status == tg.TG_ERR_CORRUPT
        assert b.pool.stats()["generation"] == gen + 1
        b.store.assemble(oplan, host)
        b.store.release(mid, True)
        b.check()
        return oplan

    oplan = failing_load(9, [rbytes(rnd, 6 * U), rbytes(rnd, 5 * U - 7)], merge=True)
    assert [(o // U, n // U) for _e, o, n in oplan.moves] == [(4, 0), (20, 16), (25, 17)]
    # fill the pool with retained models, then a failing load that has to evict
    for i in range(3):
        b.load(200 + i, [rbytes(rnd, 5 * U), rbytes(rnd, U)])
        b.release(200 + i)
    oplan = failing_load(10, [rbytes(rnd, 3 * U), rbytes(rnd, 4 * U)], evict=True, merge=True)
    assert oplan.evictions
    # the pool goes on working: a good load, a reload of a survivor in place
    b.load(11, [rbytes(rnd, 2 * U), rbytes(rnd, 700)], evict=True, merge=True)
    b.release(11, evict=True)
    b.close()


@pytest.mark.parametrize("fuse", [3, 1])
def test_large_moves_straight_and_staged(fuse):
    say("merge with large shifts (straight copies) and small shifts over long tensors (staged); "
        "moved tensors fingerprinted %s" % ("by the launches that land them" if fuse & 2 else "by a launch of their own"))
    rnd = random.Random(2)
    # F64 A200 F64 B40 F100 (MiB): a 210 MiB tensor fits nowhere; everything is compacted.
    # A shifts by 64 MiB (straight, in pieces of at most 64 MiB), B by 128 MiB.
    b = Both(468 * MIB)
    b.pool.set_profiling(True)
    b.pool.set_tuning(fuse_verify=fuse)
    carve(b, rnd, [(64, False), (200, True), (64, False), (40, True), (100, False)], MIB)
    plan, _ = b.load(9, [rbytes(rnd, 210 * MIB + 40)], merge=True)
    assert [(o // MIB, n // MIB) for _e, o, n in plan.moves] == [(64, 0), (328, 200)]
    t = b.pool.last_timing
    assert t["move_bytes"] == 240 * MIB and t["move_traffic_bytes"] == 2 * 240 * MIB
    # A goes in pieces of 64 + 64 + 64 + 8 MiB (a launch may not write at or above the first byte
    # it reads, 64 MiB ahead); B's 40 MiB land below that mark too and ride in the last launch
    assert t["move_launches"] == 4
    # the moved tensors are fingerprinted as well as the new one: piece by piece into one word
    # each where they land, or in a launch of their own afterwards
    assert t["fused_verify_bytes"] == (240 * MIB if fuse & 2 else 0)
    assert t["verify_bytes"] == 210 * MIB + 40 + (0 if fuse & 2 else 240 * MIB)
    b.close()
    # F1 A300 F100 (MiB) + a 101 MiB tensor: A shifts by 1 MiB, staged through 128 MiB at a time
    b = Both(401 * MIB)
    b.pool.set_tuning(fuse_verify=fuse)
    carve(b, rnd, [(1, False), (300, True), (100, False)], MIB)
    plan, _ = b.load(9, [rbytes(rnd, 101 * MIB - 3)], merge=True)
    assert [(o // MIB, n // MIB) for _e, o, n in plan.moves] == [(1, 0)]
    t = b.pool.last_timing
    assert t["move_launches"] == 6 and t["move_traffic_bytes"] == 4 * 300 * MIB
    assert t["fused_verify_bytes"] == (300 * MIB if fuse & 2 else 0)
    b.close()


@pytest.mark.parametrize("fuse", [3, 2, 1, 0])
def test_a_moved_tensor_that_no_longer_matches_its_row_is_dropped(fuse):
    say("a resident tensor is damaged, then moved by a merging load that verifies (fuse_verify=%d)" % fuse)
    rnd = random.Random(78)
    b = Both(30 * U)
    b.pool.set_tuning(fuse_verify=fuse)
    carve(b, rnd, [(4, False), (2, True), (4, False), (6, True), (4, False), (1, True), (4, False),
                   (1, True), (4, False)], U)
    b.pool.slab[20 * U + 5] ^= 0x10                      # model 105's tensor (moves 20 -> 16 units)
    torch.cuda.synchronize()
    tensors = [rbytes(rnd, 6 * U), rbytes(rnd, 5 * U - 7)]
    host, offs = pack(tensors)
    arena = HostArena(host.size)
    arena.numpy()[:] = host
    b.keep.append(arena)
    sizes = [len(t) for t in tensors]
    reg = b.pool.register(9, arena, offs, sizes)
    oplan = b.store.plan(9, list(zip(sizes, reg.fps, offs)), host, merge=True)
    assert [(o // U, n // U) for _e, o, n in oplan.moves] == [(4, 0), (20, 16), (25, 17)]
    with pytest.raises(tg.TgError) as e:
        b.pool.load(reg, verify=True, merge=True)
    assert e.value.status == tg.TG_ERR_CORRUPT
    # the moves happened, the model did not arrive, the damaged tensor is no longer offered for reuse
    b.store.assemble(oplan, host)
    b.store.release(9, True)
    b.store.release(105, True)
    b.check()
    # without verification nobody would have noticed: the same load now goes through
    b.load(10, tensors, merge=True)
    b.close()


@pytest.mark.parametrize("streams", ["one side stream", "null stream", "null + side", "side + null",
                                     "three side streams", "second = first", "second = gather", "null + two side"])
def test_moves_gather_and_transfer_on_any_pair_of_streams(streams):
    say("merge + gather + transfer on %s, with a transfer large enough for the pipelined verification" % streams)
    rnd = random.Random(5)
    b = Both(600 * MIB)
    side = b.pool.stream_gather
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    b.pool.stream_gather, b.pool.stream_h2d, b.pool.stream_h2d_second = {
        "one side stream": (side, side, None), "null stream": (None, None, None),
        "null + side": (None, side, None), "side + null": (side, None, None),
        "three side streams": (side, s1, s2), "second = first": (side, s1, s1),
        "second = gather": (side, s1, side), "null + two side": (None, s1, s2)}[streams]
    # F8 A40 F8 B24 F(rest): residents A and B are also tensors of the incoming model (gathered);
    # the 300 MiB miss (pipelined verification: batches of >= 64 MiB) leaves room only if A, B merge
    carve(b, rnd, [(8, False), (40, True), (8, False), (24, True), (8, False)], MIB)
    a_bytes = b.store.image[8 * MIB][:40 * MIB].copy()
    big = [rbytes(rnd, 100 * MIB - 16 * i) for i in range(3)]
    filler = rbytes(rnd, 190 * MIB)
    b.load(50, [filler])
    b.release(50)
    plan, _ = b.load(9, big + [a_bytes, rbytes(rnd, 4096), rbytes(rnd, 70000)], merge=True)
    assert plan.moves and plan.ops[3].kind == 0
    b.release(9, evict=True)
    b.close()


def test_eviction_then_load_real_bytes():
    say("stage 1 eviction")
    rnd = random.Random(3)
    b = Both(16 * U)
    for mid, sizes in ((1, [1024, 512]), (2, [768, 256]), (3, [512])):
        b.load(mid, [rbytes(rnd, n) for n in sizes])
        b.release(mid)
    b.cost(1, 0.5, 2.0, 1.0)
    b.cost(2, 1.0, 1.0, 0.1)
    plan, dsts = b.load(9, [rbytes(rnd, 1024), rbytes(rnd, 1024)], evict=True)
    assert [e.nbytes for e in plan.evictions] == [256, 768]
    b.close()


def test_alias_mode_real_bytes():
    say("alias mode")
    rnd = random.Random(4)
    b = Both(4 * MIB)
    a = [rbytes(rnd, 300000), rbytes(rnd, 512), rbytes(rnd, 70001)]
    _, a_dst = b.load(1, a)
    b.release(1)
    m2 = [a[0], rbytes(rnd, 90000), a[2]]
    plan, dsts = b.load(2, m2, alias=True)
    assert [op.kind for op in plan.ops] == [0, 1, 0]
    assert dsts[0] == a_dst[0] and dsts[2] == a_dst[2]
    assert tg.tg_pool_stats(b.pool.pool)["n_entries"] == 4
    plan, dsts = b.load(1, a, alias=True)           # comes back while 2 runs: nothing to transfer
    assert plan.transfer_bytes == 0 and dsts == a_dst
    b.release(2, evict=True)
    b.check()
    b.release(1, evict=True)
    assert b.pool.stats()["free_bytes"] == 4 * MIB
    b.close()


@pytest.mark.parametrize("seed", range(12))
def test_random_histories_with_every_flag_real_bytes(seed):
    fuse = (1, 3, 0, 2)[seed % 4]
    say("random history %d (fuse_verify=%d)" % (seed, fuse))
    rnd = random.Random(700 + seed)
    b = Both(24 * MIB)
    b.pool.set_tuning(fuse_verify=fuse)
    library = [rbytes(rnd, rnd.choice([40, 4096, 70000, 300000, 1 << 20, (1 << 20) + 24, 3 << 20, 5000000]))
               for _ in range(20)]
    running, retained, next_id = {}, [], 1
    for step in range(60):
        r = rnd.random()
        if r < 0.55 or not (running or retained):
            tensors = [library[rnd.randrange(20)] for _ in range(rnd.randrange(1, 6))]
            fl = dict(evict=rnd.random() < 0.7, merge=rnd.random() < 0.7, alias=rnd.random() < 0.5,
                      pack_text=rnd.random() < 0.5)
            mid = next_id
            if retained and rnd.random() < 0.25:
                mid = rnd.choice(retained)
            plan, dsts = b.load(mid, tensors, in_steps=rnd.choice([0, 0, 1, 3]), overlap=step % 2 == 1, **fl)
            if plan is None:
                continue
            running[mid] = (tensors, dsts)
            if mid in retained:
                retained.remove(mid)
            if mid == next_id:
                next_id += 1
        elif running and (not retained or rnd.random() < 0.6):
            mid = rnd.choice(sorted(running))
            evict = rnd.random() < 0.4
            b.release(mid, evict)
            del running[mid]
            if not evict:
                retained.append(mid)
        else:
            mid = rnd.choice(retained)
            if mid in b.store.models:
                b.release(mid, True)
            retained.remove(mid)
        retained = [m for m in retained if m in b.store.models]
        # every tensor of every running model is where the caller was told, byte for byte
        for mid, (tensors, dsts) in running.items():
            for t, d in zip(tensors, dsts):
                got = b.pool.slab[d:d + len(t)].cpu().numpy()
                assert got.tobytes() == t.tobytes(), (mid, d)
    b.check()
    b.close()


@pytest.mark.parametrize("align", [16, 4096])
def test_other_pool_alignments(align):
    say("pool alignment %d" % align)
    rnd = random.Random(align)
    b = Both(8 * MIB, align)
    a = [rbytes(rnd, n) for n in (1, 15, 16, 17, 4095, 4096, 4097, 70000, 300001, 1 << 20)]
    b.load(1, a)
    b.release(1)
    m2 = [a[i] if i % 2 else rbytes(rnd, len(a[i])) for i in range(len(a))]
    plan, dsts = b.load(2, m2)
    assert all(d % align == 0 for d in dsts)
    b.release(1, evict=True)
    b.load(3, [rbytes(rnd, 2 * MIB), a[9]], evict=True, merge=True, alias=True, pack_text=True)
    b.close()


def test_thousands_of_tiny_tensors_in_one_launch():
    say("5000 tiny tensors")
    rnd = random.Random(11)
    b = Both(8 * MIB)
    sizes = [rnd.choice([1, 8, 16, 24, 100, 256, 700]) for _ in range(5000)]
    a = [rbytes(rnd, n) for n in sizes]
    b.load(1, a)
    b.release(1)
    m2 = [a[i] if i % 3 else rbytes(rnd, sizes[i]) for i in range(5000)]
    plan, _ = b.load(2, m2)
    assert sum(1 for op in plan.ops if op.kind == 0) >= 3300
    b.close()

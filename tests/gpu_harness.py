"""Drives a synthetic workload through the HIP library and the CPU oracle side
by side (GPU tests only).  Every oracle input is host bytes; nothing the
library computes is fed to the oracle."""
import sys
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

import oracle
from oracle import ReuseStoreOracle
from paper_2512_01357_amd import synth
from paper_2512_01357_amd.runner import WorkloadRunner

DEV = "cuda:0"


def say(msg):
    print("[gpu-test] " + msg, flush=True)
    sys.stdout.flush()


def same_pool_state(pool, store):
    """The library's counters, Region List and Tensor Mapping against the oracle's, row by row."""
    from paper_2512_01357_amd import tangram as tg
    a, b = tg.tg_pool_stats(pool), store.stats()
    for key, v in b.items():
        assert a[key] == v, key
    assert tg.tg_pool_regions(pool) == [(off, length, bool(free)) for off, length, free in store.regions]
    assert tg.tg_pool_entries(pool) == sorted((e.off, e.nbytes, e.fp, len(e.owners), e.active_refs)
                                              for e in store.entries)


def oracle_fps(host_np, offs, sizes, threads=16):
    """Oracle fingerprints of many tensors; the C loop releases the GIL, so a
    thread per tensor is just a way to use the host's cores."""
    uniq = sorted(set(zip(offs, sizes)))
    with ThreadPoolExecutor(max_workers=threads) as ex:
        vals = list(ex.map(lambda os_: oracle.fingerprint(host_np[os_[0]:os_[0] + os_[1]]), uniq))
    table = dict(zip(uniq, vals))
    return [table[(o, n)] for o, n in zip(offs, sizes)]


def run_workload_both(w, image_limit=1 << 30, sample_every=37, after_load=None, overlap=False):
    """Replays `w` on the library and on the oracle.

    Fingerprints, plan rows, returned addresses and pool statistics are
    compared for every tensor.  Assembled bytes: every slot is compared with
    its source (the model's pinned image, or for a model that passes through the
    Model Cache in segments the tensor regenerated from its seed; on the
    device, by torch.equal, an independent checker); while a model is at most
    `image_limit` bytes the oracle also keeps its own image of the pool and
    every slot is compared with it, beyond that the oracle assembles every
    `sample_every`-th tensor (and the smallest and largest) on its own, from
    the host bytes, and those are compared byte for byte.
    `overlap`: models that pass through the Model Cache in pieces are loaded with
    the cache cut in two halves, one refilled while the other is copied.
    """
    r = WorkloadRunner(w, DEV, gen_device=DEV, log=say)
    store = ReuseStoreOracle(w.pool_bytes, w.align)
    small = all(m.nbytes <= image_limit for m in w.models.values())
    plans = {}
    tracked = []          # (oracle entry, tensor spec) of every slot ever filled

    def sample_of(n, sizes):
        by_size = sorted(range(n), key=lambda k: sizes[k])
        return set(range(0, n, sample_every)) | {by_size[0], by_size[-1]}

    # Models that pass through the Model Cache in segments: the oracle's inputs are the host bytes
    # of each segment, seen once when it is filled -- fingerprints of every tensor, and a copy of
    # the tensors the oracle will assemble on its own.
    seg_fp = {}           # content key -> oracle fingerprint of the host bytes
    seg_bytes = {}        # content key -> host bytes (sampled tensors only)
    wanted = set()
    for name, spec in w.models.items():
        if r.is_streamed(name):
            for k in sample_of(len(spec.tensors), [t.nbytes for t in spec.tensors]):
                wanted.add(synth.content_key(spec.tensors[k]))

    def on_segment(name, rows, arena):
        spec = w.models[name]
        host_np = arena.numpy()
        todo = [(k, off) for k, off in rows if synth.content_key(spec.tensors[k]) not in seg_fp]
        with ThreadPoolExecutor(max_workers=16) as ex:
            vals = list(ex.map(lambda ko: oracle.fingerprint(host_np[ko[1]:ko[1] + spec.tensors[ko[0]].nbytes]), todo))
        for (k, off), f in zip(todo, vals):
            key = synth.content_key(spec.tensors[k])
            seg_fp[key] = f
            if key in wanted and key not in seg_bytes:
                seg_bytes[key] = host_np[off:off + spec.tensors[k].nbytes].copy()
    r.on_segment = on_segment

    def check_residents():
        """Every tensor still resident (moved or not) holds the bytes it was
        loaded with: regenerated from its seed and compared on the device."""
        n = 0
        for e, spec in tracked:
            if not e.owners:
                continue                      # evicted
            want = synth.tensor_bytes(spec, DEV)
            assert torch.equal(r.pool.slab[e.off:e.off + e.nbytes], want), (spec.name, e.off)
            n += 1
        return n

    def load(name):
        reg = r.materialise(name)
        spec = w.models[name]
        streamed = reg.host is None
        if streamed:
            host_np = None
            want = [seg_fp[synth.content_key(t)] for t in spec.tensors]
        else:
            host_np = r.host_numpy(name)
            want = oracle_fps(host_np, reg.offs, reg.sizes)
        assert reg.fps == want, "fingerprints of %s" % name
        rows = list(zip(reg.sizes, want, reg.offs))
        flags = dict(w.load_flags) if name in w.loads else {}
        oplan = store.plan(spec.model_id, rows, host_np if small else None, **flags)
        ptrs, info = r.load(name, verify=True, overlap=overlap, **flags)
        assert info["moves"] == [(old, new, e.nbytes) for e, old, new in oplan.moves], name
        assert info["evictions"] == [e.off for e in oplan.evictions], name
        assert info["ops"] == [(op.kind, op.dst_off, op.src_off, op.nbytes) for op in oplan.ops], name
        assert info["reused_bytes"] == oplan.reused_bytes
        assert info["transfer_bytes"] == oplan.transfer_bytes
        n_before = len(store.entries) - len(oplan.evictions)
        dsts = store.assemble(oplan, host_np if small else None)
        assert ptrs == [r.pool.base + d for d in dsts]
        fresh = [k for k in range(len(rows)) if not (oplan.alias and oplan.hits[k] is not None)]
        for e, k in zip(store.entries[n_before:], fresh):
            tracked.append((e, spec.tensors[k]))
        if oplan.moves or oplan.evictions:
            say("%s: %d evicted, %d moved; %d residents re-checked"
                % (name, len(oplan.evictions), len(oplan.moves), check_residents()))
        host_t = None if streamed else r.models[name].host_tensor
        n = len(rows)
        sampled = sample_of(n, [row[0] for row in rows])
        for k, (op, (nbytes, _f, off)) in enumerate(zip(oplan.ops, rows)):
            slot = r.pool.slab[op.dst_off:op.dst_off + nbytes]
            if streamed:
                assert torch.equal(slot, synth.tensor_bytes(spec.tensors[k], DEV)), (name, k)
            else:
                assert torch.equal(slot, host_t[off:off + nbytes].to(DEV)), (name, k)
            if small:
                assert slot.cpu().numpy().tobytes() == store.image[op.dst_off].tobytes(), (name, k)
            elif k in sampled:
                src = seg_bytes[synth.content_key(spec.tensors[k])] if streamed else host_np[off:off + nbytes]
                mine = np.empty(nbytes, dtype=np.uint8)
                oracle.copy_bytes(mine, src)                             # the oracle's assemble
                assert oracle.bytes_equal(slot.cpu().numpy(), mine), (name, k)
        same_pool_state(r.pool.pool, store)
        if after_load is not None:
            after_load(name, oplan, r)
        r.drop_host(name)
        return oplan, info

    for act in w.setup:
        if act[0] == "load":
            load(act[1])
            say("setup %s checked" % act[1])
        else:
            r.release(act[1], act[2])
            store.release(w.models[act[1]].model_id, act[2])
    for name, (p, b, a) in w.costs.items():
        r.pool.set_model_cost(w.models[name].model_id, p, b, a)
        store.set_model_cost(w.models[name].model_id, p, b, a)
    before = store.stats()
    infos = {}
    for name in w.loads:
        plans[name], infos[name] = load(name)
        say("load %s checked" % name)
        r.release(name, True)
        store.release(w.models[name].model_id, True)
    after = store.stats()
    if not w.rebuild_each_step:
        assert after == before          # releasing the model undoes the load
    same_pool_state(r.pool.pool, store)
    r.close()
    torch.cuda.empty_cache()
    run_workload_both.last_infos = infos
    return plans, before

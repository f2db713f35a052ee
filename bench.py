#!/usr/bin/env python3
"""Benchmark of the Load path on one MI355X.

A step is one whole load of a model into a pool that already holds its
sibling(s): tg_plan (match + best-fit), tg_assemble (gather kernel for the
reused tensors overlapped with the host-to-device stream for the missing
ones, a fingerprint of every assembled slot, then commit) and tg_release with
eviction, which puts the pool back as it was.

The default run times the 7B Llama-shaped family (steps cycle through the
variants v1, v2, v3; --steps / --warmup apply to it) and then, as `legs` of
the same JSON line, the 70B Llama-3-shaped model at 90 %, 50 % and 0 % reuse:
one plan of 723 tensors each, the missing tensors fed through a pinned Model
Cache segment smaller than the model.

Prints one JSON line: effective load GB/s (model bytes / step time), with the
roofline of the dominant kernel, the other kernels' figures, the host-link
figure and the CPU oracle's rate on the same load.
"""
import argparse
import gc
import json
import os
import re
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0        # MI355X published HBM3E bandwidth
METRIC = "effective load GB/s (model bytes resident / load time); fingerprint HBM GB/s"
PROFILES = os.path.join(ROOT, "profiles")
TRAFFIC_FILES = ["bench_llama7b_pmc_traffic.txt", "bench_llama70b_reuse90_pmc_traffic.txt",
                 "bench_llama70b_reuse50_reuse00_pmc_traffic.txt"]
ALU_FILE = "alu_mix_probe.txt"


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


# ------------------------------------------------------------------ figures measured off line
def read_profile_records(fname, tag):
    """`<tag>: key=value ...` lines of a tracked rocprofv3 summary under profiles/."""
    out = []
    path = os.path.join(PROFILES, fname)
    if not os.path.exists(path):
        return out
    with open(path) as f:
        for line in f:
            line = line.strip()
            if line.startswith(tag + ":"):
                out.append(dict(kv.split("=", 1) for kv in line[len(tag) + 1:].split()))
    return out


def profiled_traffic(workload, kernel, shape):
    """HBM bytes per step of `kernel` as rocprofv3's FETCH_SIZE + WRITE_SIZE counters read them in
    an earlier run of this file (scaled by a copy kernel of known size), or None when no tracked
    summary covers this workload with this launch shape.  Returns (bytes, source file)."""
    for fname in TRAFFIC_FILES:
        for rec in read_profile_records(fname, "bench-traffic"):
            if rec.get("workload") == workload and rec.get("kernel") == kernel and rec.get("shape") == shape:
                return int(rec["hbm_bytes_per_step"]), "profiles/" + fname
    return None, None


def profiled_alu_rate():
    """Words per second the fingerprint's mix sustains without its loads (tracked probe run)."""
    for rec in read_profile_records(ALU_FILE, "bench-alu"):
        return float(rec["mix_words_per_s"]), "profiles/" + ALU_FILE
    return None, None


def kernel_shapes(tuning, verify):
    """Template arguments x workgroups per compute unit of the two kernels a load launches."""
    u = lambda v: 16 if v >= 16 else 8 if v >= 8 else 4 if v >= 4 else 2      # noqa: E731
    fused = "true" if (verify and tuning["fuse_verify"] & 1) else "false"
    return {"fingerprint": "fingerprint_kernel<256,%d>x%d" % (u(tuning["fingerprint_unroll"]), tuning["fingerprint_wgs_per_cu"]),
            "gather": "gather_kernel<1024,%d,%s>x%d" % (u(tuning["gather_unroll"]), fused, tuning["gather_wgs_per_cu"])}


# ------------------------------------------------------------------ pieces of a run
def measure_link_peak(torch, nbytes=2 << 30, reps=3):
    """GB/s of one large pinned-to-device hipMemcpyAsync (the host link's
    measured peak on this machine, same run): a one-tensor model loaded into an
    empty pool through the library, timed by its HIP events."""
    from paper_2512_01357_amd.loader import HostArena, RegisteredModel, ReusePool
    arena = HostArena(nbytes)
    arena.tensor.fill_(1)
    pool = ReusePool(nbytes, 256, "cuda:0")
    pool.set_profiling(True)
    reg = RegisteredModel(1, arena, [0], [nbytes], [0])
    best = 0.0
    for _ in range(reps + 1):
        _p, info = pool.load(reg, details=False)
        pool.release(1, True)
        best = max(best, nbytes / (info["timing"]["h2d_ms"] * 1e-3) / 1e9)
    pool.close()
    arena.free()
    torch.cuda.empty_cache()
    return best


def cpu_model_name():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(runner, w, name):
    """The oracle as it stands, on this machine's host cores, on the same load the
    GPU leg times: the pool holds the resident sibling, then fingerprint every
    tensor of `name`, plan (match against the sibling + best fit), assemble
    (byte copies out of the oracle's pool image for the reused tensors, out of
    host memory for the missing ones) and commit.  Once on one thread, once
    with the tensors dealt over all host threads."""
    import numpy as np
    import oracle
    from oracle import ReuseStoreOracle

    cores = len(os.sched_getaffinity(0))
    reg = runner.models[name]
    host = runner.host_numpy(name)

    def resident_store():
        """A store in the state the GPU pool is in before the load (untimed)."""
        store = ReuseStoreOracle(w.pool_bytes, w.align)
        for act in w.setup:
            if act[0] == "load":
                r0 = runner.models[act[1]]
                h0 = runner.host_numpy(act[1])
                plan = store.plan(r0.model_id, list(zip(r0.sizes, r0.fps, r0.offs)))
                store.assemble(plan)
                for op in plan.ops:          # the sibling's bytes, where the oracle keeps a pool image
                    store.image[op.dst_off] = h0[op.src_off:op.src_off + op.nbytes]
            else:
                store.release(w.models[act[1]].model_id, act[2])
        return store

    def in_threads(fn, n_items, n_threads):
        def work(tid):
            for i in range(tid, n_items, n_threads):
                fn(i)
        threads = [threading.Thread(target=work, args=(t,)) for t in range(n_threads)]
        for t in threads:
            t.start()
        for t in threads:
            t.join()

    def one_pass(n_threads):
        store = resident_store()
        n = len(reg.sizes)
        t_start = time.perf_counter()
        fps = [0] * n

        def fp(k):
            fps[k] = oracle.fingerprint(host[reg.offs[k]:reg.offs[k] + reg.sizes[k]])
        in_threads(fp, n, n_threads)
        plan = store.plan(987654, list(zip(reg.sizes, fps, reg.offs)))
        slots = [None] * n

        def fill(k):
            op = plan.ops[k]
            slot = np.empty(op.nbytes, dtype=np.uint8)
            src = store.image[op.src_off][:op.nbytes] if op.kind == oracle.REUSE else host[op.src_off:op.src_off + op.nbytes]
            oracle.copy_bytes(slot, src)
            slots[k] = slot
        in_threads(fill, n, n_threads)
        store.assemble(plan)
        elapsed = time.perf_counter() - t_start
        return elapsed, plan.reused_bytes

    t1, reused = one_pass(1)
    n_thr = min(cores, len(reg.sizes))
    tn, _ = one_pass(n_thr)
    total = sum(reg.sizes)
    return {
        "value": round(total / tn / 1e9, 4), "unit": "GB/s", "cores": n_thr, "kind": "oracle",
        "value_1core": round(total / t1 / 1e9, 4),
        "sample": "one whole load of %s (%d tensors, %.2f GB, %.1f %% found resident in the sibling): oracle fingerprint "
                  "of every tensor + plan + byte-copy assemble + commit; %d-thread leg %.1f s, 1-thread leg %.1f s"
                  % (name, len(reg.sizes), total / 1e9, 100.0 * reused / total, n_thr, tn, t1),
        "host_cores_available": cores, "cpu": cpu_model_name(),
    }


def pmc_calibration_kernel(torch):
    """One plain elementwise kernel of known traffic (reads 1 GiB, writes 1 GiB), so that a
    rocprofv3 --pmc run has something to scale its FETCH_SIZE / WRITE_SIZE read-outs by."""
    a = torch.full((1 << 28,), 1.0, dtype=torch.float32, device="cuda:0")
    b = torch.empty_like(a)
    torch.cuda.synchronize()
    torch.mul(a, 1.0, out=b)
    torch.cuda.synchronize()
    del a, b


def kernel_figures(recs, verify, tuning, workload_name, plain_load):
    """roofline objects of the fingerprint (verify launches of a step together) and the gather."""
    steps = len(recs)

    def total(key):
        return sum(rec["timing"][key] for rec in recs)

    def gbps(nbytes, ms):
        return nbytes / (ms * 1e-3) / 1e9 if ms > 0 else 0.0

    fp_bytes, fp_ms, fp_launches = total("verify_bytes"), total("verify_ms"), total("verify_launches")
    g_bytes, g_ms = 2 * total("gather_bytes"), total("gather_ms")
    g_launches = sum(1 for rec in recs if rec["timing"]["gather_ms"] > 0)
    fp_rate, g_rate = gbps(fp_bytes, fp_ms), gbps(g_bytes, g_ms)
    shapes = kernel_shapes(tuning, verify)
    kernels = {
        "fingerprint": {"bound": "hbm", "achieved": round(fp_rate, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                        "frac": round(fp_rate / HBM_PEAK_GBPS, 4),
                        "avg_launch_ms": round(fp_ms / fp_launches, 4) if fp_launches else 0.0,
                        "launches_per_step": round(fp_launches / steps, 2), "ms_per_step": round(fp_ms / steps, 4),
                        "algorithmic_bytes_per_launch": int(fp_bytes / fp_launches) if fp_launches else 0,
                        "algorithmic_bytes_per_step": int(fp_bytes / steps), "shape": shapes["fingerprint"]},
        "gather": {"bound": "hbm", "achieved": round(g_rate, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                   "frac": round(g_rate / HBM_PEAK_GBPS, 4),
                   "avg_launch_ms": round(g_ms / g_launches, 4) if g_launches else 0.0,
                   "launches_per_step": round(g_launches / steps, 2), "ms_per_step": round(g_ms / steps, 4),
                   "algorithmic_bytes_per_launch": int(g_bytes / g_launches) if g_launches else 0,
                   "algorithmic_bytes_per_step": int(g_bytes / steps), "shape": shapes["gather"]},
    }
    # a launch over a few megabytes is bound by its launch, not by HBM: no bandwidth claim is made for it
    for k in kernels:
        if 0 < kernels[k]["algorithmic_bytes_per_launch"] < (256 << 20):
            kernels[k]["launch_bound_GBps"] = kernels[k]["achieved"]
            kernels[k]["achieved"] = kernels[k]["frac"] = None
            kernels[k]["note"] = "launches of under 256 MiB: bound by launch latency, not a bandwidth figure"
    # HBM traffic per step from rocprofv3 counters: only a tracked summary of this workload in this
    # launch shape counts; anything else is reported as not measured
    for k in kernels:
        traffic, source = (None, None)
        if verify and plain_load:
            traffic, source = profiled_traffic(workload_name, k, kernels[k]["shape"])
        kernels[k]["traffic"] = traffic
        kernels[k]["traffic_is"] = "HBM bytes per step (FETCH_SIZE + WRITE_SIZE), from an earlier rocprofv3 run" if traffic else None
        kernels[k]["traffic_source"] = source
    # integer-ALU co-limit of the fingerprint: what the mix alone (no loads) sustains on this chip
    rate, source = profiled_alu_rate()
    if rate:
        # the gather launch of a verifying load does the same arithmetic on the bytes it copies
        kernels["fingerprint"]["alu_colimit"] = {"equivalent_GBps": round(rate * 8 / 1e9, 1),
                                                 "frac": round(fp_rate / (rate * 8 / 1e9), 4), "source": source}
    fused = sum(rec["timing"]["fused_verify_bytes"] for rec in recs)
    kernels["gather"]["fingerprinted_bytes_per_step"] = int(fused / steps)
    return kernels


def dominant_roofline(kernels):
    name = max(kernels, key=lambda k: kernels[k]["ms_per_step"] if kernels[k]["achieved"] is not None else -1.0)
    roofline = dict(kernels[name])
    roofline["kernel"] = name
    return roofline


def host_link_figures(recs, link_peak):
    ms = sum(rec["timing"]["h2d_ms"] for rec in recs)
    nbytes = sum(rec["timing"]["h2d_bytes"] for rec in recs)
    rate = nbytes / (ms * 1e-3) / 1e9 if ms > 0 else 0.0
    return {"achieved": round(rate, 2), "peak_measured": round(link_peak, 2), "unit": "GB/s",
            "frac": round(rate / link_peak, 4) if link_peak else None, "ms_per_step": round(ms / len(recs), 3),
            "bytes_per_step": int(nbytes / len(recs)), "copies_per_load": recs[0]["timing"]["h2d_copies"]}


def bound_ms(recs, link_peak):
    return round(max(2 * sum(rec["reused_bytes"] for rec in recs) / (HBM_PEAK_GBPS * 1e9),
                     sum(rec["transfer_bytes"] for rec in recs) / (link_peak * 1e9)) * 1e3 / len(recs), 3)


# ------------------------------------------------------------------ a workload whose models fit the Model Cache
def bench_resident(args, torch, w, link_peak, steps, warmup, with_extras, with_cpu):
    from paper_2512_01357_amd import tangram as tg
    from paper_2512_01357_amd.loader import SECOND_H2D_MEASUREMENT, RegisteredModel
    from paper_2512_01357_amd.runner import WorkloadRunner

    r = WorkloadRunner(w, "cuda:0", log=log)
    r.pool.set_profiling(True)
    if args.tune:
        r.pool.set_tuning(**{k: int(v) for k, v in (kv.split("=") for kv in args.tune.split(","))})
    r.run_setup()
    for name in w.loads:
        r.materialise(name)
    st0 = r.pool.stats()
    log("pool before loads: %s" % st0)
    log("host-to-device copies on %s (32 x 4 MiB beside a device copy: %s)"
        % ("two streams" if r.pool.stream_h2d_second is not None else "one stream", SECOND_H2D_MEASUREMENT.get("cuda:0")))

    if args.pmc_calibration:
        pmc_calibration_kernel(torch)

    verify = not args.no_verify
    names = w.loads
    tuning = tg.tg_pool_get_tuning(r.pool.pool)

    def step(i):
        """One whole load of one model (+ release).  Returns its record and, where only the load
        may be timed, its duration."""
        name = names[i % len(names)]
        if w.rebuild_each_step:
            # the load moves or evicts residents: only the load is timed, then the pool is rebuilt
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            _ptrs, info = r.load(name, verify=verify, details=False)
            torch.cuda.synchronize()
            timed = time.perf_counter() - t0
            r.reset_pool()
            info["model_bytes"] = r.models[name].nbytes
            return info, timed
        _ptrs, info = r.load(name, verify=verify, details=False)
        r.release(name, True)
        info["model_bytes"] = r.models[name].nbytes
        return info, None

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    recs = []
    timed_total = 0.0
    # no garbage-collector pass inside the timed region (as timeit does): a full pass over
    # everything torch has imported takes tens of ms, more than 100 loads of the smallest workload
    gc.collect()
    gc.disable()
    t_begin = time.perf_counter()
    for i in range(steps):
        info, timed = step(warmup + i)
        recs.append(info)
        if timed is not None:
            timed_total += timed
    torch.cuda.synchronize()
    elapsed = timed_total if w.rebuild_each_step else time.perf_counter() - t_begin
    gc.enable()
    st1 = r.pool.stats()
    if any(st1[k] != st0[k] for k in st0 if k != "generation"):
        raise RuntimeError("pool did not return to its starting state: %s vs %s" % (st1, st0))

    total_bytes = sum(rec["model_bytes"] for rec in recs)
    value = total_bytes / elapsed / 1e9
    kernels = kernel_figures(recs, verify, tuning, w.name, plain_load=not any(w.load_flags.values()))
    out = {
        "metric": METRIC,
        "value": round(value, 3), "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(elapsed / steps * 1e3, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u64", "data": "synthetic",
        "config": {"workload": w.name, "model_bytes": int(total_bytes / steps),
                   "tensors": len(w.models[names[0]].tensors), "pool_bytes": w.pool_bytes,
                   "reused_fraction": round(sum(rec["reused_bytes"] for rec in recs) / total_bytes, 4),
                   "reused_tensors": int(sum(rec["n_reused"] for rec in recs) / steps),
                   "designated_shared_tensors": sum(w.designated_shared.values()) // max(1, len(w.designated_shared)),
                   "verify_fingerprint": verify,
                   "plan_flags": sorted(k for k, v in w.load_flags.items() if v),
                   "h2d_streams": 2 if r.pool.stream_h2d_second is not None else 1,
                   "model_cache": "whole model pinned"},
        "fingerprint_GBps": kernels["fingerprint"]["achieved"] or kernels["fingerprint"].get("launch_bound_GBps"),
        "roofline": dominant_roofline(kernels),
        "kernels": kernels,
        "host_link": host_link_figures(recs, link_peak),
        "plan_host_ms": round(sum(rec["timing"]["plan_host_ms"] for rec in recs) / steps, 4),
        "load_time_bound_ms": bound_ms(recs, link_peak),
    }

    if with_extras and not w.rebuild_each_step:
        # the fingerprint kernel on its own: launches back to back over one loaded model's
        # slots (in a step it runs right after a long link-bound phase during which the
        # memory clocks have dropped, which costs it up to a fifth of its bandwidth)
        name = names[-1]
        reg = r.materialise(name)
        ptrs, _info = r.load(name)
        spans = list(zip(ptrs, reg.sizes))
        ms = []
        # launches until 40 ms of kernel time have passed (at least 6, at most 24)
        while len(ms) < 6 or (sum(ms) < 40.0 and len(ms) < 24):
            got, t_ms = tg.tg_fingerprint_ex(spans, r.pool.stream_gather, tuning=tuning, timed=True)
            ms.append(t_ms)
        if got != reg.fps:
            raise RuntimeError("fingerprints of the loaded model differ from its descriptors")
        r.release(name, True)
        best = min(ms[1:])
        out["fingerprint_back_to_back"] = {
            "GBps": round(reg.nbytes / (best * 1e-3) / 1e9, 1), "frac": round(reg.nbytes / (best * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
            "ms": round(best, 4), "bytes": reg.nbytes, "launches": len(ms),
            "first_launch_GBps": round(reg.nbytes / (ms[0] * 1e-3) / 1e9, 1)}

    # a load whose tensors are all resident already (nothing crosses the host link): the same
    # model under another id, so every tensor is gathered device to device and fingerprinted
    if with_extras and not w.rebuild_each_step and not w.load_flags.get("alias"):
        name = names[-1]
        reg = r.materialise(name)
        r.load(name)
        r.release(name, False)                      # retained: its tensors stay and match
        twin = RegisteredModel(987654321, reg.host, reg.offs, reg.sizes, reg.fps)
        times = []
        for _ in range(4):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            _p, info = r.pool.load(twin, verify=verify, details=False)
            times.append(time.perf_counter() - t0)
            tt = info["timing"]
            r.pool.release(twin.model_id, True)
        if info["transfer_bytes"] != 0:
            raise RuntimeError("the twin of a resident model must not need any transfer")
        r.release(name, True)
        best = min(times[1:])
        out["all_resident_load"] = {"GBps": round(reg.nbytes / best / 1e9, 1), "ms": round(best * 1e3, 3),
                                    "gather_ms": round(tt["gather_ms"], 4),
                                    "gather_GBps": round(2 * tt["gather_bytes"] / (tt["gather_ms"] * 1e-3) / 1e9, 1),
                                    "verify_ms": round(tt["verify_ms"], 4)}

    # the confirmation step on its own: (resident copy, fresh copy) pairs of one loaded model,
    # both operands in HBM; and one load planned with TG_PLAN_CONFIRM (the incoming bytes are read
    # over the host link through the pinned image's device mapping)
    if with_extras and not w.rebuild_each_step and not w.load_flags.get("alias"):
        name = names[-1]
        reg = r.materialise(name)
        ptrs, info = r.load(name)
        pairs = [(r.pool.base + op[2], r.pool.base + op[1], op[3]) for op in info["ops"] if op[0] == 0]
        if pairs:
            ms = []
            for _ in range(4):
                differs, t_ms = tg.tg_compare_ex(pairs, r.pool.stream_gather, tuning=tuning, timed=True)
                ms.append(t_ms)
            if any(differs):
                raise RuntimeError("a reused tensor differs from its source")
            nb = sum(p[2] for p in pairs)
            best = min(ms[1:])
            out["compare_d2d"] = {"GBps": round(2 * nb / (best * 1e-3) / 1e9, 1),
                                  "frac": round(2 * nb / (best * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                                  "ms": round(best, 4), "pairs": len(pairs), "bytes_compared": nb}
        r.release(name, True)
        t0 = time.perf_counter()
        _p, info = r.load(name, confirm=True, details=False)
        t_confirm = time.perf_counter() - t0
        tc = info["timing"]
        r.release(name, True)
        out["confirm_load"] = {"ms": round(t_confirm * 1e3, 3), "compare_ms": round(tc["compare_ms"], 3),
                               "compare_bytes": tc["compare_bytes"],
                               "host_side_GBps": round(tc["compare_bytes"] / (tc["compare_ms"] * 1e-3) / 1e9, 2)
                               if tc["compare_ms"] > 0 else 0.0}

    if any(rec.get("n_moves") or rec.get("n_evictions") for rec in recs):
        mv_ms = sum(rec["timing"]["move_ms"] for rec in recs)
        mv_traffic = sum(rec["timing"]["move_traffic_bytes"] for rec in recs)
        out["merge"] = {
            "moved_bytes_per_load": int(sum(rec["moved_bytes"] for rec in recs) / len(recs)),
            "merge_bound_per_load": int(sum(rec["merge_bound"] for rec in recs) / len(recs)),
            "merge_all_bytes": int(st0["capacity"] - st0["free_bytes"]),
            "evicted_bytes_per_load": int(sum(rec["evicted_bytes"] for rec in recs) / len(recs)),
            "move_ms": round(mv_ms / len(recs), 4),
            "move_launches": recs[0]["timing"]["move_launches"],
            "move_traffic_GBps": round(mv_traffic / (mv_ms * 1e-3) / 1e9, 1) if mv_ms > 0 else 0.0,
            "move_traffic_frac_of_hbm_peak": round(mv_traffic / (mv_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4) if mv_ms > 0 else 0.0,
            "moved_GBps": round(sum(rec["timing"]["move_bytes"] for rec in recs) / (mv_ms * 1e-3) / 1e9, 1) if mv_ms > 0 else 0.0,
        }
    if with_cpu:
        log("timing the CPU oracle on the same load ...")
        out["cpu_baseline"] = cpu_baseline(r, w, names[0])
    r.close()
    torch.cuda.empty_cache()
    return out


# ------------------------------------------------------------------ config 5: the 70B model, one plan, segmented Model Cache
def bench_llama70b(args, torch, link_peak, levels, steps, warmup, legs=None):
    """One pool that holds the 90 % sibling; per reuse level `steps` timed loads of the whole
    723-tensor model.  The pinned Model Cache segment is smaller than what a load transfers, so
    it is refilled between feeds; refilling (here: regenerating the synthetic tensors) is outside
    the timed region, everything the library does and every wait for the device is inside."""
    from paper_2512_01357_amd import synth
    from paper_2512_01357_amd import tangram as tg
    from paper_2512_01357_amd.runner import WorkloadRunner

    torch.cuda.empty_cache()
    free, _total = torch.cuda.mem_get_info()
    pool_bytes = int(args.pool_gb * 1e9) if args.pool_gb else int(free - (16 << 30))
    w = synth.workload_llama70b_sweep(pool_bytes, levels)
    log("workload %s: pool %.1f GB, loads %s" % (w.name, w.pool_bytes / 1e9, w.loads))
    r = WorkloadRunner(w, "cuda:0", log=log)
    r.pool.set_profiling(True)
    if args.tune:
        r.pool.set_tuning(**{k: int(v) for k, v in (kv.split("=") for kv in args.tune.split(","))})
    t0 = time.time()
    r.run_setup()
    log("resident sibling in place after %.1f s; pool: %s" % (time.time() - t0, r.pool.stats()))
    st0 = r.pool.stats()
    tuning = tg.tg_pool_get_tuning(r.pool.pool)
    verify = not args.no_verify
    if args.pmc_calibration:
        pmc_calibration_kernel(torch)
    legs = [] if legs is None else legs          # filled as the legs finish, so that a caller keeps what was measured
    for name in w.loads:
        r.materialise(name)
        recs, walls = [], []
        for i in range(warmup + steps):
            torch.cuda.synchronize()
            t_wall = time.perf_counter()
            _ptrs, info = r.load(name, verify=verify, details=False)
            t_rel = time.perf_counter()
            r.release(name, True)
            info["library_s"] += time.perf_counter() - t_rel
            info["model_bytes"] = r.models[name].nbytes
            if i >= warmup:
                recs.append(info)
                walls.append(time.perf_counter() - t_wall)
        st1 = r.pool.stats()
        if any(st1[k] != st0[k] for k in st0 if k != "generation"):
            raise RuntimeError("pool did not return to its starting state: %s vs %s" % (st1, st0))
        total_bytes = sum(rec["model_bytes"] for rec in recs)
        lib_s = sum(rec["library_s"] for rec in recs)
        kernels = kernel_figures(recs, verify, tuning, "llama3-70b-reuse%s" % name.split("-")[1].zfill(2), plain_load=True)
        seg_gb = r.seg_arena.nbytes / 1e9 if r.seg_arena is not None else 0.0
        leg = {
            "metric": METRIC, "value": round(total_bytes / lib_s / 1e9, 3), "unit": "GB/s", "steps": steps, "warmup": warmup,
            "ms_per_step": round(lib_s / steps * 1e3, 3),
            "config": {"workload": "llama3-70b-reuse%s" % name.split("-")[1].zfill(2), "model_bytes": int(total_bytes / steps),
                       "tensors": len(w.models[name].tensors), "plans_per_load": 1, "pool_bytes": w.pool_bytes,
                       "reused_fraction": round(sum(rec["reused_bytes"] for rec in recs) / total_bytes, 4),
                       "reused_tensors": int(sum(rec["n_reused"] for rec in recs) / steps),
                       "designated_shared_tensors": w.designated_shared[name], "verify_fingerprint": verify,
                       "h2d_streams": 2 if r.pool.stream_h2d_second is not None else 1,
                       "feeds_per_load": recs[0]["feeds"],
                       "model_cache": "one pinned segment of %.1f GB, refilled between feeds; refills are outside the "
                                      "timed region (wall time with them: ms_per_step_with_refills)" % seg_gb},
            "ms_per_step_with_refills": round(sum(walls) / steps * 1e3, 3),
            "fingerprint_GBps": kernels["fingerprint"]["achieved"],
            "roofline": dominant_roofline(kernels), "kernels": kernels,
            "host_link": host_link_figures(recs, link_peak),
            "plan_host_ms": round(sum(rec["timing"]["plan_host_ms"] for rec in recs) / steps, 4),
            "load_time_bound_ms": bound_ms(recs, link_peak),
        }
        if recs[0]["feeds"] > 1 and not args.no_extras:
            # the same load with the cache cut in two halves, one refilled while the other is copied
            # to the GPU: what a cold load costs when filling the cache overlaps emptying it (Eq. 3)
            torch.cuda.synchronize()
            _ptrs, oinfo = r.load(name, verify=verify, details=False, overlap=True)
            r.release(name, True)
            refill_s = sum(walls) / steps - lib_s / steps
            leg["overlapped_refills"] = {
                "ms": round(oinfo["overlapped_s"] * 1e3, 3),
                "GBps": round(r.models[name].nbytes / oinfo["overlapped_s"] / 1e9, 3),
                "feeds": oinfo["feeds"],
                "refill_alone_ms": round(refill_s * 1e3, 3),
                "note": "one load; the synthetic refill (tensors regenerated on the GPU, copied device to host on a "
                        "stream chosen by measurement) runs beside the host-to-device copies of the previous piece, so "
                        "the link carries both directions; the first piece is in the cache beforehand; "
                        "refill_alone_ms includes the first piece"}
            from paper_2512_01357_amd import loader
            log("overlapped refills, %s: %.1f ms per load (%.1f GB/s); streams: %s"
                % (name, leg["overlapped_refills"]["ms"], leg["overlapped_refills"]["GBps"],
                   loader.REFILL_MEASUREMENT.get(str(r.pool.device))))
        if name == w.loads[0]:
            # the fingerprint kernel on its own, launched back to back over the loaded model's slots
            ptrs, _info = r.load(name, details=False)
            reg = r.models[name]
            spans = list(zip(ptrs, reg.sizes))
            ms = []
            for _ in range(6):
                got, t_ms = tg.tg_fingerprint_ex(spans, r.pool.stream_gather, tuning=tuning, timed=True)
                ms.append(t_ms)
            if got != reg.fps:
                raise RuntimeError("fingerprints of the loaded model differ from its descriptors")
            r.release(name, True)
            best = min(ms[1:])
            leg["fingerprint_back_to_back"] = {
                "GBps": round(reg.nbytes / (best * 1e-3) / 1e9, 1),
                "frac": round(reg.nbytes / (best * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4), "ms": round(best, 4),
                "bytes": reg.nbytes, "launches": len(ms), "first_launch_GBps": round(reg.nbytes / (ms[0] * 1e-3) / 1e9, 1)}
        log("leg %s: %.1f GB/s, %.1f ms per load (bound %.1f), fingerprint %s GB/s, gather %s GB/s, link %.2f of %.2f GB/s"
            % (leg["config"]["workload"], leg["value"], leg["ms_per_step"], leg["load_time_bound_ms"],
               kernels["fingerprint"]["achieved"], kernels["gather"]["achieved"], leg["host_link"]["achieved"], link_peak))
        legs.append(leg)
    r.close()
    torch.cuda.empty_cache()
    return legs


def probe_alu(torch):
    """The fingerprint's arithmetic without its loads: words per second of the mix on register data."""
    from paper_2512_01357_amd import tangram as tg
    best = 0.0
    for _ in range(5):
        best = max(best, tg.tg_measure_mix_rate(4096))
    print(json.dumps({"probe": "alu-mix", "mix_words_per_s": best, "equivalent_GBps": round(best * 8 / 1e9, 1)}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=9)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama7b",
                    help="tiny | gpt1b | llama7b | neox20b | neox20b-tight | llama70b-0 | llama70b-50 | llama70b-90 | "
                         "merge | merge-listing | merge-notail | merge-small")
    ap.add_argument("--legs", default=None,
                    help="reuse levels of the 70B legs, e.g. 90,0 (default with the default workload: 90,50,0; "
                         "'none' switches them off)")
    ap.add_argument("--leg-steps", type=int, default=2)
    ap.add_argument("--leg-warmup", type=int, default=1)
    ap.add_argument("--alias", action="store_true",
                    help="plan with TG_PLAN_ALIAS: resident tensors are used where they lie")
    ap.add_argument("--no-verify", action="store_true", help="skip the fingerprint of assembled slots")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="only the timed steps (no back-to-back, all-resident, confirm runs)")
    ap.add_argument("--pool-gb", type=float, default=0.0, help="override pool size (70B)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one plain 1 GiB elementwise torch kernel (out = in * 1.0), so that a "
                         "rocprofv3 --pmc run has a kernel of known traffic to scale its counters by")
    ap.add_argument("--probe-alu", action="store_true", help="only measure the fingerprint's mix without loads")
    ap.add_argument("--tune", default="", help="fields of tg_tuning to override, e.g. gather_wgs_per_cu=2,fuse_verify=0")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding or collectives are part of "
              "it); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2512_01357_amd import synth
    from paper_2512_01357_amd import tangram as tg

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    tg.lib()
    if args.probe_alu:
        probe_alu(torch)
        return

    link_peak = measure_link_peak(torch)
    log("host link peak (2 GiB pinned->device): %.2f GB/s" % link_peak)

    if args.workload.startswith("llama70b"):
        level = int(args.workload.split("-")[1]) / 100.0
        leg = bench_llama70b(args, torch, link_peak, (level,), args.steps, args.warmup)[0]
        leg.update({"n_gpus": 1, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u64",
                    "data": "synthetic"})
        print(json.dumps(leg), flush=True)
        return

    w = synth.WORKLOADS[args.workload]()
    if args.alias:
        w.load_flags = dict(w.load_flags, alias=True)
    log("workload %s: pool %.1f GB, loads %s, flags %s" % (w.name, w.pool_bytes / 1e9, w.loads, w.load_flags))
    out = bench_resident(args, torch, w, link_peak, args.steps, args.warmup, with_extras=not args.no_extras,
                         with_cpu=not args.no_cpu_baseline)
    legs = args.legs if args.legs is not None else ("90,50,0" if args.workload == "llama7b" else "none")
    if legs != "none":
        levels = tuple(int(x) / 100.0 for x in re.split(r"[ ,]+", legs.strip()) if x)
        out["legs"] = []
        try:
            bench_llama70b(args, torch, link_peak, levels, args.leg_steps, args.leg_warmup, out["legs"])
        except Exception as e:          # the headline above stands on its own: report it with the legs that finished
            log("70B legs stopped: %r" % (e,))
            out["legs_error"] = repr(e)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()

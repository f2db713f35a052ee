#!/usr/bin/env python3
"""Benchmark of the Load path on one MI355X.

A step is one whole load of a model into a pool that already holds its
sibling(s): tg_plan (match + best-fit), tg_assemble (gather kernel for the
reused tensors overlapped with the host-to-device stream for the missing
ones, then a fingerprint launch over every assembled slot, then commit) and
tg_release with eviction, which puts the pool back as it was.  Steps cycle
through the workload's models (for the 7B family: variants v1, v2, v3).

Prints one JSON line: effective load GB/s (model bytes / step time), with the
roofline of the dominant kernel, the other kernels' figures, the host-link
figure and the CPU oracle's rate on a bounded sample of the same workload.
"""
import argparse
import gc
import json
import os
import statistics
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0        # MI355X published HBM3E bandwidth
ALU_MIX_GBPS = 17100.0        # 2.14e12 mixed words/s x 8 B: the fingerprint's arithmetic without its loads

# HBM bytes per step (the gather launch; the five verify fingerprint launches together) from two rocprofv3 --pmc runs of this file (FETCH_SIZE, then WRITE_SIZE,
# each scaled by what the counter reads for a plain 1 GiB elementwise kernel); measured off line
# for the default workload, so reported only when that workload and launch configuration run.
PMC_TRAFFIC_BYTES = {
    "llama-7b-family": {"fingerprint": (13161268 + 168) * 1024, "gather": (6836866 + 6843164) * 1024},
}


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def measure_link_peak(torch, nbytes=2 << 30, reps=3):
    """GB/s of one large pinned-to-device hipMemcpyAsync (the host link's
    measured peak on this machine, same run): a one-tensor model loaded into an
    empty pool through the library, timed by its HIP events."""
    from paper_2512_01357_amd import tangram as tg
    from paper_2512_01357_amd.loader import HostArena, RegisteredModel, ReusePool
    arena = HostArena(nbytes)
    arena.tensor.fill_(1)
    pool = ReusePool(nbytes, 256, "cuda:0")
    reg = RegisteredModel(1, arena, [0], [nbytes], [0])
    tg.tg_set_profiling(True)
    best = 0.0
    for _ in range(reps + 1):
        pool.load(reg)
        t = tg.tg_last_timing()
        pool.release(1, True)
        best = max(best, nbytes / (t["h2d_ms"] * 1e-3) / 1e9)
    pool.close()
    arena.free()
    torch.cuda.empty_cache()
    return best


def cpu_baseline(runner, w, name, budget_s=20.0):
    """The oracle as it stands, on this machine's host cores, on a bounded sample
    of the workload's load: fingerprint + match/plan + assemble (byte copy
    into its image) of the first tensors of `name`, against a store that holds
    the matching tensors of the resident sibling."""
    import oracle
    from oracle import ReuseStoreOracle

    reg = runner.models[name]
    host = runner.host_numpy(name)
    # calibrate on a small piece, then size the sample to the budget
    probe = host[:32 << 20]
    t0 = time.perf_counter()
    oracle.fingerprint(probe)
    dst = probe.copy()
    oracle.copy_bytes(dst, probe)
    per_byte = (time.perf_counter() - t0) / probe.size
    cores = len(os.sched_getaffinity(0))
    # whole tensors, from the front of the model, until the all-cores leg fills its share
    target_1core = int(budget_s * 0.4 / per_byte)
    order = list(range(len(reg.sizes)))
    sample, total = [], 0
    for k in order:
        if total + reg.sizes[k] > target_1core and sample:
            break
        sample.append(k)
        total += reg.sizes[k]

    def one_pass(n_threads):
        store = ReuseStoreOracle(w.pool_bytes, w.align)
        # resident sibling: the sampled tensors that the real pool also holds
        base_name = w.setup[0][1] if w.setup else None
        t_start = time.perf_counter()
        fps = [0] * len(sample)

        def work(tid):
            for i in range(tid, len(sample), n_threads):
                k = sample[i]
                fps[i] = oracle.fingerprint(host[reg.offs[k]:reg.offs[k] + reg.sizes[k]])
        threads = [threading.Thread(target=work, args=(t,)) for t in range(n_threads)]
        for t in threads:
            t.start()
        for t in threads:
            t.join()
        rows = [(reg.sizes[k], fps[i], reg.offs[k]) for i, k in enumerate(sample)]
        plan = store.plan(999, rows, host)
        # assemble: byte copies into the oracle's image, tensors spread over threads
        import numpy as np
        slots = [None] * len(sample)

        def copy(tid):
            for i in range(tid, len(sample), n_threads):
                op = plan.ops[i]
                slot = np.empty(op.nbytes, dtype=np.uint8)
                oracle.copy_bytes(slot, host[op.src_off:op.src_off + op.nbytes])
                slots[i] = slot
        threads = [threading.Thread(target=copy, args=(t,)) for t in range(n_threads)]
        for t in threads:
            t.start()
        for t in threads:
            t.join()
        return time.perf_counter() - t_start, base_name

    t1, _ = one_pass(1)
    n_thr = min(cores, max(1, len(sample)))
    tn, _ = one_pass(n_thr)
    return {
        "value": round(total / tn / 1e9, 4), "unit": "GB/s", "cores": n_thr, "kind": "oracle",
        "value_1core": round(total / t1 / 1e9, 4),
        "sample": "first %d tensors of %s (%.2f GB): oracle fingerprint + plan + byte-copy assemble, "
                  "no resident sibling (every tensor copied from host memory); %d-thread leg %.1f s, "
                  "1-thread leg %.1f s" % (len(sample), name, total / 1e9, n_thr, tn, t1),
        "host_cores_available": cores,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=9)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama7b",
                    help="tiny | gpt1b | llama7b | neox20b | llama70b-0 | llama70b-50 | llama70b-90 | "
                         "merge | merge-listing | merge-notail | merge-small")
    ap.add_argument("--alias", action="store_true",
                    help="plan with TG_PLAN_ALIAS: resident tensors are used where they lie")
    ap.add_argument("--no-verify", action="store_true", help="skip the fingerprint of assembled slots")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pool-gb", type=float, default=0.0, help="override pool size (70B)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one plain 1 GiB elementwise torch kernel (out = in * 1.0), so that a "
                         "rocprofv3 --pmc run has a kernel of known traffic to scale its counters by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding or collectives are part of "
              "it); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2512_01357_amd import synth
    from paper_2512_01357_amd import tangram as tg
    from paper_2512_01357_amd.runner import WorkloadRunner

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    tg.lib()
    if args.workload.startswith("llama70b"):
        frac = int(args.workload.split("-")[1]) / 100.0
        free, _total = torch.cuda.mem_get_info()
        pool = int(args.pool_gb * 1e9) if args.pool_gb else int(free - (16 << 30))
        w = synth.workload_llama70b(frac, pool)
    else:
        w = synth.WORKLOADS[args.workload]()
    if args.alias:
        w.load_flags = dict(w.load_flags, alias=True)
    log("workload %s: pool %.1f GB, loads %s, flags %s" % (w.name, w.pool_bytes / 1e9, w.loads, w.load_flags))

    link_peak = measure_link_peak(torch)
    log("host link peak (2 GiB pinned->device): %.2f GB/s" % link_peak)

    r = WorkloadRunner(w, "cuda:0", log=log)
    r.run_setup()
    if not w.streamed:
        for name in w.loads:
            r.materialise(name)
    st0 = r.pool.stats()
    log("pool before loads: %s" % st0)
    from paper_2512_01357_amd.loader import SECOND_H2D_MEASUREMENT
    log("host-to-device copies on %s (32 x 4 MiB beside a device copy: %s)"
        % ("two streams" if r.pool.stream_h2d_second is not None else "one stream", SECOND_H2D_MEASUREMENT.get("cuda:0")))

    if args.pmc_calibration:
        a = torch.full((1 << 28,), 1.0, dtype=torch.float32, device="cuda:0")
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        torch.mul(a, 1.0, out=b)          # an elementwise kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del a, b

    verify = not args.no_verify
    tg.tg_set_profiling(True)
    names = w.loads
    baseline = {}

    def step(i):
        """One whole load of one model (+ release).  Returns its records."""
        if w.rebuild_each_step:
            # the load moves or evicts residents: only the load is timed, then the
            # pool is rebuilt from scratch
            name = names[i % len(names)]
            reg = r.materialise(name)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ptrs, info = r.load(name, verify=verify, details=False)
            torch.cuda.synchronize()
            timed = time.perf_counter() - t0
            t = tg.tg_last_timing()
            r.reset_pool()
            return [(name, info, t, reg.nbytes)], timed
        if not w.streamed:
            name = names[i % len(names)]
            ptrs, info = r.load(name, verify=verify, details=False)
            t = tg.tg_last_timing()
            r.release(name, True)
            return [(name, info, t, r.models[name].nbytes)], None
        # streamed: the model passes through the Model Cache part by part; only the
        # loads are timed, filling the cache with the next part is not
        out, timed = [], 0.0
        for name in names:
            reg = r.materialise(name)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ptrs, info = r.load(name, verify=verify, details=False)
            torch.cuda.synchronize()
            timed += time.perf_counter() - t0
            out.append((name, info, tg.tg_last_timing(), reg.nbytes))
            if name == names[-1] and not args.no_cpu_baseline and not baseline and i == args.warmup + args.steps - 1:
                log("timing the CPU oracle on a bounded sample ...")
                baseline.update(cpu_baseline(r, w, name))
            r.drop_host(name)
        t0 = time.perf_counter()
        for name in names:
            r.release(name, True)
        timed += time.perf_counter() - t0
        return out, timed

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    recs = []
    timed_total = 0.0
    # no garbage-collector pass inside the timed region (as timeit does): a full pass over
    # everything torch has imported takes tens of ms, more than 100 loads of the smallest workload
    gc.collect()
    gc.disable()
    t_begin = time.perf_counter()
    for i in range(args.steps):
        out, timed = step(args.warmup + i)
        recs += out
        if timed is not None:
            timed_total += timed
    torch.cuda.synchronize()
    elapsed = timed_total if (w.streamed or w.rebuild_each_step) else time.perf_counter() - t_begin
    gc.enable()
    st1 = r.pool.stats()
    if any(st1[k] != st0[k] for k in st0 if k != "generation"):
        raise RuntimeError("pool did not return to its starting state: %s vs %s" % (st1, st0))

    total_bytes = sum(rec[3] for rec in recs)
    model_bytes_per_step = total_bytes / args.steps
    value = total_bytes / elapsed / 1e9

    def avg(key):
        return sum(rec[2][key] for rec in recs) / len(recs)

    def rate(bytes_key, ms_key, factor=1.0):
        ms = sum(rec[2][ms_key] for rec in recs)
        b = sum(rec[2][bytes_key] for rec in recs)
        return (factor * b / (ms * 1e-3) / 1e9) if ms > 0 else 0.0

    fp_key_ms, fp_key_b = ("verify_ms", "verify_bytes") if verify else ("fingerprint_ms", "fingerprint_bytes")
    fp_gbps = rate(fp_key_b, fp_key_ms)
    gather_gbps = rate("gather_bytes", "gather_ms", 2.0)
    h2d_gbps = rate("h2d_bytes", "h2d_ms")
    kernels = {
        "fingerprint": {"bound": "hbm", "achieved": round(fp_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                        "frac": round(fp_gbps / HBM_PEAK_GBPS, 4), "avg_ms": round(avg(fp_key_ms), 4),
                        "algorithmic_bytes_per_launch": int(sum(rec[2][fp_key_b] for rec in recs) / len(recs)),
                        "traffic": None},
        "gather": {"bound": "hbm", "achieved": round(gather_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                   "frac": round(gather_gbps / HBM_PEAK_GBPS, 4), "avg_ms": round(avg("gather_ms"), 4),
                   "algorithmic_bytes_per_launch": int(2 * sum(rec[2]["gather_bytes"] for rec in recs) / len(recs)),
                   "traffic": None},
    }
    # integer-ALU co-limit of the fingerprint: the mix alone (no loads) sustains 2.14e12 words/s
    # on this chip (measured once with a load-free variant of the kernel), i.e. 17.1 TB/s of input
    kernels["fingerprint"]["alu_colimit"] = {"equivalent_GBps": ALU_MIX_GBPS,
                                             "frac": round(fp_gbps / ALU_MIX_GBPS, 4)}
    if verify and w.name in PMC_TRAFFIC_BYTES and not any(w.load_flags.values()):
        for k, v in PMC_TRAFFIC_BYTES[w.name].items():
            kernels[k]["traffic"] = v
    dominant = max(kernels, key=lambda k: kernels[k]["avg_ms"])
    roofline = dict(kernels[dominant])
    roofline["kernel"] = dominant

    out = {
        "metric": "effective load GB/s (model bytes resident / load time); fingerprint HBM GB/s",
        "value": round(value, 3), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(elapsed / args.steps * 1e3, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u64", "data": "synthetic",
        "config": {"workload": w.name, "model_bytes": int(model_bytes_per_step),
                   "tensors": sum(len(w.models[n].tensors) for n in (names if w.streamed else names[:1])),
                   "pool_bytes": w.pool_bytes,
                   "reused_fraction": round(sum(rec[1]["reused_bytes"] for rec in recs) / total_bytes, 4),
                   "reused_tensors": int(sum(rec[1]["n_reused"] for rec in recs) / args.steps),
                   "designated_shared_tensors": sum(w.designated_shared.values()) // max(1, len(w.designated_shared)),
                   "verify_fingerprint": verify,
                   "plan_flags": sorted(k for k, v in w.load_flags.items() if v),
                   "h2d_streams": 2 if r.pool.stream_h2d_second is not None else 1,
                   "model_cache": ("streamed in %d parts (pinned host memory is capped below the model size); "
                                   "only the loads are timed" % len(names)) if w.streamed else "whole model pinned"},
        "fingerprint_GBps": round(fp_gbps, 1),
        "roofline": roofline,
        "kernels": kernels,
        "host_link": {"achieved": round(h2d_gbps, 2), "peak_measured": round(link_peak, 2), "unit": "GB/s",
                      "frac": round(h2d_gbps / link_peak, 4) if link_peak else None,
                      "avg_ms": round(avg("h2d_ms"), 3), "copies_per_load": recs[0][2]["h2d_copies"]},
        "plan_host_ms": round(avg("plan_host_ms"), 4),
        "load_time_bound_ms": round(max(2 * sum(rec[1]["reused_bytes"] for rec in recs) / (HBM_PEAK_GBPS * 1e9),
                                        sum(rec[1]["transfer_bytes"] for rec in recs) / (link_peak * 1e9))
                                    * 1e3 / args.steps, 3),
    }

    # the fingerprint kernel on its own: launches back to back over one loaded model's
    # slots (in a step it runs once, right after a long link-bound phase during which
    # the memory clocks have dropped, which costs it up to a fifth of its bandwidth)
    if not w.rebuild_each_step:
        name = names[-1]
        reg = r.materialise(name)
        ptrs, _info = r.load(name)
        spans = list(zip(ptrs, reg.sizes))
        ms = []
        # launches until 40 ms of kernel time have passed (at least 6, at most 24): after a
        # link-bound load the first ones still run at the lower clocks
        while len(ms) < 6 or (sum(ms) < 40.0 and len(ms) < 24):
            got = tg.tg_fingerprint(spans, r.pool.stream_gather)
            ms.append(tg.tg_last_timing()["fingerprint_ms"])
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
    if not w.rebuild_each_step and not w.streamed and not w.load_flags.get("alias"):
        from paper_2512_01357_amd.loader import RegisteredModel
        name = names[-1]
        reg = r.materialise(name)
        r.load(name)
        r.release(name, False)                      # retained: its tensors stay and match
        twin = RegisteredModel(987654321, reg.host, reg.offs, reg.sizes, reg.fps)
        times = []
        for _ in range(4):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            _p, info = r.pool.load(twin, verify=verify)
            times.append(time.perf_counter() - t0)
            tt = tg.tg_last_timing()
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
    if not w.rebuild_each_step and not w.load_flags.get("alias"):
        name = names[-1]
        reg = r.materialise(name)
        ptrs, info = r.load(name)
        pairs = [(r.pool.base + op[2], r.pool.base + op[1], op[3]) for op in info["ops"] if op[0] == 0]
        if pairs:
            ms = []
            for _ in range(4):
                differs = tg.tg_compare(pairs, r.pool.stream_gather)
                ms.append(tg.tg_last_timing()["compare_ms"])
            if any(differs):
                raise RuntimeError("a reused tensor differs from its source")
            nb = sum(p[2] for p in pairs)
            best = min(ms[1:])
            out["compare_d2d"] = {"GBps": round(2 * nb / (best * 1e-3) / 1e9, 1),
                                  "frac": round(2 * nb / (best * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                                  "ms": round(best, 4), "pairs": len(pairs), "bytes_compared": nb}
        r.release(name, True)
        t0 = time.perf_counter()
        r.load(name, confirm=True)
        t_confirm = time.perf_counter() - t0
        tc = tg.tg_last_timing()
        r.release(name, True)
        out["confirm_load"] = {"ms": round(t_confirm * 1e3, 3), "compare_ms": round(tc["compare_ms"], 3),
                               "compare_bytes": tc["compare_bytes"],
                               "host_side_GBps": round(tc["compare_bytes"] / (tc["compare_ms"] * 1e-3) / 1e9, 2)
                               if tc["compare_ms"] > 0 else 0.0}

    if any(rec[1].get("n_moves") or rec[1].get("n_evictions") for rec in recs):
        mv_ms = sum(rec[2]["move_ms"] for rec in recs)
        mv_traffic = sum(rec[2]["move_traffic_bytes"] for rec in recs)
        out["merge"] = {
            "moved_bytes_per_load": int(sum(rec[1]["moved_bytes"] for rec in recs) / len(recs)),
            "merge_bound_per_load": int(sum(rec[1]["merge_bound"] for rec in recs) / len(recs)),
            "merge_all_bytes": int(st0["capacity"] - st0["free_bytes"]),
            "evicted_bytes_per_load": int(sum(rec[1]["evicted_bytes"] for rec in recs) / len(recs)),
            "move_ms": round(mv_ms / len(recs), 4),
            "move_launches": recs[0][2]["move_launches"],
            "move_traffic_GBps": round(mv_traffic / (mv_ms * 1e-3) / 1e9, 1) if mv_ms > 0 else 0.0,
            "move_traffic_frac_of_hbm_peak": round(mv_traffic / (mv_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4) if mv_ms > 0 else 0.0,
            "moved_GBps": round(sum(rec[2]["move_bytes"] for rec in recs) / (mv_ms * 1e-3) / 1e9, 1) if mv_ms > 0 else 0.0,
        }
    if not args.no_cpu_baseline:
        if not baseline:
            log("timing the CPU oracle on a bounded sample ...")
            baseline.update(cpu_baseline(r, w, names[0]))
        out["cpu_baseline"] = baseline
    r.close()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()

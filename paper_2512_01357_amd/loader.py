"""Device memory and streams around the C ABI (PyTorch is plumbing here).

``ReusePool`` owns the slab (one torch uint8 tensor on the GPU), two streams
and the library's pool handle; every step of a load is a call into
libtangram.so through ``tangram.py``.  ``HostArena`` is pinned Model Cache
memory from tg_host_alloc, seen as a torch / numpy byte array.
"""
import ctypes
import time
from typing import List, Optional, Sequence, Tuple

import torch

from . import tangram as tg


class HostArena:
    """nbytes of pinned, device-mapped host memory (a Model Cache image)."""

    def __init__(self, nbytes: int):
        self.nbytes = nbytes
        self.ptr = tg.tg_host_alloc(nbytes)
        self._c = (ctypes.c_uint8 * nbytes).from_address(self.ptr)
        self.tensor = torch.frombuffer(self._c, dtype=torch.uint8)

    def numpy(self):
        return self.tensor.numpy()

    def free(self) -> None:
        if self.ptr:
            self.tensor = None
            self._c = None
            tg.tg_host_free(self.ptr)
            self.ptr = 0

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def _host_view(host) -> Tuple[torch.Tensor, int, int]:
    """(uint8 CPU tensor, address, length) of a HostArena or a pinned tensor."""
    if isinstance(host, HostArena):
        return host.tensor, host.ptr, host.nbytes
    if not host.is_pinned():
        raise ValueError("the Model Cache buffer must be pinned host memory")
    return host, host.data_ptr(), host.numel()


class RegisteredModel:
    """A model known to the Reuse Store: per-tensor rows and, if the whole model
    fits the CPU-side Model Cache, its pinned image.  With ``host=None`` only
    the rows exist (``offs`` are then the caller's own references) and the
    missing tensors of a load are handed over segment by segment
    (ReusePool.load_streamed)."""

    def __init__(self, model_id: int, host, offs: Sequence[int], sizes: Sequence[int],
                 fps: Sequence[int]):
        self.model_id = model_id
        self.host = host                       # keeps the pinned memory alive
        if host is None:
            self.host_tensor, ptr, length = None, 0, 0
        else:
            self.host_tensor, ptr, length = _host_view(host)
        self.offs = list(offs)
        self.sizes = list(sizes)
        self.fps = list(fps)
        self.desc = tg.ModelDesc(model_id, ptr, length, list(zip(self.sizes, self.fps, self.offs)))

    @property
    def nbytes(self) -> int:
        return sum(self.sizes)


def fingerprint_host_buffer(host: torch.Tensor, offs: Sequence[int], sizes: Sequence[int],
                            stage_bytes: int = 2 << 30, stream=None,
                            device: str = "cuda:0") -> List[int]:
    """Fingerprints of tensors that live in a host buffer (registration time).

    The bytes are staged through a bounded device buffer in runs of
    consecutive tensors; each run is one host-to-device copy and one
    tg_fingerprint launch over the staged spans.  Tensors that share an offset
    (stored once in the cache) are fingerprinted once.
    """
    n = len(offs)
    fps = [0] * n
    if n == 0:
        return fps
    order = sorted(range(n), key=lambda k: (offs[k], sizes[k]))
    cap = max(stage_bytes, max(sizes))
    cap = (cap + 255) // 256 * 256
    stage = torch.empty(cap + 256, dtype=torch.uint8, device=device)   # room for the phase
    i = 0
    while i < n:
        start = offs[order[i]]
        j = i
        end = start
        while j < n and offs[order[j]] + sizes[order[j]] - start <= cap:
            end = max(end, offs[order[j]] + sizes[order[j]])
            j += 1
        # the run's first byte keeps its 16-byte phase inside the staging buffer
        phase = start % 16
        stage[phase:phase + end - start].copy_(host[start:end])
        torch.cuda.synchronize()
        uniq = {}
        for m in range(i, j):
            uniq.setdefault((offs[order[m]], sizes[order[m]]), []).append(order[m])
        keys = list(uniq)
        got = tg.tg_fingerprint([(stage.data_ptr() + phase + o - start, s) for o, s in keys], stream)
        for key, f in zip(keys, got):
            for k in uniq[key]:
                fps[k] = f
        i = j
    del stage
    return fps


_STREAM_PAIR = {}


def concurrent_stream_pair(device: torch.device, candidates: int = 6):
    """Two torch streams on which a device copy and a host-to-device copy
    really run at the same time.

    HIP multiplexes streams onto a few hardware queues (4 per process on this
    platform) and two streams that share a queue run one after the other, so
    a pair picked blindly overlaps only most of the time.  The pair is chosen
    by measurement, once per device: a 1 GiB device copy on one stream, a
    128 MiB pinned-host copy on the other, alone and together.
    """
    key = str(device)
    if key in _STREAM_PAIR:
        return _STREAM_PAIR[key]
    streams = [torch.cuda.Stream(device=device) for _ in range(candidates)]
    a = torch.empty(1 << 30, dtype=torch.uint8, device=device)
    b = torch.empty(1 << 30, dtype=torch.uint8, device=device)
    c = torch.empty(128 << 20, dtype=torch.uint8, device=device)
    h = torch.empty(128 << 20, dtype=torch.uint8, pin_memory=True)

    def run(sa, sb):
        torch.cuda.synchronize(device)
        t0 = time.perf_counter()
        if sa is not None:
            with torch.cuda.stream(sa):
                for _ in range(4):
                    b.copy_(a, non_blocking=True)
        if sb is not None:
            with torch.cuda.stream(sb):
                c.copy_(h, non_blocking=True)
        torch.cuda.synchronize(device)
        return time.perf_counter() - t0

    run(streams[0], streams[1])                                  # warm-up
    best = (streams[0], streams[1])
    found = False
    for i in range(candidates):
        for j in range(i + 1, candidates):
            alone = run(streams[i], None) + run(None, streams[j])
            both = min(run(streams[i], streams[j]) for _ in range(2))
            if both < 0.8 * alone:
                best, found = (streams[i], streams[j]), True
                break
        if found:
            break
    del a, b, c
    _STREAM_PAIR[key] = best
    _SECOND_H2D[key] = _pick_second_transfer_stream(device, best, [x for x in streams if x not in best], h)
    _SPARE[key] = [x for x in streams if x not in best and x is not _SECOND_H2D[key]]
    del h
    return best


_SECOND_H2D = {}
SECOND_H2D_MEASUREMENT = {}          # what the choice was based on, per device (for logs)


def _pick_second_transfer_stream(device, pair, others, pinned):
    """A third stream whose host-to-device copies run beside those of pair[1]
    (while a kernel runs on pair[0]), or None.  A copy takes about 10 us to
    start on its stream; dealt over two streams that cost disappears -- if the
    two really are independent queues, which only a measurement shows."""
    gather, h2d = pair
    piece = 4 << 20
    n = pinned.numel() // piece
    dst = torch.empty(pinned.numel(), dtype=torch.uint8, device=device)
    a = torch.empty(512 << 20, dtype=torch.uint8, device=device)
    b = torch.empty(512 << 20, dtype=torch.uint8, device=device)

    def run(second):
        torch.cuda.synchronize(device)
        t0 = time.perf_counter()
        with torch.cuda.stream(gather):
            for _ in range(4):
                b.copy_(a, non_blocking=True)
        for k in range(n):
            st = second if (second is not None and k & 1) else h2d
            with torch.cuda.stream(st):
                dst[k * piece:(k + 1) * piece].copy_(pinned[k * piece:(k + 1) * piece], non_blocking=True)
        torch.cuda.synchronize(device)
        return time.perf_counter() - t0

    run(None)
    alone = min(run(None) for _ in range(3))
    best, best_t = None, 0.96 * alone
    tried = []
    for st in others:
        t = min(run(st) for _ in range(3))
        tried.append(round(t * 1e3, 3))
        if t < best_t:
            best, best_t = st, t
    SECOND_H2D_MEASUREMENT[str(device)] = {"one_stream_ms": round(alone * 1e3, 3), "two_streams_ms": tried}
    del dst, a, b
    return best


_SPARE = {}
_REFILL = {}
REFILL_MEASUREMENT = {}              # what that choice was based on, per device (for logs)


def refill_stream(device: torch.device):
    """A stream on which a device-to-host copy runs beside the host-to-device
    copies of a load (the host link carries both directions at once, but only
    between streams that the runtime keeps apart), or None.  A caller whose
    Model Cache is refilled by the GPU -- the synthetic tensors here -- does
    that work on this stream while the previous piece is being copied in.
    Chosen by measurement, once per device: 1 GiB up on the transfer streams,
    1 GiB down on the candidate, alone and together; first with both transfer
    streams of a load in use, then, if nothing runs beside those, with the
    first one only.  Returns (stream, whether the load may keep its second
    transfer stream)."""
    key = str(device)
    if key in _REFILL:
        return _REFILL[key]
    _gather, h2d = concurrent_stream_pair(device)
    second = _SECOND_H2D.get(key)
    n = 1 << 30
    up_h = torch.empty(n, dtype=torch.uint8, pin_memory=True)
    down_h = torch.empty(n, dtype=torch.uint8, pin_memory=True)
    up_d = torch.empty(n, dtype=torch.uint8, device=device)
    down_d = torch.empty(n, dtype=torch.uint8, device=device)
    piece = n // 8

    def run(up, down, two=True):
        torch.cuda.synchronize(device)
        t0 = time.perf_counter()
        if up:
            for k in range(8):
                st = second if (two and second is not None and k & 1) else h2d
                with torch.cuda.stream(st):
                    up_d[k * piece:(k + 1) * piece].copy_(up_h[k * piece:(k + 1) * piece], non_blocking=True)
        if down is not None:
            with torch.cuda.stream(down):
                down_h.copy_(down_d, non_blocking=True)
        torch.cuda.synchronize(device)
        return time.perf_counter() - t0

    candidates = list(_SPARE.get(key, [])) + [torch.cuda.Stream(device=device) for _ in range(2)]
    run(True, candidates[0])
    best, best_t, keep_second = None, None, True
    REFILL_MEASUREMENT[key] = {}
    for two in ([True, False] if second is not None else [False]):
        up_alone = min(run(True, None, two) for _ in range(2))
        tried = []
        for st in candidates:
            down_alone = min(run(False, st) for _ in range(2))
            both = min(run(True, st, two) for _ in range(2))
            tried.append({"down_alone_ms": round(down_alone * 1e3, 2), "both_ms": round(both * 1e3, 2)})
            if both < 0.75 * (up_alone + down_alone) and (best_t is None or both < best_t):
                best, best_t, keep_second = st, both, two
        REFILL_MEASUREMENT[key]["two transfer streams" if two else "one transfer stream"] = {
            "up_alone_ms": round(up_alone * 1e3, 2), "candidates": tried}
        if best is not None:
            break
    del up_h, down_h, up_d, down_d
    _REFILL[key] = (best, keep_second)
    return _REFILL[key]


def second_transfer_stream(device: torch.device):
    """The stream chosen by concurrent_stream_pair's measurement for the second
    half of the host-to-device copies, or None if none helped."""
    concurrent_stream_pair(device)
    return _SECOND_H2D.get(str(device))


class ReusePool:
    """One Unified Memory Pool on one GPU, plus the streams a load runs on."""

    def __init__(self, capacity: int, align: int = 256, device: str = "cuda:0"):
        self.device = torch.device(device)
        self.capacity = capacity
        self.align = align
        self.slab = torch.empty(capacity, dtype=torch.uint8, device=self.device)
        if self.slab.data_ptr() % align:
            raise RuntimeError("slab is not aligned to %d" % align)
        self.stream_gather, self.stream_h2d = concurrent_stream_pair(self.device)
        self.stream_h2d_second = second_transfer_stream(self.device)
        self.pool = tg.tg_pool_create(self.slab.data_ptr(), capacity, align)
        self.base = self.slab.data_ptr()
        self.last_timing: dict = {}            # tg_timing of the most recent load

    def set_tuning(self, **kw) -> None:
        tg.tg_pool_set_tuning(self.pool, **kw)

    def set_profiling(self, on: bool) -> None:
        tg.tg_pool_set_profiling(self.pool, on)

    def close(self) -> None:
        if self.pool is not None:
            tg.tg_pool_destroy(self.pool)
            self.pool = None
        self.slab = None

    def register(self, model_id: int, host, offs: Sequence[int], sizes: Sequence[int],
                 fps: Optional[Sequence[int]] = None, stage_bytes: int = 2 << 30) -> RegisteredModel:
        if fps is None:
            view, _, _ = _host_view(host)
            fps = fingerprint_host_buffer(view, offs, sizes, stage_bytes, self.stream_gather,
                                          str(self.device))
        return RegisteredModel(model_id, host, offs, sizes, fps)

    @staticmethod
    def _plan_flags(confirm=False, evict=False, merge=False, alias=False, pack_text=False, cap_text=False) -> int:
        return ((tg.TG_PLAN_CONFIRM if confirm else 0) | (tg.TG_PLAN_EVICT if evict else 0)
                | (tg.TG_PLAN_MERGE if merge else 0) | (tg.TG_PLAN_ALIAS if alias else 0)
                | (tg.TG_PLAN_PACK_TEXT if pack_text else 0) | (tg.TG_PLAN_CAP_TEXT if cap_text else 0))

    def _plan_info(self, plan, details: bool) -> dict:
        info = tg.tg_plan_info(plan)
        if details:
            rows, _reused, _transfer = tg.tg_plan_ops(plan)
            info.update({"ops": rows, "moves": tg.tg_plan_moves(plan),
                         "evictions": tg.tg_plan_evictions(plan)})
        return info

    def _stream_args(self) -> dict:
        return dict(stream_gather=self.stream_gather, stream_h2d=self.stream_h2d,
                    stream_h2d_second=self.stream_h2d_second,
                    use_second_h2d_stream=self.stream_h2d_second is not None)

    def load(self, model: RegisteredModel, confirm: bool = False, verify: bool = False,
             evict: bool = False, merge: bool = False, alias: bool = False,
             pack_text: bool = False, cap_text: bool = False, details: bool = True) -> Tuple[List[int], dict]:
        """tg_plan + tg_assemble.  Returns device addresses and what the plan held
        (with details=False only its totals: no per-tensor rows are fetched);
        info["timing"] is the plan's tg_timing."""
        flags = self._plan_flags(confirm, evict, merge, alias, pack_text, cap_text)
        plan = tg.tg_plan(self.pool, model.desc, flags, self.stream_gather)
        try:
            info = self._plan_info(plan, details)
            ptrs = tg.tg_assemble_ex(self.pool, plan, model.desc.n,
                                     tg.TG_ASSEMBLE_VERIFY if verify else 0, **self._stream_args())
            info["timing"] = self.last_timing = tg.tg_plan_timing(plan)
        finally:
            tg.tg_plan_free(plan)
        return ptrs, info

    def load_streamed(self, model: RegisteredModel, segments, verify: bool = False, evict: bool = False,
                      merge: bool = False, alias: bool = False, pack_text: bool = False,
                      cap_text: bool = False, details: bool = True, overlap: bool = False) -> Tuple[List[int], dict]:
        """A load whose missing tensors pass through a Model Cache smaller than
        the model: tg_plan (no host image needed), tg_assemble_begin, then one
        tg_assemble_feed per segment, then tg_assemble_wait.

        ``segments(missing)`` is a generator: given the indices of the tensors
        the plan transfers, it yields (pinned address, length, [(tensor index,
        offset in the segment)]) each time its buffer holds the next piece.  The
        first piece is asked for before the load begins (the Model Cache holds it
        when the model is switched in); the generator is resumed only after the
        device has finished everything that the previous feed started, so that
        whatever it does to refill its buffer never runs beside the load's own
        kernels and copies.
        info["library_s"] is the time spent inside the library's calls and
        waiting for the device; the rest of the wall time is the generator
        refilling its buffer.

        With ``overlap`` the generator is resumed right after a piece has been
        fed, while that piece's copies are in flight, and the wait for them
        comes afterwards: filling the cache and emptying it run side by side,
        so the slower of the two sets the time (Eq. 3).  The generator must
        then fill a buffer other than the one it yielded last.
        info["overlapped_s"] is the wall time from tg_plan to the end of the
        load, without the first piece (which the cache holds beforehand)."""
        flags = self._plan_flags(False, evict, merge, alias, pack_text, cap_text)
        t_start = t0 = time.perf_counter()
        plan = tg.tg_plan(self.pool, model.desc, flags, self.stream_gather)
        lib_s = time.perf_counter() - t0
        try:
            info = self._plan_info(plan, True)
            missing = [k for k, op in enumerate(info["ops"]) if op[0] == tg.TG_OP_H2D]
            if not details:
                for key in ("ops", "moves", "evictions"):
                    info.pop(key)
            pieces = iter(segments(missing))
            t_first = time.perf_counter()
            piece = next(pieces, None)                       # the cache's first piece: there before the load starts
            torch.cuda.synchronize(self.device)
            t_first = time.perf_counter() - t_first
            t0 = time.perf_counter()
            streams = self._stream_args()
            if overlap and not refill_stream(self.device)[1]:
                streams.update(stream_h2d_second=None, use_second_h2d_stream=False)
            tg.tg_assemble_begin(self.pool, plan, tg.TG_ASSEMBLE_VERIFY if verify else 0, **streams)
            lib_s += time.perf_counter() - t0
            n_feeds = 0
            while piece is not None:
                ptr, nbytes, rows = piece
                t0 = time.perf_counter()
                ticket = tg.tg_assemble_feed(self.pool, plan, ptr, nbytes, rows)
                n_feeds += 1
                if overlap:
                    lib_s += time.perf_counter() - t0
                    piece = next(pieces, None)               # the next piece is fetched while this one is copied
                    t0 = time.perf_counter()
                    tg.tg_assemble_feed_wait(self.pool, plan, ticket)
                    lib_s += time.perf_counter() - t0
                    continue
                tg.tg_assemble_feed_wait(self.pool, plan, ticket)
                lib_s += time.perf_counter() - t0
                # the fingerprints of this piece finish before the refill of the next one starts
                t0 = time.perf_counter()
                self.stream_gather.synchronize()
                lib_s += time.perf_counter() - t0
                piece = next(pieces, None)
            t0 = time.perf_counter()
            ptrs = tg.tg_assemble_wait(self.pool, plan, model.desc.n)
            lib_s += time.perf_counter() - t0
            info["timing"] = self.last_timing = tg.tg_plan_timing(plan)
            info["library_s"] = lib_s
            info["overlapped_s"] = time.perf_counter() - t_start - t_first
            info["feeds"] = n_feeds
        finally:
            tg.tg_plan_free(plan)
        return ptrs, info

    def set_model_cost(self, model_id: int, miss_prob: float, load_bw: float, alpha: float = 1.0) -> None:
        tg.tg_set_model_cost(self.pool, model_id, miss_prob, load_bw, alpha)

    def release(self, model_id: int, evict: bool = False) -> None:
        tg.tg_release(self.pool, model_id, tg.TG_RELEASE_EVICT if evict else 0)

    def stats(self) -> dict:
        return tg.tg_pool_stats(self.pool)

    def view(self, ptr: int, nbytes: int) -> torch.Tensor:
        """The slab bytes at a returned address, as a uint8 device tensor."""
        off = ptr - self.base
        if off < 0 or off + nbytes > self.capacity:
            raise ValueError("address outside the pool")
        return self.slab[off:off + nbytes]

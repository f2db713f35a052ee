"""ctypes binding of libtangram.so: the same names as include/tangram.h.

Argument marshalling only -- every step of the Load path (fingerprint, match,
allocation, gather, host-to-device stream, commit) runs inside the library.
There is no fallback: if the shared object is missing or fails to load, the
import of this module's functions raises.
"""
import ctypes
import os
from typing import List, Optional, Sequence, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtangram.so")

TG_OK = 0
TG_ERR_INVALID = -1
TG_ERR_NOSPACE = -2
TG_ERR_STALE = -3
TG_ERR_NOTFOUND = -4
TG_ERR_HIP = -5
TG_ERR_NOMEM = -6
TG_ERR_CORRUPT = -7

TG_PLAN_CONFIRM = 1
TG_PLAN_EVICT = 2
TG_PLAN_MERGE = 4
TG_PLAN_ALIAS = 8
TG_PLAN_PACK_TEXT = 16
TG_PLAN_CAP_TEXT = 32
TG_ASSEMBLE_VERIFY = 1
TG_RELEASE_EVICT = 1
TG_OP_REUSE = 0
TG_OP_H2D = 1


class tg_span(ctypes.Structure):
    _fields_ = [("ptr", ctypes.c_void_p), ("nbytes", ctypes.c_uint64)]


class tg_pair(ctypes.Structure):
    _fields_ = [("a", ctypes.c_void_p), ("b", ctypes.c_void_p), ("nbytes", ctypes.c_uint64)]


class tg_tensor_desc(ctypes.Structure):
    _fields_ = [("nbytes", ctypes.c_uint64), ("fp", ctypes.c_uint64), ("src_off", ctypes.c_uint64)]


class tg_model_desc(ctypes.Structure):
    _fields_ = [("model_id", ctypes.c_uint64), ("host_base", ctypes.c_void_p),
                ("host_bytes", ctypes.c_uint64), ("n_tensors", ctypes.c_uint32),
                ("reserved", ctypes.c_uint32), ("tensors", ctypes.POINTER(tg_tensor_desc))]


class tg_plan_op(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_uint32), ("reserved", ctypes.c_uint32),
                ("dst_off", ctypes.c_uint64), ("src_off", ctypes.c_uint64),
                ("nbytes", ctypes.c_uint64)]


class tg_stats(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint64) for n in (
        "capacity", "free_bytes", "largest_free", "n_regions", "n_free_regions",
        "n_entries", "n_active", "generation")]


class tg_region(ctypes.Structure):
    _fields_ = [("off", ctypes.c_uint64), ("len", ctypes.c_uint64), ("free", ctypes.c_uint32),
                ("reserved", ctypes.c_uint32)]


class tg_entry(ctypes.Structure):
    _fields_ = [("off", ctypes.c_uint64), ("nbytes", ctypes.c_uint64), ("fp", ctypes.c_uint64),
                ("n_owners", ctypes.c_uint32), ("active_refs", ctypes.c_uint32)]


class tg_assemble_args(ctypes.Structure):
    _fields_ = [("flags", ctypes.c_uint32), ("use_second_h2d_stream", ctypes.c_uint32),
                ("stream_gather", ctypes.c_void_p), ("stream_h2d", ctypes.c_void_p),
                ("stream_h2d_second", ctypes.c_void_p)]


class tg_move(ctypes.Structure):
    _fields_ = [("old_off", ctypes.c_uint64), ("new_off", ctypes.c_uint64), ("nbytes", ctypes.c_uint64)]


class tg_plan_summary(ctypes.Structure):
    _fields_ = ([(n, ctypes.c_uint32) for n in ("n_tensors", "n_evictions", "n_moves", "alias", "n_reused",
                                                "reserved")]
                + [(n, ctypes.c_uint64) for n in (
                    "reused_bytes", "transfer_bytes", "copy_bytes", "evicted_bytes", "moved_bytes",
                    "merge_bound")])


class tg_timing(ctypes.Structure):
    _fields_ = ([(n, ctypes.c_float) for n in (
        "compare_ms", "gather_ms", "h2d_ms", "verify_ms", "plan_host_ms", "move_ms")]
        + [(n, ctypes.c_uint64) for n in ("compare_bytes", "gather_bytes", "h2d_bytes", "verify_bytes")]
        + [(n, ctypes.c_uint32) for n in ("h2d_copies", "move_launches", "verify_launches", "feeds")]
        + [("move_bytes", ctypes.c_uint64), ("move_traffic_bytes", ctypes.c_uint64),
           ("fused_verify_bytes", ctypes.c_uint64)])


class tg_tuning(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint32) for n in (
        "fingerprint_unroll", "fingerprint_wgs_per_cu", "gather_unroll", "gather_wgs_per_cu",
        "compare_unroll", "compare_wgs_per_cu")] + [("h2d_kernel_max_bytes", ctypes.c_uint64),
                                                     ("h2d_group_bytes", ctypes.c_uint64),
                                                     ("fuse_verify", ctypes.c_uint32),
                                                     ("reserved", ctypes.c_uint32)]


class tg_feed_row(ctypes.Structure):
    _fields_ = [("tensor", ctypes.c_uint32), ("reserved", ctypes.c_uint32), ("seg_off", ctypes.c_uint64)]


class TgError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (%d)" % (where, tg_strerror(status), status))


_lib = None

EXPORTS = [
    "tg_pool_create", "tg_pool_destroy", "tg_pool_stats", "tg_pool_regions", "tg_pool_entries",
    "tg_default_tuning", "tg_pool_set_tuning", "tg_pool_get_tuning", "tg_pool_set_profiling",
    "tg_measure_mix_rate", "tg_fingerprint", "tg_fingerprint_ex", "tg_fingerprint_noalloc", "tg_compare", "tg_compare_ex",
    "tg_plan", "tg_plan_ops", "tg_plan_info", "tg_plan_moves", "tg_plan_evictions", "tg_plan_timing", "tg_plan_free",
    "tg_assemble", "tg_assemble_ex", "tg_assemble_async", "tg_assemble_begin", "tg_assemble_feed",
    "tg_assemble_feed_wait", "tg_assemble_wait", "tg_commit", "tg_abandon", "tg_release",
    "tg_set_model_cost", "tg_reuse_size", "tg_host_alloc", "tg_host_free", "tg_host_device_ptr", "tg_shutdown",
    "tg_strerror",
]


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                "libtangram.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                "or `python paper_2512_01357_amd/build.py` first")
        L = ctypes.CDLL(LIB_PATH)
        vp, u32, u64, i32 = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_int32
        P = ctypes.POINTER
        sig = {
            "tg_pool_create": ([vp, u64, u32, P(vp)], i32),
            "tg_pool_destroy": ([vp], i32),
            "tg_pool_stats": ([vp, P(tg_stats)], i32),
            "tg_pool_regions": ([vp, P(tg_region), u32, P(u32)], i32),
            "tg_pool_entries": ([vp, P(tg_entry), u32, P(u32)], i32),
            "tg_default_tuning": ([P(tg_tuning)], i32),
            "tg_pool_set_tuning": ([vp, P(tg_tuning)], i32),
            "tg_pool_get_tuning": ([vp, P(tg_tuning)], i32),
            "tg_pool_set_profiling": ([vp, ctypes.c_int], i32),
            "tg_fingerprint": ([P(tg_span), u32, P(u64), vp], i32),
            "tg_fingerprint_ex": ([P(tg_span), u32, P(u64), vp, P(tg_tuning), P(ctypes.c_float)], i32),
            "tg_compare_ex": ([P(tg_pair), u32, P(u32), vp, P(tg_tuning), P(ctypes.c_float)], i32),
            "tg_plan_timing": ([vp, P(tg_timing)], i32),
            "tg_assemble_async": ([vp, vp, P(tg_assemble_args)], i32),
            "tg_assemble_begin": ([vp, vp, P(tg_assemble_args)], i32),
            "tg_assemble_feed": ([vp, vp, vp, u64, P(tg_feed_row), u32, P(u32)], i32),
            "tg_assemble_feed_wait": ([vp, vp, u32], i32),
            "tg_assemble_wait": ([vp, vp, P(vp)], i32),
            "tg_fingerprint_noalloc": ([P(tg_span), u32, P(u64), vp], i32),
            "tg_compare": ([P(tg_pair), u32, P(u32), vp], i32),
            "tg_plan": ([vp, P(tg_model_desc), u32, vp, P(vp)], i32),
            "tg_plan_ops": ([vp, P(P(tg_plan_op)), P(u32), P(u64), P(u64)], i32),
            "tg_plan_info": ([vp, P(tg_plan_summary)], i32),
            "tg_plan_moves": ([vp, P(P(tg_move)), P(u32)], i32),
            "tg_plan_evictions": ([vp, P(P(u64)), P(u32)], i32),
            "tg_set_model_cost": ([vp, u64, ctypes.c_double, ctypes.c_double, ctypes.c_double], i32),
            "tg_plan_free": ([vp], None),
            "tg_assemble": ([vp, vp, u32, vp, vp, P(vp)], i32),
            "tg_assemble_ex": ([vp, vp, P(tg_assemble_args), P(vp)], i32),
            "tg_commit": ([vp, vp, P(vp)], i32),
            "tg_abandon": ([vp, vp], i32),
            "tg_release": ([vp, u64, u32], i32),
            "tg_reuse_size": ([vp, P(tg_model_desc), ctypes.c_double, P(u64), P(ctypes.c_double)], i32),
            "tg_host_alloc": ([u64, P(vp)], i32),
            "tg_host_free": ([vp], i32),
            "tg_host_device_ptr": ([vp, P(vp)], i32),
            "tg_measure_mix_rate": ([u32, vp, P(ctypes.c_double)], i32),
            "tg_shutdown": ([], None),
            "tg_strerror": ([i32], ctypes.c_char_p),
        }
        for name, (args, res) in sig.items():
            fn = getattr(L, name)
            fn.argtypes = args
            fn.restype = res
        _lib = L
    return _lib


def _check(status: int, where: str) -> None:
    if status != TG_OK:
        raise TgError(status, where)


def tg_strerror(status: int) -> str:
    return lib().tg_strerror(status).decode()


def _stream(stream) -> ctypes.c_void_p:
    """A torch.cuda.Stream, a raw hipStream_t integer, or None (null stream)."""
    if stream is None:
        return ctypes.c_void_p(0)
    if hasattr(stream, "cuda_stream"):
        return ctypes.c_void_p(stream.cuda_stream)
    return ctypes.c_void_p(int(stream))


# --------------------------------------------------------------------- pool
def tg_pool_create(dev_base: int, capacity: int, align: int = 256) -> ctypes.c_void_p:
    out = ctypes.c_void_p()
    _check(lib().tg_pool_create(ctypes.c_void_p(dev_base), capacity, align, ctypes.byref(out)),
           "tg_pool_create")
    return out


def tg_pool_destroy(pool) -> None:
    _check(lib().tg_pool_destroy(pool), "tg_pool_destroy")


def tg_pool_stats(pool) -> dict:
    st = tg_stats()
    _check(lib().tg_pool_stats(pool, ctypes.byref(st)), "tg_pool_stats")
    return {n: int(getattr(st, n)) for n, _ in tg_stats._fields_}


def tg_pool_regions(pool) -> List[Tuple[int, int, bool]]:
    """(offset, length, is_free) rows of the Region List in physical order."""
    n = ctypes.c_uint32()
    _check(lib().tg_pool_regions(pool, None, 0, ctypes.byref(n)), "tg_pool_regions")
    arr = (tg_region * max(n.value, 1))()
    _check(lib().tg_pool_regions(pool, arr, n.value, ctypes.byref(n)), "tg_pool_regions")
    return [(int(arr[i].off), int(arr[i].len), bool(arr[i].free)) for i in range(n.value)]


def tg_pool_entries(pool) -> List[Tuple[int, int, int, int, int]]:
    """(offset, nbytes, fingerprint, owners, active refs) rows of the Tensor Mapping, by offset."""
    n = ctypes.c_uint32()
    _check(lib().tg_pool_entries(pool, None, 0, ctypes.byref(n)), "tg_pool_entries")
    arr = (tg_entry * max(n.value, 1))()
    _check(lib().tg_pool_entries(pool, arr, n.value, ctypes.byref(n)), "tg_pool_entries")
    return [(int(arr[i].off), int(arr[i].nbytes), int(arr[i].fp), int(arr[i].n_owners), int(arr[i].active_refs))
            for i in range(n.value)]


# ---------------------------------------------------------------- device ops
def _span_array(spans):
    n = len(spans)
    arr = (tg_span * max(n, 1))()
    for i, (ptr, nbytes) in enumerate(spans):
        arr[i].ptr = ptr
        arr[i].nbytes = nbytes
    return arr, n


def _tuning(tuning: Optional[dict]):
    """A tg_tuning made of the defaults overridden by `tuning`, or None."""
    if tuning is None:
        return None
    cur = tg_default_tuning()
    cur.update(tuning)
    return tg_tuning(**cur)


def tg_fingerprint(spans: Sequence[Tuple[int, int]], stream=None) -> List[int]:
    """spans: (device address, nbytes) rows.  Returns their fingerprints."""
    arr, n = _span_array(spans)
    out = (ctypes.c_uint64 * max(n, 1))()
    _check(lib().tg_fingerprint(arr, n, out, _stream(stream)), "tg_fingerprint")
    return [int(out[i]) for i in range(n)]


def tg_fingerprint_ex(spans: Sequence[Tuple[int, int]], stream=None, tuning: Optional[dict] = None,
                      timed: bool = False) -> Tuple[List[int], Optional[float]]:
    """(fingerprints, kernel milliseconds or None); tuning: fields of tg_tuning to override."""
    arr, n = _span_array(spans)
    out = (ctypes.c_uint64 * max(n, 1))()
    t = _tuning(tuning)
    ms = ctypes.c_float()
    _check(lib().tg_fingerprint_ex(arr, n, out, _stream(stream), ctypes.byref(t) if t is not None else None,
                                   ctypes.byref(ms) if timed else None), "tg_fingerprint_ex")
    return [int(out[i]) for i in range(n)], (float(ms.value) if timed else None)


TG_NOALLOC_MAX_SPANS = 4096


def tg_fingerprint_noalloc(spans: Sequence[Tuple[int, int]], stream=None) -> List[int]:
    """tg_fingerprint through the entry point that allocates nothing (at most
    TG_NOALLOC_MAX_SPANS spans)."""
    arr, n = _span_array(spans)
    out = (ctypes.c_uint64 * max(n, 1))()
    _check(lib().tg_fingerprint_noalloc(arr, n, out, _stream(stream)), "tg_fingerprint_noalloc")
    return [int(out[i]) for i in range(n)]


def _pair_array(pairs):
    n = len(pairs)
    arr = (tg_pair * max(n, 1))()
    for i, (a, b, nbytes) in enumerate(pairs):
        arr[i].a = a
        arr[i].b = b
        arr[i].nbytes = nbytes
    return arr, n


def tg_compare(pairs: Sequence[Tuple[int, int, int]], stream=None) -> List[int]:
    """pairs: (address a, address b, nbytes) rows.  1 where the bytes differ."""
    arr, n = _pair_array(pairs)
    out = (ctypes.c_uint32 * max(n, 1))()
    _check(lib().tg_compare(arr, n, out, _stream(stream)), "tg_compare")
    return [int(out[i]) for i in range(n)]


def tg_compare_ex(pairs: Sequence[Tuple[int, int, int]], stream=None, tuning: Optional[dict] = None,
                  timed: bool = False) -> Tuple[List[int], Optional[float]]:
    arr, n = _pair_array(pairs)
    out = (ctypes.c_uint32 * max(n, 1))()
    t = _tuning(tuning)
    ms = ctypes.c_float()
    _check(lib().tg_compare_ex(arr, n, out, _stream(stream), ctypes.byref(t) if t is not None else None,
                               ctypes.byref(ms) if timed else None), "tg_compare_ex")
    return [int(out[i]) for i in range(n)], (float(ms.value) if timed else None)


# --------------------------------------------------------------------- model
class ModelDesc:
    """Owns the ctypes storage behind a tg_model_desc."""

    def __init__(self, model_id: int, host_base: int, host_bytes: int,
                 tensors: Sequence[Tuple[int, int, int]]):
        """tensors: (nbytes, fp, src_off) rows in the model's tensor order."""
        self.n = len(tensors)
        self._rows = (tg_tensor_desc * max(self.n, 1))()
        for k, (nbytes, fp, off) in enumerate(tensors):
            self._rows[k].nbytes = nbytes
            self._rows[k].fp = fp
            self._rows[k].src_off = off
        self.c = tg_model_desc(model_id, host_base, host_bytes, self.n, 0,
                               ctypes.cast(self._rows, ctypes.POINTER(tg_tensor_desc)))
        self.model_id = model_id
        self.nbytes = sum(t[0] for t in tensors)


def tg_plan(pool, model: ModelDesc, flags: int = 0, stream=None) -> ctypes.c_void_p:
    out = ctypes.c_void_p()
    _check(lib().tg_plan(pool, ctypes.byref(model.c), flags, _stream(stream), ctypes.byref(out)),
           "tg_plan")
    return out


def tg_plan_ops(plan) -> Tuple[List[Tuple[int, int, int, int]], int, int]:
    """((kind, dst_off, src_off, nbytes) rows, reused_bytes, transfer_bytes)."""
    ops = ctypes.POINTER(tg_plan_op)()
    n = ctypes.c_uint32()
    reused = ctypes.c_uint64()
    transfer = ctypes.c_uint64()
    _check(lib().tg_plan_ops(plan, ctypes.byref(ops), ctypes.byref(n), ctypes.byref(reused),
                             ctypes.byref(transfer)), "tg_plan_ops")
    rows = [(int(ops[k].kind), int(ops[k].dst_off), int(ops[k].src_off), int(ops[k].nbytes))
            for k in range(n.value)]
    return rows, int(reused.value), int(transfer.value)


_SUMMARY_FIELDS = tuple(n for n, _ in tg_plan_summary._fields_)
_TIMING_FIELDS = tuple(n for n, _ in tg_timing._fields_)


def tg_plan_info(plan) -> dict:
    out = tg_plan_summary()
    _check(lib().tg_plan_info(plan, ctypes.byref(out)), "tg_plan_info")
    return {n: getattr(out, n) for n in _SUMMARY_FIELDS}


def tg_plan_moves(plan) -> List[Tuple[int, int, int]]:
    """(old_off, new_off, nbytes) of the resident tensors the plan moves, in execution order."""
    rows = ctypes.POINTER(tg_move)()
    n = ctypes.c_uint32()
    _check(lib().tg_plan_moves(plan, ctypes.byref(rows), ctypes.byref(n)), "tg_plan_moves")
    return [(int(rows[i].old_off), int(rows[i].new_off), int(rows[i].nbytes)) for i in range(n.value)]


def tg_plan_evictions(plan) -> List[int]:
    """Pool offsets of the tensors the plan evicts, in eviction order."""
    offs = ctypes.POINTER(ctypes.c_uint64)()
    n = ctypes.c_uint32()
    _check(lib().tg_plan_evictions(plan, ctypes.byref(offs), ctypes.byref(n)), "tg_plan_evictions")
    return [int(offs[i]) for i in range(n.value)]


def tg_set_model_cost(pool, model_id: int, miss_prob: float, load_bw: float, alpha: float = 1.0) -> None:
    _check(lib().tg_set_model_cost(pool, model_id, miss_prob, load_bw, alpha), "tg_set_model_cost")


def tg_plan_free(plan) -> None:
    lib().tg_plan_free(plan)


def tg_assemble(pool, plan, n_tensors: int, flags: int = 0, stream_gather=None,
                stream_h2d=None) -> List[int]:
    out = (ctypes.c_void_p * max(n_tensors, 1))()
    _check(lib().tg_assemble(pool, plan, flags, _stream(stream_gather), _stream(stream_h2d), out),
           "tg_assemble")
    return [int(out[k] or 0) for k in range(n_tensors)]


def tg_assemble_ex(pool, plan, n_tensors: int, flags: int = 0, stream_gather=None, stream_h2d=None,
                   stream_h2d_second=None, use_second_h2d_stream: bool = False) -> List[int]:
    out = (ctypes.c_void_p * max(n_tensors, 1))()
    args = tg_assemble_args(flags, 1 if use_second_h2d_stream else 0, _stream(stream_gather),
                            _stream(stream_h2d), _stream(stream_h2d_second))
    _check(lib().tg_assemble_ex(pool, plan, ctypes.byref(args), out), "tg_assemble_ex")
    return [int(out[k] or 0) for k in range(n_tensors)]


def _assemble_args(flags, stream_gather, stream_h2d, stream_h2d_second, use_second_h2d_stream):
    return tg_assemble_args(flags, 1 if use_second_h2d_stream else 0, _stream(stream_gather),
                            _stream(stream_h2d), _stream(stream_h2d_second))


def tg_assemble_async(pool, plan, flags: int = 0, stream_gather=None, stream_h2d=None,
                      stream_h2d_second=None, use_second_h2d_stream: bool = False) -> None:
    args = _assemble_args(flags, stream_gather, stream_h2d, stream_h2d_second, use_second_h2d_stream)
    _check(lib().tg_assemble_async(pool, plan, ctypes.byref(args)), "tg_assemble_async")


def tg_assemble_begin(pool, plan, flags: int = 0, stream_gather=None, stream_h2d=None,
                      stream_h2d_second=None, use_second_h2d_stream: bool = False) -> None:
    args = _assemble_args(flags, stream_gather, stream_h2d, stream_h2d_second, use_second_h2d_stream)
    _check(lib().tg_assemble_begin(pool, plan, ctypes.byref(args)), "tg_assemble_begin")


def tg_assemble_feed(pool, plan, seg_base: int, seg_bytes: int, rows: Sequence[Tuple[int, int]]) -> int:
    """rows: (tensor index, offset inside the segment).  Returns the feed's ticket."""
    n = len(rows)
    arr = (tg_feed_row * max(n, 1))()
    for i, (k, off) in enumerate(rows):
        arr[i].tensor = k
        arr[i].seg_off = off
    ticket = ctypes.c_uint32()
    _check(lib().tg_assemble_feed(pool, plan, ctypes.c_void_p(seg_base), seg_bytes, arr, n,
                                  ctypes.byref(ticket)), "tg_assemble_feed")
    return int(ticket.value)


def tg_assemble_feed_wait(pool, plan, ticket: int) -> None:
    _check(lib().tg_assemble_feed_wait(pool, plan, ticket), "tg_assemble_feed_wait")


def tg_assemble_wait(pool, plan, n_tensors: int) -> List[int]:
    out = (ctypes.c_void_p * max(n_tensors, 1))()
    _check(lib().tg_assemble_wait(pool, plan, out), "tg_assemble_wait")
    return [int(out[k] or 0) for k in range(n_tensors)]


def tg_commit(pool, plan, n_tensors: int) -> List[int]:
    out = (ctypes.c_void_p * max(n_tensors, 1))()
    _check(lib().tg_commit(pool, plan, out), "tg_commit")
    return [int(out[k] or 0) for k in range(n_tensors)]


def tg_abandon(pool, plan) -> None:
    _check(lib().tg_abandon(pool, plan), "tg_abandon")


def tg_release(pool, model_id: int, flags: int = 0) -> None:
    _check(lib().tg_release(pool, model_id, flags), "tg_release")


def tg_reuse_size(pool, model: ModelDesc, link_bytes_per_s: Optional[float] = None
                  ) -> Tuple[int, Optional[float]]:
    reuse = ctypes.c_uint64()
    if link_bytes_per_s is None:
        _check(lib().tg_reuse_size(pool, ctypes.byref(model.c), 0.0, ctypes.byref(reuse), None),
               "tg_reuse_size")
        return int(reuse.value), None
    est = ctypes.c_double()
    _check(lib().tg_reuse_size(pool, ctypes.byref(model.c), link_bytes_per_s, ctypes.byref(reuse),
                               ctypes.byref(est)), "tg_reuse_size")
    return int(reuse.value), float(est.value)


# ------------------------------------------------------------ tuning, timing
def tg_default_tuning() -> dict:
    t = tg_tuning()
    _check(lib().tg_default_tuning(ctypes.byref(t)), "tg_default_tuning")
    return {n: int(getattr(t, n)) for n, _ in tg_tuning._fields_}


def tg_pool_get_tuning(pool) -> dict:
    t = tg_tuning()
    _check(lib().tg_pool_get_tuning(pool, ctypes.byref(t)), "tg_pool_get_tuning")
    return {n: int(getattr(t, n)) for n, _ in tg_tuning._fields_}


def tg_pool_set_tuning(pool, **kw) -> None:
    """Overrides the named fields of the pool's tg_tuning."""
    cur = tg_pool_get_tuning(pool)
    cur.update(kw)
    t = tg_tuning(**cur)
    _check(lib().tg_pool_set_tuning(pool, ctypes.byref(t)), "tg_pool_set_tuning")


def tg_pool_set_profiling(pool, on: bool) -> None:
    _check(lib().tg_pool_set_profiling(pool, 1 if on else 0), "tg_pool_set_profiling")


def tg_plan_timing(plan) -> dict:
    t = tg_timing()
    _check(lib().tg_plan_timing(plan, ctypes.byref(t)), "tg_plan_timing")
    return {n: getattr(t, n) for n in _TIMING_FIELDS}


def tg_host_alloc(nbytes: int) -> int:
    """Address of nbytes of pinned, device-mapped host memory."""
    out = ctypes.c_void_p()
    _check(lib().tg_host_alloc(nbytes, ctypes.byref(out)), "tg_host_alloc")
    return int(out.value)


def tg_host_free(ptr: int) -> None:
    _check(lib().tg_host_free(ctypes.c_void_p(ptr)), "tg_host_free")


def tg_measure_mix_rate(iters: int = 4096, stream=None) -> float:
    """Words per second of the fingerprint's arithmetic without its loads."""
    out = ctypes.c_double()
    _check(lib().tg_measure_mix_rate(iters, _stream(stream), ctypes.byref(out)), "tg_measure_mix_rate")
    return float(out.value)


def tg_host_device_ptr(ptr: int) -> int:
    """The device-side address of a piece of pinned host memory."""
    out = ctypes.c_void_p()
    _check(lib().tg_host_device_ptr(ctypes.c_void_p(ptr), ctypes.byref(out)), "tg_host_device_ptr")
    return int(out.value)


def tg_shutdown() -> None:
    lib().tg_shutdown()

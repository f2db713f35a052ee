"""ctypes access to ``oracle.c`` (oracle, test infrastructure).

The shared object is built with gcc on first use when it is missing or older
than its source; nothing here touches the HIP library.
"""
import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lock = threading.Lock()
_lib = None


def build_liboracle(force: bool = False) -> str:
    """Compile ``oracle.c`` with gcc at -O2 and return the library's path."""
    stale = (not os.path.exists(_LIB)
             or os.path.getmtime(_LIB) < os.path.getmtime(_SRC))
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fPIC", "-shared",
             "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(build_liboracle())
            lib.tgo_splitmix64.argtypes = [ctypes.c_uint64]
            lib.tgo_splitmix64.restype = ctypes.c_uint64
            lib.tgo_fingerprint.argtypes = [ctypes.c_void_p, ctypes.c_uint64]
            lib.tgo_fingerprint.restype = ctypes.c_uint64
            lib.tgo_bytes_equal.argtypes = [ctypes.c_void_p, ctypes.c_void_p,
                                            ctypes.c_uint64]
            lib.tgo_bytes_equal.restype = ctypes.c_int
            lib.tgo_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p,
                                     ctypes.c_uint64]
            lib.tgo_copy.restype = None
            _lib = lib
    return _lib


def _as_u8(buf) -> np.ndarray:
    """A contiguous uint8 view of ``buf`` (bytes, bytearray, numpy array)."""
    if isinstance(buf, np.ndarray):
        arr = buf
        if arr.dtype != np.uint8:
            arr = arr.view(np.uint8)
        arr = arr.reshape(-1)
    else:
        arr = np.frombuffer(buf, dtype=np.uint8)
    if not arr.flags["C_CONTIGUOUS"]:
        raise ValueError("oracle needs contiguous bytes")
    return arr


def splitmix64(x: int) -> int:
    return int(_load().tgo_splitmix64(ctypes.c_uint64(x & (2**64 - 1))))


def fingerprint(buf) -> int:
    """Fingerprint of a whole tensor's bytes (word index starts at 0)."""
    arr = _as_u8(buf)
    return int(_load().tgo_fingerprint(arr.ctypes.data, arr.size))


def bytes_equal(a, b) -> bool:
    a = _as_u8(a)
    b = _as_u8(b)
    if a.size != b.size:
        return False
    return bool(_load().tgo_bytes_equal(a.ctypes.data, b.ctypes.data, a.size))


def copy_bytes(dst: np.ndarray, src) -> None:
    """dst[:] = src, both uint8 and of equal length, through the C loop."""
    src = _as_u8(src)
    dst = _as_u8(dst)
    if dst.size != src.size:
        raise ValueError("length mismatch")
    if not dst.flags["WRITEABLE"]:
        raise ValueError("destination is read-only")
    _load().tgo_copy(dst.ctypes.data, src.ctypes.data, src.size)

"""Python face of the CPU oracle (oracle/spqt_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's cpu_baseline leg may import this
package; the product package never does.  Everything here is argument marshalling for
the plain C functions; the arithmetic lives in the C file, where each function cites the
passage of the paper it follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "spqt_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over output rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        c = ctypes
        p = c.c_void_p
        lib.spqt_oracle_half_to_double.restype = c.c_double
        lib.spqt_oracle_half_to_double.argtypes = [c.c_uint16]
        lib.spqt_oracle_dequant_row.restype = None
        lib.spqt_oracle_dequant_row.argtypes = [p, p, c.c_int64, c.c_int, c.c_int64, p]
        lib.spqt_oracle_mask.restype = None
        lib.spqt_oracle_mask.argtypes = [p, c.c_int64, c.c_int, c.c_float, p]
        lib.spqt_oracle_gather.restype = c.c_int64
        lib.spqt_oracle_gather.argtypes = [p, c.c_int64, c.c_int, c.c_float, p]
        lib.spqt_oracle_gemv.restype = None
        lib.spqt_oracle_gemv.argtypes = [p, p, c.c_int64, c.c_int64, c.c_int, p, c.c_int,
                                         c.c_float, p]
        lib.spqt_oracle_gemv_rows.restype = None
        lib.spqt_oracle_gemv_rows.argtypes = [p, p, c.c_int64, c.c_int64, c.c_int, p, c.c_int,
                                              c.c_float, p, c.c_int64, p]
        lib.spqt_oracle_partition.restype = None
        lib.spqt_oracle_partition.argtypes = [c.c_int64, c.c_int64, c.c_int64, p, p]
        lib.spqt_oracle_packed_bytes.restype = c.c_int64
        lib.spqt_oracle_packed_bytes.argtypes = [c.c_int64, c.c_int64]
        lib.spqt_oracle_pack.restype = c.c_int
        lib.spqt_oracle_pack.argtypes = [p, p, c.c_int64, c.c_int64, p]
        lib.spqt_oracle_unpack.restype = c.c_int
        lib.spqt_oracle_unpack.argtypes = [p, c.c_int64, c.c_int64, p, p]
        lib.spqt_oracle_packed_bytes_g.restype = c.c_int64
        lib.spqt_oracle_packed_bytes_g.argtypes = [c.c_int64, c.c_int64, c.c_int]
        lib.spqt_oracle_pack_g.restype = c.c_int
        lib.spqt_oracle_pack_g.argtypes = [p, p, c.c_int64, c.c_int64, c.c_int, p]
        lib.spqt_oracle_unpack_g.restype = c.c_int
        lib.spqt_oracle_unpack_g.argtypes = [p, c.c_int64, c.c_int64, c.c_int, p, p]
        lib.spqt_oracle_threads.restype = c.c_int
        lib.spqt_oracle_threads.argtypes = []
        lib.spqt_oracle_set_threads.restype = None
        lib.spqt_oracle_set_threads.argtypes = [c.c_int]
        _lib = lib
    return _lib


def _ptr(a: np.ndarray):
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.c_void_p)


def _u16(a: np.ndarray) -> np.ndarray:
    """fp16 (or already uint16) array -> contiguous uint16 bit patterns."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        return a.view(np.uint16)
    assert a.dtype == np.uint16
    return a


def _x2d(x: np.ndarray) -> np.ndarray:
    x = _u16(x)
    return x.reshape(1, -1) if x.ndim == 1 else x


def half_to_double(bits: int) -> float:
    return float(_load().spqt_oracle_half_to_double(int(bits) & 0xFFFF))


def dequant(q_rowmajor: np.ndarray, scales: np.ndarray, group: int = 128) -> np.ndarray:
    """Dense fp64 matrix Wd[M, K] (small shapes only: it materializes M*K doubles)."""
    q_rowmajor = np.ascontiguousarray(q_rowmajor, dtype=np.uint8)
    s = _u16(scales)
    M, K = q_rowmajor.shape[0], q_rowmajor.shape[1] * 2
    out = np.empty((M, K), dtype=np.float64)
    lib = _load()
    for m in range(M):
        lib.spqt_oracle_dequant_row(_ptr(q_rowmajor), _ptr(s), K, group, m, _ptr(out[m]))
    return out


def mask(x: np.ndarray, thr: float) -> np.ndarray:
    x = _x2d(x)
    keep = np.empty(x.shape[1], dtype=np.uint8)
    _load().spqt_oracle_mask(_ptr(x), x.shape[1], x.shape[0], float(thr), _ptr(keep))
    return keep.astype(bool)


def gather(x: np.ndarray, thr: float):
    """(idx int32[n_ns] ascending, n_ns)."""
    x = _x2d(x)
    idx = np.empty(x.shape[1], dtype=np.int32)
    n = int(_load().spqt_oracle_gather(_ptr(x), x.shape[1], x.shape[0], float(thr), _ptr(idx)))
    return idx[:n].copy(), n


def gemv(q_rowmajor: np.ndarray, scales: np.ndarray, x: np.ndarray, thr: float,
         group: int = 128) -> np.ndarray:
    """y fp64 [batch, M]: masked dense GEMV by definition."""
    q_rowmajor = np.ascontiguousarray(q_rowmajor, dtype=np.uint8)
    s = _u16(scales)
    x = _x2d(x)
    M, K = q_rowmajor.shape[0], q_rowmajor.shape[1] * 2
    assert x.shape[1] == K and s.shape == (M, K // group)
    y = np.empty((x.shape[0], M), dtype=np.float64)
    _load().spqt_oracle_gemv(_ptr(q_rowmajor), _ptr(s), M, K, group, _ptr(x), x.shape[0],
                             float(thr), _ptr(y))
    return y


def gemv_rows(q_rowmajor: np.ndarray, scales: np.ndarray, x: np.ndarray, thr: float,
              rows, group: int = 128) -> np.ndarray:
    """y fp64 [batch, len(rows)] for the chosen output rows only."""
    q_rowmajor = np.ascontiguousarray(q_rowmajor, dtype=np.uint8)
    s = _u16(scales)
    x = _x2d(x)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    M, K = q_rowmajor.shape[0], q_rowmajor.shape[1] * 2
    y = np.empty((x.shape[0], rows.size), dtype=np.float64)
    _load().spqt_oracle_gemv_rows(_ptr(q_rowmajor), _ptr(s), M, K, group, _ptr(x), x.shape[0],
                                  float(thr), _ptr(rows), rows.size, _ptr(y))
    return y


def partition(n_ns: int, parts: int):
    """List of (begin, end) slices of idx[0:n_ns], one per part."""
    lib = _load()
    b, e = ctypes.c_int64(), ctypes.c_int64()
    out = []
    for j in range(parts):
        lib.spqt_oracle_partition(n_ns, parts, j, ctypes.byref(b), ctypes.byref(e))
        out.append((b.value, e.value))
    return out


def packed_bytes(M: int, K: int, group: int = 128) -> int:
    return int(_load().spqt_oracle_packed_bytes_g(M, K, group))


def pack(q_rowmajor: np.ndarray, scales: np.ndarray, group: int = 128) -> np.ndarray:
    q_rowmajor = np.ascontiguousarray(q_rowmajor, dtype=np.uint8)
    s = _u16(scales)
    M, K = q_rowmajor.shape[0], q_rowmajor.shape[1] * 2
    if group not in (64, 128) or K % group:
        raise ValueError("shape not packable: group must be 64 or 128 and divide K")
    assert s.shape == (M, K // group)
    out = np.empty(packed_bytes(M, K, group), dtype=np.uint8)
    rc = _load().spqt_oracle_pack_g(_ptr(q_rowmajor), _ptr(s), M, K, group, _ptr(out))
    if rc != 0:
        raise ValueError("shape not packable")
    return out


def unpack(packed: np.ndarray, M: int, K: int, group: int = 128):
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    q = np.empty((M, K // 2), dtype=np.uint8)
    s = np.empty((M, K // group), dtype=np.uint16)
    rc = _load().spqt_oracle_unpack_g(_ptr(packed), M, K, group, _ptr(q), _ptr(s))
    if rc != 0:
        raise ValueError("shape not packable")
    return q, s.view(np.float16)


def threads() -> int:
    return int(_load().spqt_oracle_threads())


def set_threads(n: int) -> None:
    """Threads the row loops use from now on (the results do not depend on it)."""
    _load().spqt_oracle_set_threads(int(n))

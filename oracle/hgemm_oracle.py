"""ctypes front end of the CPU oracle (``hgemm_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by
the benchmark's ``cpu_baseline`` leg.  It never imports the GPU package, and
the GPU package never imports it.

The oracle computes the definition of HGEMM (paper Section 2.1, C = A*B with
alpha=1, beta=0) the way Section 2.3.2 / Eq. 1 describes the reference: a CPU
product of the up-cast fp16 inputs -- here with fp64 accumulation and a single
round-to-nearest-even to fp16.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hgemm_oracle.c")
_LIB = os.path.join(_HERE, "libhgemm_oracle.so")
_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no fast-math) and return the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        cmd = ["gcc", "-O2", "-fopenmp", "-fno-fast-math", "-ffp-contract=off", "-shared", "-fPIC",
               "-o", tmp, _SRC]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(build())
            i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
            lib.oracle_hgemm.restype = ci
            lib.oracle_hgemm.argtypes = [i64, i64, i64, vp, i64, vp, i64, ci, vp, i64]
            lib.oracle_hgemm_at.restype = ci
            lib.oracle_hgemm_at.argtypes = [i64, i64, i64, vp, i64, vp, i64, ci, i64, vp, vp, vp]
            lib.oracle_hgemm_sum_at.restype = ci
            lib.oracle_hgemm_sum_at.argtypes = [i64, i64, i64, vp, i64, vp, i64, ci, i64, vp, vp, vp]
            lib.oracle_hgemm_acc16.restype = ci
            lib.oracle_hgemm_acc16.argtypes = [i64, i64, i64, i64, vp, i64, vp, i64, ci, vp, i64]
            lib.oracle_hgemm_acc16_at.restype = ci
            lib.oracle_hgemm_acc16_at.argtypes = [i64, i64, i64, i64, vp, i64, vp, i64, ci, i64, vp, vp, vp]
            lib.oracle_half_to_double_n.restype = None
            lib.oracle_half_to_double_n.argtypes = [i64, vp, vp]
            lib.oracle_double_to_half_n.restype = None
            lib.oracle_double_to_half_n.argtypes = [i64, vp, vp]
            _lib = lib
    return _lib


def _as_u16(x: np.ndarray, name: str) -> np.ndarray:
    """View a float16 (or uint16 bit-pattern) 2-D array as C-contiguous uint16."""
    x = np.asarray(x)
    if x.dtype == np.float16:
        x = x.view(np.uint16)
    if x.dtype != np.uint16:
        raise TypeError(f"{name} must be float16 or uint16 bit patterns, got {x.dtype}")
    if x.ndim != 2:
        raise ValueError(f"{name} must be 2-D")
    return np.ascontiguousarray(x)


def _shapes(A, B, b_col_major):
    M, K = A.shape
    if b_col_major:
        N, Kb = B.shape
    else:
        Kb, N = B.shape
    if Kb != K:
        raise ValueError(f"inner dimensions differ: A is {A.shape}, B is {B.shape}, b_col_major={b_col_major}")
    return M, N, K


def hgemm(A, B, b_col_major: bool = False) -> np.ndarray:
    """Full oracle product.  A: (M,K) fp16.  B: (K,N) fp16, or (N,K) when
    ``b_col_major`` (the TN layout of Section 2.2.2).  Returns (M,N) float16."""
    A = _as_u16(A, "A")
    B = _as_u16(B, "B")
    M, N, K = _shapes(A, B, b_col_major)
    C = np.empty((M, N), dtype=np.uint16)
    rc = _load().oracle_hgemm(M, N, K, A.ctypes.data, A.shape[1], B.ctypes.data, B.shape[1],
                              int(bool(b_col_major)), C.ctypes.data, N)
    if rc != 0:
        raise RuntimeError("oracle_hgemm rejected its arguments")
    return C.view(np.float16)


def hgemm_at(A, B, ii, jj, b_col_major: bool = False) -> np.ndarray:
    """Oracle values C[ii[t], jj[t]] only (for shapes too large for the full product)."""
    A = _as_u16(A, "A")
    B = _as_u16(B, "B")
    M, N, K = _shapes(A, B, b_col_major)
    ii = np.ascontiguousarray(ii, dtype=np.int64)
    jj = np.ascontiguousarray(jj, dtype=np.int64)
    if ii.shape != jj.shape or ii.ndim != 1:
        raise ValueError("ii and jj must be 1-D and of equal length")
    out = np.empty(ii.shape[0], dtype=np.uint16)
    rc = _load().oracle_hgemm_at(M, N, K, A.ctypes.data, A.shape[1], B.ctypes.data, B.shape[1],
                                 int(bool(b_col_major)), ii.shape[0], ii.ctypes.data, jj.ctypes.data,
                                 out.ctypes.data)
    if rc != 0:
        raise RuntimeError("oracle_hgemm_at rejected its arguments (index out of range?)")
    return out.view(np.float16)


def hgemm_sum_at(A, B, ii, jj, b_col_major: bool = False) -> np.ndarray:
    """Unrounded fp64 sums at chosen positions."""
    A = _as_u16(A, "A")
    B = _as_u16(B, "B")
    M, N, K = _shapes(A, B, b_col_major)
    ii = np.ascontiguousarray(ii, dtype=np.int64)
    jj = np.ascontiguousarray(jj, dtype=np.int64)
    out = np.empty(ii.shape[0], dtype=np.float64)
    rc = _load().oracle_hgemm_sum_at(M, N, K, A.ctypes.data, A.shape[1], B.ctypes.data, B.shape[1],
                                     int(bool(b_col_major)), ii.shape[0], ii.ctypes.data, jj.ctypes.data,
                                     out.ctypes.data)
    if rc != 0:
        raise RuntimeError("oracle_hgemm_sum_at rejected its arguments")
    return out


def hgemm_acc16(A, B, block: int = 16, b_col_major: bool = False) -> np.ndarray:
    """The 16-bit accumulator variant (Section 1: fp16 accumulators are a valid choice; Section 2.3.2's
    exact-match test is built for them): the running sum is an fp16 value that takes in ``block`` products at a
    time, one round-to-nearest-even per block.  ``block`` = 16 is one matrix-core instruction."""
    A = _as_u16(A, "A")
    B = _as_u16(B, "B")
    M, N, K = _shapes(A, B, b_col_major)
    C = np.empty((M, N), dtype=np.uint16)
    rc = _load().oracle_hgemm_acc16(M, N, K, int(block), A.ctypes.data, A.shape[1], B.ctypes.data, B.shape[1],
                                    int(bool(b_col_major)), C.ctypes.data, N)
    if rc != 0:
        raise RuntimeError("oracle_hgemm_acc16 rejected its arguments")
    return C.view(np.float16)


def hgemm_acc16_at(A, B, ii, jj, block: int = 16, b_col_major: bool = False) -> np.ndarray:
    """Values of the 16-bit accumulator variant at chosen positions."""
    A = _as_u16(A, "A")
    B = _as_u16(B, "B")
    M, N, K = _shapes(A, B, b_col_major)
    ii = np.ascontiguousarray(ii, dtype=np.int64)
    jj = np.ascontiguousarray(jj, dtype=np.int64)
    if ii.shape != jj.shape or ii.ndim != 1:
        raise ValueError("ii and jj must be 1-D and of equal length")
    out = np.empty(ii.shape[0], dtype=np.uint16)
    rc = _load().oracle_hgemm_acc16_at(M, N, K, int(block), A.ctypes.data, A.shape[1], B.ctypes.data, B.shape[1],
                                       int(bool(b_col_major)), ii.shape[0], ii.ctypes.data, jj.ctypes.data,
                                       out.ctypes.data)
    if rc != 0:
        raise RuntimeError("oracle_hgemm_acc16_at rejected its arguments (index out of range?)")
    return out.view(np.float16)


def half_bits_to_double(h) -> np.ndarray:
    h = np.ascontiguousarray(h, dtype=np.uint16).ravel()
    d = np.empty(h.shape[0], dtype=np.float64)
    _load().oracle_half_to_double_n(h.shape[0], h.ctypes.data, d.ctypes.data)
    return d


def double_to_half_bits(d) -> np.ndarray:
    d = np.ascontiguousarray(d, dtype=np.float64).ravel()
    h = np.empty(d.shape[0], dtype=np.uint16)
    _load().oracle_double_to_half_n(d.shape[0], d.ctypes.data, h.ctypes.data)
    return h


def threads() -> int:
    """Number of OpenMP threads the oracle will use (OMP_NUM_THREADS, else all cores)."""
    v = os.environ.get("OMP_NUM_THREADS")
    if v and v.isdigit() and int(v) > 0:
        return int(v)
    return os.cpu_count() or 1

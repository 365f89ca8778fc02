"""ctypes binding of the C ABI (include/hgemm.h).  Same names, argument marshalling only.

PyTorch appears here only as the owner of device memory and streams: tensors are
passed as raw device pointers, the current torch stream as a ``hipStream_t``.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libhgemm.so")

# every symbol include/hgemm.h declares
EXPORTS = (
    "hgemm_plan", "hgemm_plan_override", "hgemm_run", "hgemm_destroy", "hgemm_status_string",
    "hgemm_plan_describe", "hgemm_plan_workspace_bytes", "hgemm_plan_launch_info", "hgemm_spec_help",
    "hgemm_candidates", "hgemm_tiles", "hgemm_padded", "hgemm_tile_of_workgroup",
    "hgemm_calibrate_mfma", "hgemm_calibrate_hbm_read", "hgemm_predict_us", "hgemm_run_static", "hgemm_run_many", "hgemm_plan_choice",
)

STATIC_SCRATCH_BYTES = 64 << 20      # HGEMM_STATIC_SCRATCH_BYTES of include/hgemm.h
ERR_WORKSPACE = 6

ROW_MAJOR, COL_MAJOR = 0, 1


class HgemmError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {status_string(status)} (status {status})")


class Layouts(ctypes.Structure):
    _fields_ = [("a", ctypes.c_int), ("b", ctypes.c_int), ("c", ctypes.c_int),
                ("lda", ctypes.c_int64), ("ldb", ctypes.c_int64), ("ldc", ctypes.c_int64)]

    @classmethod
    def make(cls, b_col_major: bool = False, lda: int = 0, ldb: int = 0, ldc: int = 0) -> "Layouts":
        return cls(ROW_MAJOR, COL_MAJOR if b_col_major else ROW_MAJOR, ROW_MAJOR, lda, ldb, ldc)


_lib = None


def lib_path() -> str:
    return _LIB_PATH


def load() -> ctypes.CDLL:
    """Load libhgemm.so (built by paper_2512_02551_amd.build).  No fallback: a missing library is an error."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: run `python -m paper_2512_02551_amd.build` "
                          "(or __graft_entry__.build()) first; there is no CPU fallback")
    # PyTorch ships its own copy of the HIP runtime.  Device pointers and streams handed to this
    # library come from torch, so both must sit on ONE runtime: import torch first, then the dynamic
    # loader binds libhgemm.so to the runtime that is already in the process.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(_LIB_PATH)
    _check_single_hip_runtime()
    i64, vp, ci, cp = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int, ctypes.c_char_p
    lp = ctypes.POINTER(Layouts)
    lib.hgemm_plan.restype = ci
    lib.hgemm_plan.argtypes = [ctypes.POINTER(vp), i64, i64, i64, lp]
    lib.hgemm_plan_override.restype = ci
    lib.hgemm_plan_override.argtypes = [ctypes.POINTER(vp), i64, i64, i64, lp, cp]
    lib.hgemm_run.restype = ci
    lib.hgemm_run.argtypes = [vp, vp, vp, vp, vp]
    lib.hgemm_run_many.restype = ci
    lib.hgemm_run_many.argtypes = [vp, i64, i64, i64, vp, vp, vp, vp]
    lib.hgemm_run_static.restype = ci
    lib.hgemm_run_static.argtypes = [i64, i64, i64, lp, vp, vp, vp, vp]
    lib.hgemm_destroy.restype = ci
    lib.hgemm_destroy.argtypes = [vp]
    lib.hgemm_status_string.restype = cp
    lib.hgemm_status_string.argtypes = [ci]
    lib.hgemm_plan_describe.restype = ci
    lib.hgemm_plan_describe.argtypes = [vp, ctypes.c_char_p, ctypes.c_size_t]
    lib.hgemm_plan_workspace_bytes.restype = ctypes.c_size_t
    lib.hgemm_plan_workspace_bytes.argtypes = [vp]
    lib.hgemm_plan_launch_info.restype = ci
    lib.hgemm_plan_launch_info.argtypes = [vp, ctypes.POINTER(i64), ctypes.POINTER(i64), ctypes.POINTER(i64)]
    lib.hgemm_spec_help.restype = cp
    lib.hgemm_spec_help.argtypes = []
    lib.hgemm_candidates.restype = ci
    lib.hgemm_candidates.argtypes = [i64, i64, i64, lp, ctypes.c_char_p, ctypes.c_size_t]
    lib.hgemm_plan_choice.restype = ci
    lib.hgemm_plan_choice.argtypes = [i64, i64, i64, lp, ctypes.c_char_p, ctypes.c_size_t]
    lib.hgemm_predict_us.restype = ci
    lib.hgemm_predict_us.argtypes = [i64, i64, i64, cp, ctypes.POINTER(ctypes.c_double)]
    lib.hgemm_tiles.restype = i64
    lib.hgemm_tiles.argtypes = [i64, i64]
    lib.hgemm_padded.restype = i64
    lib.hgemm_padded.argtypes = [i64, i64]
    lib.hgemm_tile_of_workgroup.restype = i64
    lib.hgemm_tile_of_workgroup.argtypes = [i64, i64, i64, i64]
    lib.hgemm_calibrate_mfma.restype = ci
    lib.hgemm_calibrate_mfma.argtypes = [i64, vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    lib.hgemm_calibrate_hbm_read.restype = ci
    lib.hgemm_calibrate_hbm_read.argtypes = [vp, ctypes.c_size_t, vp, ctypes.POINTER(ctypes.c_double)]
    _lib = lib
    return lib


def _check_single_hip_runtime() -> None:
    try:
        with open("/proc/self/maps") as f:
            paths = {line.split()[-1] for line in f if "libamdhip64" in line}
    except OSError:
        return
    if len(paths) > 1:
        raise ImportError("two HIP runtimes are loaded in this process (" + ", ".join(sorted(paths)) +
                          "): import torch before loading libhgemm.so so that they share one")


def status_string(status: int) -> str:
    return load().hgemm_status_string(int(status)).decode()


def spec_help() -> str:
    return load().hgemm_spec_help().decode()


def tiles(dim: int, tile: int) -> int:
    return int(load().hgemm_tiles(dim, tile))


def padded(dim: int, tile: int) -> int:
    return int(load().hgemm_padded(dim, tile))


def tile_of_workgroup(wg: int, tiles_m: int, tiles_n: int, swizzle: int) -> int:
    return int(load().hgemm_tile_of_workgroup(wg, tiles_m, tiles_n, swizzle))


def candidates(M: int, N: int, K: int, layouts: Optional[Layouts] = None) -> list:
    buf = ctypes.create_string_buffer(1 << 19)
    st = load().hgemm_candidates(M, N, K, ctypes.byref(layouts) if layouts is not None else None, buf, len(buf))
    if st != 0:
        raise HgemmError(st, "hgemm_candidates")
    return [s for s in buf.value.decode().split("\n") if s]


def plan_choice(M: int, N: int, K: int, layouts: Optional[Layouts] = None) -> str:
    """What hgemm_plan would choose for the problem, and from where ("table: ...", "model: ..."); host only."""
    buf = ctypes.create_string_buffer(512)
    st = load().hgemm_plan_choice(M, N, K, ctypes.byref(layouts) if layouts is not None else None, buf, len(buf))
    if st != 0:
        raise HgemmError(st, "hgemm_plan_choice")
    return buf.value.decode()


def predict_us(M: int, N: int, K: int, spec: str) -> float:
    """The planner's cost-model prediction for one specialisation (host only)."""
    us = ctypes.c_double()
    st = load().hgemm_predict_us(M, N, K, spec.encode(), ctypes.byref(us))
    if st != 0:
        raise HgemmError(st, f"hgemm_predict_us({spec!r})")
    return us.value


class Plan:
    """Owns one hgemm_plan_t."""

    def __init__(self, M: int, N: int, K: int, layouts: Optional[Layouts] = None, spec: Optional[str] = None):
        lib = load()
        self._h = ctypes.c_void_p()
        self.M, self.N, self.K = int(M), int(N), int(K)
        lref = ctypes.byref(layouts) if layouts is not None else None
        if spec is None:
            st = lib.hgemm_plan(ctypes.byref(self._h), M, N, K, lref)
            what = "hgemm_plan"
        else:
            st = lib.hgemm_plan_override(ctypes.byref(self._h), M, N, K, lref, spec.encode())
            what = f"hgemm_plan_override({spec!r})"
        if st != 0:
            self._h = ctypes.c_void_p()
            raise HgemmError(st, what)

    def run(self, a_ptr: int, b_ptr: int, c_ptr: int, stream: int = 0) -> None:
        st = load().hgemm_run(self._h, a_ptr, b_ptr, c_ptr, stream)
        if st != 0:
            raise HgemmError(st, "hgemm_run")

    def pointer_sets(self, sets):
        """Marshal [(a_ptr, b_ptr, c_ptr), ...] into the three host arrays hgemm_run_many takes."""
        n = len(sets)
        arr = ctypes.c_void_p * n
        return (n, arr(*[s[0] for s in sets]), arr(*[s[1] for s in sets]), arr(*[s[2] for s in sets]))

    def run_many(self, count: int, sets, stream: int = 0, first: int = 0) -> None:
        """hgemm_run_many: `count` back-to-back calls, call i on operand set (first + i) % len(sets).
        `sets` is a list of (a_ptr, b_ptr, c_ptr) or the result of pointer_sets()."""
        n, a, b, c = sets if isinstance(sets[0], int) else self.pointer_sets(sets)
        st = load().hgemm_run_many(self._h, count, n, first, a, b, c, stream)
        if st != 0:
            raise HgemmError(st, "hgemm_run_many")

    def run_status(self, a_ptr, b_ptr, c_ptr, stream: int = 0) -> int:
        return int(load().hgemm_run(self._h, a_ptr, b_ptr, c_ptr, stream))

    def describe(self) -> str:
        buf = ctypes.create_string_buffer(256)
        st = load().hgemm_plan_describe(self._h, buf, len(buf))
        if st != 0:
            raise HgemmError(st, "hgemm_plan_describe")
        return buf.value.decode()

    def workspace_bytes(self) -> int:
        return int(load().hgemm_plan_workspace_bytes(self._h))

    def launch_info(self) -> dict:
        wg, lds, th = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
        st = load().hgemm_plan_launch_info(self._h, ctypes.byref(wg), ctypes.byref(lds), ctypes.byref(th))
        if st != 0:
            raise HgemmError(st, "hgemm_plan_launch_info")
        return {"workgroups": wg.value, "lds_bytes": lds.value, "threads": th.value}

    def destroy(self) -> None:
        if self._h:
            load().hgemm_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.destroy()


def run_static(M: int, N: int, K: int, layouts: Optional[Layouts], a_ptr: int, b_ptr: int, c_ptr: int, stream: int = 0) -> None:
    """hgemm_run_static: plan and enqueue in one call that allocates nothing (static scratch workspace)."""
    st = load().hgemm_run_static(M, N, K, ctypes.byref(layouts) if layouts is not None else None, a_ptr, b_ptr, c_ptr, stream)
    if st != 0:
        raise HgemmError(st, "hgemm_run_static")


def plan(M: int, N: int, K: int, layouts: Optional[Layouts] = None, spec: Optional[str] = None) -> Plan:
    return Plan(M, N, K, layouts, spec)


def hgemm(a, b, out=None, spec: Optional[str] = None, b_col_major: bool = False):
    """Convenience wrapper for torch CUDA tensors: C = A @ B through hgemm_plan / hgemm_run.

    a: (M,K) float16, b: (K,N) float16 (or (N,K) when b_col_major), both contiguous on the GPU.
    """
    import torch

    if a.dtype != torch.float16 or b.dtype != torch.float16 or not a.is_cuda or not b.is_cuda:
        raise TypeError("hgemm needs float16 CUDA tensors")
    if not a.is_contiguous() or not b.is_contiguous():
        raise ValueError("hgemm needs contiguous tensors")
    M, K = a.shape
    N = b.shape[0] if b_col_major else b.shape[1]
    if (b.shape[1] if b_col_major else b.shape[0]) != K:
        raise ValueError("inner dimensions differ")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=a.device)
    lay = Layouts.make(b_col_major=b_col_major)
    with Plan(M, N, K, lay, spec) as p:
        p.run(a.data_ptr(), b.data_ptr(), out.data_ptr(), torch.cuda.current_stream().cuda_stream)
        if p.workspace_bytes():
            torch.cuda.current_stream().synchronize()     # the plan's workspace is freed on exit
    return out


def calibrate_mfma(iters: int = 20000, stream: int = 0):
    ms, flop = ctypes.c_double(), ctypes.c_double()
    st = load().hgemm_calibrate_mfma(iters, stream, ctypes.byref(ms), ctypes.byref(flop))
    if st != 0:
        raise HgemmError(st, "hgemm_calibrate_mfma")
    return ms.value, flop.value


def calibrate_hbm_read(ptr: int, nbytes: int, stream: int = 0) -> float:
    ms = ctypes.c_double()
    st = load().hgemm_calibrate_hbm_read(ptr, nbytes, stream, ctypes.byref(ms))
    if st != 0:
        raise HgemmError(st, "hgemm_calibrate_hbm_read")
    return ms.value

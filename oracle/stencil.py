"""ctypes front end of stencil_oracle.c (TEST INFRASTRUCTURE ONLY).

`build()` compiles the C file with gcc into oracle/_build/; `apply()` runs `iters`
out-of-place applications of one customising function over a numpy grid and returns a new
array.  Border modes and kernels are named by strings so that no constant is shared with the
GPU library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "stencil_oracle.c")
_OUT_DIR = os.path.join(_HERE, "_build")
_LIB_PATH = os.path.join(_OUT_DIR, "libstencil_oracle.so")

_BORDER = {"clamp": 0, "wrap": 1, "constant": 2}
_lib: Optional[ctypes.CDLL] = None


def build(force: bool = False) -> str:
    """Compile the oracle (plain -O2, FP contraction off, OpenMP over rows)."""
    os.makedirs(_OUT_DIR, exist_ok=True)
    stale = (not os.path.exists(_LIB_PATH)
             or os.path.getmtime(_LIB_PATH) < os.path.getmtime(_SRC))
    if force or stale:
        tmp = _LIB_PATH + ".tmp.%d" % os.getpid()
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra", _SRC, "-o", tmp, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB_PATH)
    return _LIB_PATH


def _load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, i32, f32, f64 = ctypes.c_int64, ctypes.c_int, ctypes.c_float, ctypes.c_double
        p = ctypes.c_void_p
        lib.oracle_weighted_sum_f32.argtypes = [p, p, i64, i64, i32, i32, i32, i32, i32, f32, p, i32, i32]
        lib.oracle_sincos_f32.argtypes = [p, p, i64, i64, i32, i32, i32, i32, i32, f32, p, i32, i32]
        lib.oracle_weighted_sum_f64.argtypes = [p, p, i64, i64, i32, i32, i32, i32, i32, f64, p, i32, i32]
        lib.oracle_weighted_sum_i32.argtypes = [p, p, i64, i64, i32, i32, i32, i32, i32, i32, p, i32, i32]
        lib.oracle_life_u8.argtypes = [p, p, i64, i64, i32, i32, i32, i32, i32, ctypes.c_uint8, i32, i32]
        lib.oracle_heat_f32.argtypes = [p, p, i64, i64, i32, f32, f32, i32, i32]
        lib.oracle_heat_f64.argtypes = [p, p, i64, i64, i32, f64, f64, i32, i32]
        lib.oracle_sobel_f32.argtypes = [p, p, i64, i64, i32, f32, i32, i32]
        lib.oracle_nms_f32.argtypes = [p, p, i64, i64, i32, f32, i32, i32]
        lib.oracle_threshold_f32_u8.argtypes = [p, p, i64, i64, f32, i32]
        lib.oracle_weighted_sum_u8_f32.argtypes = [p, p, i64, i64, i32, i32, i32, i32, i32, ctypes.c_uint8, p, i32]
        for fn in (lib.oracle_weighted_sum_f32, lib.oracle_sincos_f32, lib.oracle_weighted_sum_f64,
                   lib.oracle_weighted_sum_i32, lib.oracle_life_u8,
                   lib.oracle_heat_f32, lib.oracle_heat_f64, lib.oracle_sobel_f32, lib.oracle_nms_f32,
                   lib.oracle_threshold_f32_u8, lib.oracle_weighted_sum_u8_f32, lib.oracle_max_threads):
            fn.restype = i32
        _lib = lib
    return _lib


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def _ptr(a: np.ndarray) -> ctypes.c_void_p:
    return ctypes.c_void_p(a.ctypes.data)


def _check_weights(weights, halo) -> np.ndarray:
    n, s, e, w = halo
    wt = np.ascontiguousarray(np.asarray(weights, dtype=np.float32))
    if wt.shape != (n + s + 1, e + w + 1):
        raise ValueError("weights must be (N+S+1, E+W+1) = %r, got %r" % ((n + s + 1, e + w + 1), wt.shape))
    return wt


def apply(grid: np.ndarray, kernel: str, halo: Sequence[int], border: str, pad: float = 0.0,
          weights: Optional[np.ndarray] = None, scalars: Sequence[float] = (), iters: int = 1,
          threads: int = 0, precision: str = "native") -> np.ndarray:
    """`iters` applications of the stencil (Section 2) to `grid`; returns the final grid.

    kernel: "weighted_sum" (f32; also f64 and i32, and u8 in / f32 out, chosen by the grid's dtype), "life" (u8, cells 0/1), "heat" (f32; scalars=(alpha,);
    precision="f64" carries the state in float64 instead), "sincos" (f32), and the Canny detector's
    "sobel", "nms" (f32) and "threshold" (f32 in, u8 out; scalars=(level,)).
    halo = (north, south, east, west).  threads=0 leaves OpenMP's default.
    """
    lib = _load()
    if grid.ndim != 2:
        raise ValueError("grid must be 2D")
    rows, cols = grid.shape
    n, s, e, w = (int(h) for h in halo)
    b = _BORDER[border]
    if kernel == "weighted_sum" and grid.dtype == np.uint8:
        if int(iters) != 1:
            raise ValueError("a weighted sum of a byte matrix is applied once (bytes in, floats out)")
        a = np.ascontiguousarray(grid)
        wt = _check_weights(weights, (n, s, e, w))
        out = np.empty(a.shape, dtype=np.float32)
        rc = lib.oracle_weighted_sum_u8_f32(_ptr(a), _ptr(out), rows, cols, n, s, e, w, b, int(pad), _ptr(wt),
                                            int(threads))
    elif kernel == "weighted_sum" and grid.dtype in (np.float64, np.int32):
        a = np.ascontiguousarray(grid)
        wt = _check_weights(weights, (n, s, e, w))
        out = np.empty_like(a)
        if a.dtype == np.float64:
            rc = lib.oracle_weighted_sum_f64(_ptr(a), _ptr(out), rows, cols, n, s, e, w, b, float(pad), _ptr(wt),
                                             int(iters), int(threads))
        else:
            if np.any(wt != np.rint(wt)):
                raise ValueError("an int32 matrix needs integer weights")
            rc = lib.oracle_weighted_sum_i32(_ptr(a), _ptr(out), rows, cols, n, s, e, w, b, int(pad), _ptr(wt),
                                             int(iters), int(threads))
    elif kernel in ("weighted_sum", "sincos"):
        a = np.ascontiguousarray(grid, dtype=np.float32)
        wt = _check_weights(weights, (n, s, e, w))
        out = np.empty_like(a)
        fn = lib.oracle_weighted_sum_f32 if kernel == "weighted_sum" else lib.oracle_sincos_f32
        rc = fn(_ptr(a), _ptr(out), rows, cols, n, s, e, w, b, float(pad), _ptr(wt), int(iters), int(threads))
    elif kernel == "life":
        a = np.ascontiguousarray(grid, dtype=np.uint8)
        if a.max(initial=0) > 1:
            raise ValueError("life cells must be 0 or 1")
        out = np.empty_like(a)
        rc = lib.oracle_life_u8(_ptr(a), _ptr(out), rows, cols, n, s, e, w, b, int(pad), int(iters), int(threads))
    elif kernel == "heat":
        if (n, s, e, w) != (1, 1, 1, 1):
            raise ValueError("heat is the 5-point stencil: halo must be (1,1,1,1)")
        alpha = float(scalars[0])
        if precision == "f64":
            a = np.ascontiguousarray(grid, dtype=np.float64)
            out = np.empty_like(a)
            rc = lib.oracle_heat_f64(_ptr(a), _ptr(out), rows, cols, b, float(pad), alpha, int(iters), int(threads))
        else:
            a = np.ascontiguousarray(grid, dtype=np.float32)
            out = np.empty_like(a)
            rc = lib.oracle_heat_f32(_ptr(a), _ptr(out), rows, cols, b, float(pad), alpha, int(iters), int(threads))
    elif kernel in ("sobel", "nms"):
        if (n, s, e, w) != (1, 1, 1, 1):
            raise ValueError("%s has border region 1/1/1/1" % kernel)
        a = np.ascontiguousarray(grid, dtype=np.float32)
        out = np.empty_like(a)
        fn = lib.oracle_sobel_f32 if kernel == "sobel" else lib.oracle_nms_f32
        rc = fn(_ptr(a), _ptr(out), rows, cols, b, float(pad), int(iters), int(threads))
    elif kernel == "threshold":
        if (n, s, e, w) != (0, 0, 0, 0) or int(iters) != 1:
            raise ValueError("threshold has no border region and is applied once (float in, bytes out)")
        a = np.ascontiguousarray(grid, dtype=np.float32)
        out = np.empty(a.shape, dtype=np.uint8)
        rc = lib.oracle_threshold_f32_u8(_ptr(a), _ptr(out), rows, cols, float(scalars[0]), int(threads))
    else:
        raise ValueError("unknown kernel %r" % kernel)
    if rc != 0:
        raise MemoryError("oracle allocation failed")
    return out


def apply_workload(wl, grid: Optional[np.ndarray] = None, iters: Optional[int] = None,
                   threads: int = 0) -> np.ndarray:
    """Run the oracle on a workload description (any object with the fields of
    `workloads.Workload`)."""
    g = wl.grid() if grid is None else grid
    return apply(g, wl.kernel, wl.halo, wl.border, wl.pad, wl.weights, wl.scalars,
                 wl.iters if iters is None else iters, threads)

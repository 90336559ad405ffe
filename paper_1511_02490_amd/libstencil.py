"""Thin ctypes binding over the C-ABI library (include/libstencil.h).

Argument marshalling only: every step of the stencil and of the sweep runs inside
libstencil.so.  PyTorch tensors are used for device memory and streams.  Importing this
module loads the shared library and raises if it has not been built - there is no fallback.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "_lib", "libstencil.so")

OK, E_INVALID, E_REFUSED, E_RESOURCES, E_HIP = 0, -1, -2, -3, -4
F32, U8, I32, F64 = 0, 1, 2, 3
CLAMP, WRAP, CONSTANT = 0, 1, 2
WEIGHTED_SUM, LIFE, HEAT, SINCOS, SOBEL, NMS, THRESHOLD = 0, 1, 2, 3, 4, 5, 6
ENUM_POW2, ENUM_EVEN = 0, 1
STAGING_LOCAL, STAGING_DIRECT, STAGING_TEMPORAL, STAGING_STREAM = 0, 1, 2, 3
OPT_XCD_REMAP, OPT_TEMPORAL_DEPTH, OPT_SWEEP_CUTOFF, OPT_NT_STORE, OPT_FAIL_LAUNCH = 0, 1, 2, 3, 4
_STAGINGS = {"local": STAGING_LOCAL, "direct": STAGING_DIRECT, "temporal": STAGING_TEMPORAL,
             "stream": STAGING_STREAM}
N_FEATURES = 16
STATIC_MATRIX_BYTES = 16 << 20      # STENCIL_STATIC_MATRIX_BYTES

_DTYPES = {"f32": F32, "u8": U8, "i32": I32, "f64": F64}
_BORDERS = {"clamp": CLAMP, "wrap": WRAP, "constant": CONSTANT}
_KERNELS = {"weighted_sum": WEIGHTED_SUM, "life": LIFE, "heat": HEAT, "sincos": SINCOS, "sobel": SOBEL, "nms": NMS,
            "threshold": THRESHOLD}


class StencilError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__("libstencil error %d: %s" % (code, text))
        self.code = code


class Refused(StencilError):
    """The workgroup size is not legal for the scenario (Section 3.1's refused parameter)."""


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            "libstencil.so is not built (%s missing): run `python -c 'import __graft_entry__ as g; "
            "g.build()'` or `python paper_1511_02490_amd/build.py` first" % LIB_PATH)
    # PyTorch ships its own copy of the HIP runtime; it has to be the one already in the process
    # when the library is loaded, or the library would bring in a second runtime that finds no device
    try:
        import torch  # noqa: F401
    except ImportError:
        pass          # host-side functions (enumeration, legality, predictors) still work
    lib = ctypes.CDLL(LIB_PATH)
    c_int, c_i64, c_dbl, vp = ctypes.c_int, ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
    ip, dp, fp = ctypes.POINTER(c_int), ctypes.POINTER(c_dbl), ctypes.POINTER(ctypes.c_float)
    sig = {
        "stencil_create": (c_int, [ctypes.POINTER(vp), c_i64, c_i64, c_int, c_int, c_int, c_int, c_int, c_int]),
        "stencil_destroy": (None, [vp]),
        "stencil_set_kernel": (c_int, [vp, c_int, fp, c_int, fp, c_int]),
        "stencil_set_border_value": (c_int, [vp, c_dbl]),
        "stencil_set_mapping": (c_int, [vp, c_int, c_int, c_int]),
        "stencil_get_mapping": (c_int, [vp, ip, ip, ip]),
        "stencil_stream_segment_rows": (c_int, [vp, c_int, ip]),
        "stencil_set_sweep_rotation": (c_int, [vp, ctypes.POINTER(vp), ctypes.POINTER(vp), c_int]),
        "stencil_output_dtype": (c_int, [vp]),
        "stencil_set_option": (c_int, [vp, c_int, c_int]),
        "stencil_max_wg_size": (c_int, [vp]),
        "stencil_tile_bytes": (c_i64, [vp, c_int, c_int]),
        "stencil_is_legal": (c_int, [vp, c_int, c_int]),
        "stencil_enumerate_wg": (c_int, [c_int, c_int, ip, ip, c_int]),
        "stencil_run": (c_int, [vp, vp, vp, c_int, c_int, c_int, vp]),
        "stencil_run_static": (c_int, [vp, vp, vp, c_int, c_int, c_int, vp]),
        "stencil_sweep_wg": (c_int, [vp, vp, vp, c_int, ip, ip, c_int, c_int, c_int, c_int,
                                     dp, dp, dp, dp, ip, ip, dp, vp]),
        "stencil_sweep_configs": (c_int, [vp, vp, vp, c_int, vp, c_int, c_int, dp, ip, ip, vp]),
        "stencil_device_copy": (c_int, [vp, vp, c_i64, vp]),
        "stencil_time_copy": (c_int, [vp, vp, c_i64, c_int, c_int, dp, dp, vp]),
        "stencil_sweep_reduce": (c_int, [ip, ip, c_int, dp, ip, c_dbl, ip, dp, dp]),
        "stencil_baseline_wg": (c_int, [dp, c_int, c_int, ip]),
        "stencil_features": (c_int, [vp, dp]),
        "stencil_predictor_create": (c_int, [ctypes.POINTER(vp), c_int]),
        "stencil_predictor_destroy": (None, [vp]),
        "stencil_predictor_add": (c_int, [vp, dp, c_int, c_int, c_int]),
        "stencil_predictor_classify": (c_int, [vp, dp, c_int, ip, ip]),
        "stencil_predict_wg": (c_int, [vp, vp, ip, ip, c_int, c_int, c_int, c_int, ctypes.c_uint64, ip, ip]),
        "stencil_attach_predictor": (c_int, [vp, vp, c_int]),
        "stencil_default_wg": (c_int, [vp, ip, ip]),
        "stencil_predictor_load": (c_int, [ctypes.POINTER(vp), ctypes.c_char_p, c_int]),
        "stencil_regressor_create": (c_int, [ctypes.POINTER(vp)]),
        "stencil_regressor_destroy": (None, [vp]),
        "stencil_regressor_add": (c_int, [vp, dp, c_int, c_int, c_int, c_dbl]),
        "stencil_regressor_predict": (c_int, [vp, dp, c_int, c_int, c_int, dp]),
        "stencil_regressor_fit_forest": (c_int, [vp, c_int, c_int, ip, ctypes.POINTER(ctypes.c_ubyte), c_int, c_int]),
        "stencil_predict_wg_regression": (c_int, [vp, vp, ip, ip, c_int, c_int, ip, ip, ip]),
        "stencil_last_error": (ctypes.c_char_p, []),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)          # AttributeError if the library lacks a declared symbol
        fn.restype, fn.argtypes = res, args
    return lib


_lib = _load()
EXPORTS = ("stencil_create", "stencil_destroy", "stencil_set_kernel", "stencil_set_border_value",
           "stencil_set_mapping", "stencil_get_mapping", "stencil_stream_segment_rows", "stencil_set_sweep_rotation", "stencil_output_dtype", "stencil_set_option",
           "stencil_max_wg_size", "stencil_tile_bytes", "stencil_is_legal", "stencil_enumerate_wg", "stencil_run",
           "stencil_run_static",
           "stencil_sweep_wg", "stencil_sweep_configs", "stencil_device_copy", "stencil_time_copy",
           "stencil_sweep_reduce", "stencil_baseline_wg", "stencil_features", "stencil_predictor_create",
           "stencil_predictor_destroy", "stencil_predictor_add", "stencil_predictor_classify",
           "stencil_predict_wg", "stencil_attach_predictor", "stencil_default_wg", "stencil_predictor_load", "stencil_regressor_create", "stencil_regressor_destroy",
           "stencil_regressor_add", "stencil_regressor_predict", "stencil_regressor_fit_forest",
           "stencil_predict_wg_regression",
           "stencil_last_error")


def last_error() -> str:
    return _lib.stencil_last_error().decode()


def _check(rc: int) -> int:
    if rc < 0:
        raise (Refused if rc == E_REFUSED else StencilError)(rc, last_error())
    return rc


def _ints(vals: Sequence[int]):
    return (ctypes.c_int * len(vals))(*[int(v) for v in vals])


def _dbls(vals: Sequence[float]):
    return (ctypes.c_double * len(vals))(*[float(v) for v in vals])


def enumerate_wg(mode: str = "pow2", max_threads: int = 1024) -> List[Tuple[int, int]]:
    m = ENUM_POW2 if mode == "pow2" else ENUM_EVEN if mode == "even" else int(mode)
    n = _check(_lib.stencil_enumerate_wg(m, max_threads, None, None, 0))
    r, c = (ctypes.c_int * n)(), (ctypes.c_int * n)()
    _check(_lib.stencil_enumerate_wg(m, max_threads, r, c, n))
    return list(zip(r, c))


def device_copy(tin, tout, stream=None):
    """Plain copy kernel between two equally sized CUDA tensors (bandwidth reference)."""
    nbytes = tin.numel() * tin.element_size()
    assert tout.numel() * tout.element_size() == nbytes and tin.is_cuda and tout.is_cuda
    _check(_lib.stencil_device_copy(ctypes.c_void_p(tin.data_ptr()), ctypes.c_void_p(tout.data_ptr()),
                                    nbytes, Stencil._stream_ptr(stream)))
    return tout


def time_copy(tin, tout, burst: int = 10, reps: int = 30, stream=None) -> Tuple[float, float]:
    """(mean, min) milliseconds per launch of the plain copy kernel, timed like a sweep sample:
    3 warm-ups, then `reps` event-timed bursts of `burst` launches."""
    nbytes = tin.numel() * tin.element_size()
    assert tout.numel() * tout.element_size() == nbytes and tin.is_cuda and tout.is_cuda
    mean, lo = ctypes.c_double(), ctypes.c_double()
    _check(_lib.stencil_time_copy(ctypes.c_void_p(tin.data_ptr()), ctypes.c_void_p(tout.data_ptr()), nbytes,
                                  int(burst), int(reps), ctypes.byref(mean), ctypes.byref(lo),
                                  Stencil._stream_ptr(stream)))
    return mean.value, lo.value


def sweep_reduce(sizes: Sequence[Tuple[int, int]], mean_ms: Sequence[float], status: Sequence[int],
                 fixed_ms: float = float("nan")):
    n = len(sizes)
    best, sp = ctypes.c_int(-1), ctypes.c_double(float("nan"))
    perf = (ctypes.c_double * max(n, 1))()
    _check(_lib.stencil_sweep_reduce(_ints([s[0] for s in sizes]), _ints([s[1] for s in sizes]), n,
                                     _dbls(mean_ms), _ints(status), float(fixed_ms),
                                     ctypes.byref(best), perf, ctypes.byref(sp)))
    return best.value, list(perf)[:n], sp.value


def baseline_wg(performance: Sequence[Sequence[float]]) -> int:
    """Index of the best safe fixed size (Algorithm 1, Baseline) for a scenarios x sizes table of
    p(s, w) with NaN for illegal sizes; -1 if no size is legal everywhere."""
    n_s, n_w = len(performance), len(performance[0])
    flat = [float(x) for row in performance for x in row]
    best = ctypes.c_int(-1)
    _check(_lib.stencil_baseline_wg(_dbls(flat), n_s, n_w, ctypes.byref(best)))
    return best.value


class _Config(ctypes.Structure):
    _fields_ = [("staging", ctypes.c_int), ("cells_rows", ctypes.c_int), ("cells_cols", ctypes.c_int),
                ("depth", ctypes.c_int), ("xcd_remap", ctypes.c_int), ("nt_store", ctypes.c_int),
                ("wg_rows", ctypes.c_int), ("wg_cols", ctypes.c_int)]


class SweepResult:
    def __init__(self, sizes, mean_ms, min_ms, median_ms, stddev_ms, status, best_index, speedup):
        self.sizes, self.mean_ms, self.min_ms = sizes, mean_ms, min_ms
        self.median_ms, self.stddev_ms, self.status = median_ms, stddev_ms, status
        self.best_index, self.speedup_over_fixed = best_index, speedup

    @property
    def best(self) -> Optional[Tuple[int, int]]:
        return self.sizes[self.best_index] if self.best_index >= 0 else None

    @property
    def best_ms(self) -> float:
        return self.mean_ms[self.best_index] if self.best_index >= 0 else float("nan")

    def legal(self):
        return [(s, t) for s, t, st in zip(self.sizes, self.mean_ms, self.status) if st == OK]

    @property
    def worst_ms(self) -> float:
        ts = [t for _, t in self.legal()]
        return max(ts) if ts else float("nan")

    def ms_of(self, size) -> float:
        for s, t, st in zip(self.sizes, self.mean_ms, self.status):
            if tuple(s) == tuple(size) and st == OK:
                return t
        return float("nan")


class Stencil:
    """One scenario: matrix size and type, border region, border mode, customising function."""

    def __init__(self, rows: int, cols: int, dtype: str = "f32", halo: Sequence[int] = (1, 1, 1, 1),
                 border: str = "clamp", pad: float = 0.0):
        self._h = ctypes.c_void_p()
        n, s, e, w = (int(x) for x in halo)
        dt = _DTYPES[dtype] if isinstance(dtype, str) else int(dtype)
        bm = _BORDERS[border] if isinstance(border, str) else int(border)
        _check(_lib.stencil_create(ctypes.byref(self._h), int(rows), int(cols), dt, n, s, e, w, bm))
        self.rows, self.cols, self.dtype, self.halo = int(rows), int(cols), dtype, (n, s, e, w)
        if pad:
            self.set_border_value(pad)

    @classmethod
    def from_workload(cls, wl) -> "Stencil":
        st = cls(wl.rows, wl.cols, wl.dtype, wl.halo, wl.border, wl.pad)
        st.set_kernel(wl.kernel, wl.weights, wl.scalars)
        return st

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            _lib.stencil_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        if _lib is not None:          # at interpreter exit the module's globals may be gone already
            self.close()

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    # -- configuration ---------------------------------------------------------------------
    def set_kernel(self, kernel, weights=None, scalars: Sequence[float] = ()):
        kid = _KERNELS[kernel] if isinstance(kernel, str) else int(kernel)
        wbuf, nw = None, 0
        if weights is not None:
            import numpy as np
            flat = np.asarray(weights, dtype=np.float32).ravel()
            nw = int(flat.size)
            wbuf = (ctypes.c_float * nw)(*flat.tolist())
        sc = (ctypes.c_float * max(1, len(scalars)))(*[float(x) for x in scalars])
        _check(_lib.stencil_set_kernel(self._h, kid, wbuf, nw, sc, len(scalars)))

    def set_border_value(self, v: float):
        _check(_lib.stencil_set_border_value(self._h, float(v)))

    def set_mapping(self, staging="local", cells_rows: int = 1, cells_cols: int = 1):
        sg = _STAGINGS[staging] if isinstance(staging, str) else int(staging)
        _check(_lib.stencil_set_mapping(self._h, sg, int(cells_rows), int(cells_cols)))

    def set_blocking(self, cells_rows: int, cells_cols: int):
        """Register blocking under the current staging."""
        self.set_mapping(self.get_mapping()[0], cells_rows, cells_cols)

    def get_mapping(self) -> Tuple[int, int, int]:
        a, b, c = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
        _check(_lib.stencil_get_mapping(self._h, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)))
        return a.value, b.value, c.value

    def stream_segment_rows(self, wavefronts_per_simd: int) -> int:
        """Segment height at which the streaming mapping's wavefronts just fill that many slots per SIMD."""
        h = ctypes.c_int()
        _check(_lib.stencil_stream_segment_rows(self._h, int(wavefronts_per_simd), ctypes.byref(h)))
        return h.value

    def get_blocking(self) -> Tuple[int, int]:
        return self.get_mapping()[1:]

    def set_option(self, option: int, value: int):
        _check(_lib.stencil_set_option(self._h, int(option), int(value)))

    # -- legality ----------------------------------------------------------------------------
    def max_wg_size(self) -> int:
        return _check(_lib.stencil_max_wg_size(self._h))

    def tile_bytes(self, wg_rows: int, wg_cols: int) -> int:
        return _check(_lib.stencil_tile_bytes(self._h, int(wg_rows), int(wg_cols)))

    def is_legal(self, wg_rows: int, wg_cols: int) -> bool:
        return bool(_lib.stencil_is_legal(self._h, int(wg_rows), int(wg_cols)))

    def features(self) -> List[float]:
        f = (ctypes.c_double * N_FEATURES)()
        _check(_lib.stencil_features(self._h, f))
        return list(f)

    # -- execution ---------------------------------------------------------------------------
    @staticmethod
    def _stream_ptr(stream):
        if stream is None:
            import torch
            stream = torch.cuda.current_stream()
        return ctypes.c_void_p(getattr(stream, "cuda_stream", stream))

    def _check_tensors(self, tin, tout):
        import torch
        types = {"f32": torch.float32, F32: torch.float32, "u8": torch.uint8, U8: torch.uint8,
                 "i32": torch.int32, I32: torch.int32, "f64": torch.float64, F64: torch.float64}
        for t, want in ((tin, types[self.dtype]), (tout, types[self.output_dtype()])):
            if not t.is_cuda or not t.is_contiguous() or t.dtype != want or t.numel() != self.rows * self.cols:
                raise ValueError("tensors must be contiguous CUDA %s of %d x %d" % (want, self.rows, self.cols))

    def output_dtype(self) -> int:
        """Element type of the output matrix (the input's, except bytes for the threshold stencil)."""
        return _check(_lib.stencil_output_dtype(self._h))

    def run(self, tin, tout, iters: int = 1, wg: Tuple[int, int] = (0, 0), stream=None):
        self._check_tensors(tin, tout)
        _check(_lib.stencil_run(self._h, ctypes.c_void_p(tin.data_ptr()), ctypes.c_void_p(tout.data_ptr()),
                                int(iters), int(wg[0]), int(wg[1]), self._stream_ptr(stream)))
        return tout

    def run_static(self, tin, tout, iters: int = 1, wg: Tuple[int, int] = (0, 0), stream=None):
        """stencil_run out of the library's fixed device buffer (allocates nothing)."""
        self._check_tensors(tin, tout)
        _check(_lib.stencil_run_static(self._h, ctypes.c_void_p(tin.data_ptr()), ctypes.c_void_p(tout.data_ptr()),
                                       int(iters), int(wg[0]), int(wg[1]), self._stream_ptr(stream)))
        return tout

    def sweep(self, tin, tout, sizes: Sequence[Tuple[int, int]], iters: int = 1,
              fixed: Tuple[int, int] = (4, 4), reps: int = 30, stream=None) -> SweepResult:
        self._check_tensors(tin, tout)
        n = len(sizes)
        arr = lambda: (ctypes.c_double * max(n, 1))()
        mean, mn, med, sd = arr(), arr(), arr(), arr()
        status = (ctypes.c_int * max(n, 1))()
        best, sp = ctypes.c_int(-1), ctypes.c_double(float("nan"))
        _check(_lib.stencil_sweep_wg(self._h, ctypes.c_void_p(tin.data_ptr()), ctypes.c_void_p(tout.data_ptr()),
                                     int(iters), _ints([s[0] for s in sizes]), _ints([s[1] for s in sizes]), n,
                                     int(fixed[0]), int(fixed[1]), int(reps), mean, mn, med, sd, status,
                                     ctypes.byref(best), ctypes.byref(sp), self._stream_ptr(stream)))
        return SweepResult([tuple(s) for s in sizes], list(mean)[:n], list(mn)[:n], list(med)[:n],
                           list(sd)[:n], list(status)[:n], best.value, sp.value)

    def sweep_configs(self, tin, tout, configs, iters: int = 1, reps: int = 30, stream=None):
        """Sweep whole configurations: each is (staging, cells_rows, cells_cols, depth, (wg_rows,
        wg_cols)) with depth 0 = leave as is, optionally followed by the workgroup numbering and then
        the non-temporal-store switch (0 / 1 each; left as is when absent).  Returns (mean_ms list, status list, best index); the scenario is
        left on the fastest configuration."""
        self._check_tensors(tin, tout)
        n = len(configs)
        arr = (_Config * max(n, 1))()
        for k, cfg in enumerate(configs):
            staging, cr, cc, depth, wg = cfg[:5]
            remap = int(cfg[5]) if len(cfg) > 5 else -1
            nt = int(cfg[6]) if len(cfg) > 6 else -1
            sg = _STAGINGS[staging] if isinstance(staging, str) else int(staging)
            arr[k] = _Config(sg, int(cr), int(cc), int(depth), remap, nt, int(wg[0]), int(wg[1]))
        mean = (ctypes.c_double * max(n, 1))()
        status = (ctypes.c_int * max(n, 1))()
        best = ctypes.c_int(-1)
        _check(_lib.stencil_sweep_configs(self._h, ctypes.c_void_p(tin.data_ptr()), ctypes.c_void_p(tout.data_ptr()),
                                          int(iters), ctypes.cast(arr, ctypes.c_void_p), n, int(reps), mean, status,
                                          ctypes.byref(best), self._stream_ptr(stream)))
        return list(mean)[:n], list(status)[:n], best.value

    def set_sweep_rotation(self, pairs):
        """Matrix pairs [(in, out), ...] the sweeps' applications go round instead of chaining on one pair
        (an empty list clears).  The handle keeps the tensors alive."""
        pairs = list(pairs)
        for tin, tout in pairs:
            self._check_tensors(tin, tout)
        n = len(pairs)
        ins = (ctypes.c_void_p * max(n, 1))(*[t.data_ptr() for t, _ in pairs])
        outs = (ctypes.c_void_p * max(n, 1))(*[t.data_ptr() for _, t in pairs])
        _check(_lib.stencil_set_sweep_rotation(self._h, ins, outs, n))
        self._rotation = pairs

    def attach_predictor(self, predictor: Optional["Predictor"], handler: str = "nearest"):
        """The classifier run(..., wg=(0, 0)) consults when no sweep has been made (None detaches).
        The handle keeps a reference, so the predictor outlives its use."""
        h = {"nearest": 0, "baseline": 1, "random": 2}[handler]
        _check(_lib.stencil_attach_predictor(self._h, predictor._h if predictor is not None else None, h))
        self._predictor = predictor

    def default_wg(self) -> Tuple[int, int]:
        """The size run(..., wg=(0, 0)) would use now."""
        wr, wc = ctypes.c_int(), ctypes.c_int()
        _check(_lib.stencil_default_wg(self._h, ctypes.byref(wr), ctypes.byref(wc)))
        return wr.value, wc.value

    def predict_regression(self, regressor: "Regressor", candidates: Sequence[Tuple[int, int]],
                           fitness: str = "reciprocal") -> Tuple[Tuple[int, int], int]:
        """Algorithm 2: ((wg_rows, wg_cols), number of refused candidates struck on the way)."""
        wr, wc, nref = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
        fit = {"reciprocal": 0, "identity": 1}[fitness]
        _check(_lib.stencil_predict_wg_regression(self._h, regressor._h, _ints([c[0] for c in candidates]),
                                                  _ints([c[1] for c in candidates]), len(candidates), fit,
                                                  ctypes.byref(wr), ctypes.byref(wc), ctypes.byref(nref)))
        return (wr.value, wc.value), nref.value

    def predict(self, predictor: "Predictor", candidates: Sequence[Tuple[int, int]], handler: str = "nearest",
                baseline: Tuple[int, int] = (0, 0), random: int = 0) -> Tuple[int, int]:
        """Algorithm 1 with the chosen fallback handler ("nearest", "baseline" or "random")."""
        wr, wc = ctypes.c_int(), ctypes.c_int()
        h = {"nearest": 0, "baseline": 1, "random": 2}[handler]
        _check(_lib.stencil_predict_wg(self._h, predictor._h, _ints([c[0] for c in candidates]),
                                       _ints([c[1] for c in candidates]), len(candidates), h,
                                       int(baseline[0]), int(baseline[1]), int(random),
                                       ctypes.byref(wr), ctypes.byref(wc)))
        return wr.value, wc.value


class Regressor:
    """Regressor over (f(s), w, y) tuples (Sections 4.2 / 4.3): nearest neighbour, or, after
    `fit_forest`, a random forest of regression trees (Section 5)."""

    def __init__(self):
        self._h = ctypes.c_void_p()
        _check(_lib.stencil_regressor_create(ctypes.byref(self._h)))

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            _lib.stencil_regressor_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        if _lib is not None:
            self.close()

    def add(self, features: Sequence[float], wg: Tuple[int, int], value: float):
        _check(_lib.stencil_regressor_add(self._h, _dbls(features), len(features), int(wg[0]), int(wg[1]), float(value)))

    def fit_forest(self, bootstrap=None, masks=None, n_trees: Optional[int] = None, min_leaf: int = 1,
                   max_depth: int = 64):
        """bootstrap: n_trees rows of tuple indices (None: every tuple once per tree); masks: n_trees
        rows of n_features + 2 flags (None: every input open).  The draws are the caller's."""
        if n_trees is None:
            n_trees = len(bootstrap) if bootstrap is not None else len(masks) if masks is not None else 1
        b_arr, n_rows = None, 0
        if bootstrap is not None:
            assert len(bootstrap) == n_trees
            n_rows = len(bootstrap[0])
            flat = [int(i) for row in bootstrap for i in row]
            assert len(flat) == n_trees * n_rows
            b_arr = (ctypes.c_int * len(flat))(*flat)
        m_arr = None
        if masks is not None:
            assert len(masks) == n_trees
            flat = [1 if m else 0 for row in masks for m in row]
            m_arr = (ctypes.c_ubyte * len(flat))(*flat)
        _check(_lib.stencil_regressor_fit_forest(self._h, int(n_trees), int(n_rows), b_arr, m_arr, int(min_leaf),
                                                 int(max_depth)))

    def predict(self, features: Sequence[float], wg: Tuple[int, int]) -> float:
        y = ctypes.c_double()
        _check(_lib.stencil_regressor_predict(self._h, _dbls(features), len(features), int(wg[0]), int(wg[1]),
                                              ctypes.byref(y)))
        return y.value


_CLASSIFIERS = {"nearest": 0, "tree": 1, "zeror": 2}


def tuning_data_path(mapping: str = "local,1,1") -> str:
    """The training pairs recorded on an MI355X under a mapping ("local,1,1": the paper's; "local,2,4")."""
    path = os.path.join(_HERE, "tuning_data", "mi355x_%s.txt" % mapping.replace(",", "_"))
    if not os.path.exists(path):
        raise ValueError("no training data for mapping %r (have: local,1,1 and local,2,4)" % mapping)
    return path


def pretrained_predictor(mapping: str = "local,1,1", classifier: str = "tree") -> "Predictor":
    """A classifier already trained on this device (Section 4.1: training data is collected
    offline, prediction happens at run time): the (f(s), oracle size) pairs of the 128-scenario
    sweeps that autotune_study recorded on an MI355X, loaded by stencil_predictor_load.  Use with
    Stencil.predict(predictor, candidate sizes) or Stencil.attach_predictor(predictor)."""
    return Predictor.load(tuning_data_path(mapping), classifier)


class Predictor:
    """Classifier over (f(s), Omega(s)) pairs (Section 4.1): "nearest", "tree" or "zeror"."""

    def __init__(self, classifier: str = "nearest"):
        self._h = ctypes.c_void_p()
        _check(_lib.stencil_predictor_create(ctypes.byref(self._h), _CLASSIFIERS[classifier]))

    @classmethod
    def load(cls, path: str, classifier: str = "tree") -> "Predictor":
        """Training pairs from a text file (stencil_predictor_load's format)."""
        self = cls.__new__(cls)
        self._h = ctypes.c_void_p()
        _check(_lib.stencil_predictor_load(ctypes.byref(self._h), os.fsencode(path), _CLASSIFIERS[classifier]))
        return self

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            _lib.stencil_predictor_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        if _lib is not None:
            self.close()

    def add(self, features: Sequence[float], wg: Tuple[int, int]):
        _check(_lib.stencil_predictor_add(self._h, _dbls(features), len(features), int(wg[0]), int(wg[1])))

    def classify(self, features: Sequence[float]) -> Tuple[int, int]:
        wr, wc = ctypes.c_int(), ctypes.c_int()
        _check(_lib.stencil_predictor_classify(self._h, _dbls(features), len(features),
                                               ctypes.byref(wr), ctypes.byref(wc)))
        return wr.value, wc.value

"""Seeded synthetic workloads for the 2D stencil skeleton.

This module only *makes data*: grids, weight tables and workgroup-size lists that
are handed, unchanged, to whichever implementation is being run.  It holds none of
the stencil arithmetic (no border resolution, no customising function) and imports
neither the HIP binding nor the CPU oracle, so both can be fed from it without
sharing any of the method's code.

The paper (Section 5) measures synthetic stencils and four reference applications
(Gaussian blur, Game of Life, heat equation, Canny) on 512^2..4096^2 matrices of
int / float / double, and prints neither the inputs nor the customising functions.
The five workloads below stand in for them: same kinds of kernels (Table 2), same
matrix sizes (plus one 8192^2 grid that does not fit the last-level cache), values
drawn from a seeded generator.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np

BASE_SEED = 151102490

# Kernel names (strings on purpose: each side maps them to its own constants).
WEIGHTED_SUM = "weighted_sum"
LIFE = "life"
HEAT = "heat"
SINCOS = "sincos"
SOBEL = "sobel"
NMS = "nms"
THRESHOLD = "threshold"


@dataclass
class Workload:
    """One scenario: a grid, a stencil shape, a border mode and a customising function."""

    name: str
    rows: int
    cols: int
    dtype: str                      # "f32", "u8", "i32" or "f64"
    halo: Tuple[int, int, int, int]  # (north, south, east, west)
    border: str                     # "clamp" | "wrap" | "constant"
    pad: float                      # padding value for "constant"
    kernel: str
    iters: int
    seed: int
    sweep: str                      # "list" | "pow2" | "even"
    weights: np.ndarray | None = None   # (N+S+1, E+W+1) float32, row-major
    scalars: Tuple[float, ...] = ()
    sweep_list: List[Tuple[int, int]] = field(default_factory=list)

    @property
    def cells(self) -> int:
        return self.rows * self.cols

    @property
    def out_dtype(self) -> str:
        """Element type of the output matrix: the input's, except bytes for the threshold stencil
        and floats for the weighted sum of a byte image."""
        if self.kernel == THRESHOLD:
            return "u8"
        if self.kernel == WEIGHTED_SUM and self.dtype == "u8":
            return "f32"
        return self.dtype

    @property
    def bytes_per_cell_update(self) -> int:
        """One read and one write of a cell per application of the stencil."""
        size = {"f32": 4, "u8": 1, "i32": 4, "f64": 8}
        return size[self.dtype] + size[self.out_dtype]

    def grid(self) -> np.ndarray:
        return make_grid(self)

    def wg_sizes(self, max_threads: int = 1024) -> List[Tuple[int, int]]:
        if self.sweep == "list":
            return list(self.sweep_list)
        return enumerate_wg(self.sweep, max_threads)


def enumerate_wg(mode: str, max_threads: int = 1024) -> List[Tuple[int, int]]:
    """Workgroup-size lists swept per scenario (Section 5: every (w_r, w_c) up to the
    maximum workgroup size).

    "pow2": w_r, w_c powers of two, w_r*w_c <= max_threads  (66 pairs for 1024).
    "even": w_r, w_c in {2,4,..,64},  w_r*w_c <= max_threads (590 pairs for 1024).
    """
    if mode == "pow2":
        vals = []
        v = 1
        while v <= max_threads:
            vals.append(v)
            v *= 2
    elif mode == "even":
        vals = list(range(2, 65, 2))
    else:
        raise ValueError(mode)
    return [(r, c) for r in vals for c in vals if r * c <= max_threads]


def gaussian_weights(radius: int, sigma: float) -> np.ndarray:
    """(2*radius+1)^2 table: outer product of exp(-k^2 / (2 sigma^2)), k = -radius..radius,
    normalised to sum 1 in float64, then rounded once to float32.  That float32 table is
    the data both implementations receive."""
    k = np.arange(-radius, radius + 1, dtype=np.float64)
    g = np.exp(-(k * k) / (2.0 * sigma * sigma))
    w = np.outer(g, g)
    w /= w.sum()
    return np.ascontiguousarray(w.astype(np.float32))


def binomial3_weights() -> np.ndarray:
    """[1,2,1]^T [1,2,1] / 16, exact in float32."""
    b = np.array([1.0, 2.0, 1.0])
    return np.ascontiguousarray((np.outer(b, b) / 16.0).astype(np.float32))


def make_grid(w: "Workload") -> np.ndarray:
    rng = np.random.default_rng(w.seed)
    shape = (w.rows, w.cols)
    if w.kernel == LIFE:
        return np.ascontiguousarray((rng.random(shape, dtype=np.float32) < 0.3).astype(np.uint8))
    if w.kernel == HEAT:
        u = rng.random(shape, dtype=np.float32) * np.float32(100.0)
        side = min(32, w.rows, w.cols)
        n_sq = 64
        tops = rng.integers(0, w.rows - side + 1, size=n_sq)
        lefts = rng.integers(0, w.cols - side + 1, size=n_sq)
        for t, l in zip(tops, lefts):           # overlaps allowed; written after the fill
            u[t:t + side, l:l + side] = np.float32(1000.0)
        return np.ascontiguousarray(u)
    if w.kernel == SINCOS:
        return np.ascontiguousarray(rng.random(shape, dtype=np.float32) * np.float32(2.0) - np.float32(1.0))
    if w.dtype == "u8":
        return np.ascontiguousarray(rng.integers(0, 256, size=shape, dtype=np.uint8))     # an 8-bit image
    if w.dtype == "f64":
        return np.ascontiguousarray(rng.random(shape, dtype=np.float64))
    if w.dtype == "i32":
        return np.ascontiguousarray(rng.integers(-1000, 1001, size=shape, dtype=np.int32))
    return np.ascontiguousarray(rng.random(shape, dtype=np.float32))


def sincos_weights(halo: Tuple[int, int, int, int], seed: int) -> np.ndarray:
    n, s, e, w = halo
    rng = np.random.default_rng(seed)
    return np.ascontiguousarray(rng.random((n + s + 1, e + w + 1), dtype=np.float32))


def config(index: int, rows: int | None = None, cols: int | None = None,
           iters: int | None = None) -> Workload:
    """Workload C1..C5 (index 0..4).  rows/cols/iters override the full size, which is how
    the parity tests get a small grid of the same recipe."""
    seed = BASE_SEED + index
    if index == 0:
        wl = Workload("C1 gaussian3x3 256x256 f32 clamp", 256, 256, "f32", (1, 1, 1, 1), "clamp", 0.0,
                      WEIGHTED_SUM, 1, seed, "list", weights=binomial3_weights(),
                      sweep_list=[(8, 8), (16, 16), (32, 8), (64, 4), (8, 32), (4, 64)])
    elif index == 1:
        wl = Workload("C2 gaussian5x5 2048x2048 f32 clamp", 2048, 2048, "f32", (2, 2, 2, 2), "clamp", 0.0,
                      WEIGHTED_SUM, 1, seed, "pow2", weights=gaussian_weights(2, 1.0))
    elif index == 2:
        wl = Workload("C3 life 4096x4096 u8 wrap x100", 4096, 4096, "u8", (1, 1, 1, 1), "wrap", 0.0,
                      LIFE, 100, seed, "pow2")
    elif index == 3:
        wl = Workload("C4 heat 4096x4096 f32 wrap x1000", 4096, 4096, "f32", (1, 1, 1, 1), "wrap", 0.0,
                      HEAT, 1000, seed, "pow2", scalars=(0.2,))
    elif index == 4:
        halo = (1, 5, 3, 0)
        wl = Workload("C5 sincos N1S5E3W0 8192x8192 f32 const0", 8192, 8192, "f32", halo, "constant", 0.0,
                      SINCOS, 1, seed, "even", weights=sincos_weights(halo, seed + 1000))
    else:
        raise ValueError("config index must be 0..4")
    if rows is not None:
        wl.rows = rows
    if cols is not None:
        wl.cols = cols
    if iters is not None:
        wl.iters = iters
    return wl


def all_configs() -> Dict[str, Workload]:
    return {"C%d" % (i + 1): config(i) for i in range(5)}


# ---- scenario sets for the autotuning study (Section 3.3 / Section 5) -------------------------

def synthetic_scenarios(n: int, seed: int = BASE_SEED + 100) -> List[Workload]:
    """Synthetic stencils after the paper's template (Section 3.3): four shape parameters, and a
    boolean complexity - lightweight (a weighted sum) or compute-intensive (w sin x + cos x per
    region cell) - on the paper's matrix sizes.  Border extents are drawn from 0..8 (up to 30,
    Table 2's limit, on the smallest matrix only, so that one-work-item workgroups stay
    affordable); border mode and values are random."""
    rng = np.random.default_rng(seed)
    out = []
    for k in range(n):
        heavy = bool(rng.integers(0, 2))
        big = (not heavy) and rng.random() < 0.2
        if big:
            side = 512
            halo = tuple(int(h) for h in rng.integers(4, 31, size=4))
        else:
            side = int(rng.choice([512, 1024, 2048, 4096] if not heavy else [512, 1024, 2048]))
            halo = tuple(int(h) for h in rng.integers(0, 9 if not heavy else 6, size=4))
        border = str(rng.choice(["clamp", "wrap", "constant"]))
        n_, s_, e_, w_ = halo
        weights = rng.random((n_ + s_ + 1, e_ + w_ + 1), dtype=np.float32)
        if not heavy:
            weights /= weights.sum()
        name = "syn-%s-%02d %dx%d N%dS%dE%dW%d %s" % ("b" if heavy else "a", k, side, side, n_, s_, e_, w_, border)
        out.append(Workload(name, side, side, "f32", halo, border, 0.5, SINCOS if heavy else WEIGHTED_SUM, 1,
                            seed + 1 + k, "pow2", weights=np.ascontiguousarray(weights)))
    return out


def forest_draws(n_trees: int, n_tuples: int, n_inputs: int, seed: int = BASE_SEED + 200,
                 open_fraction: float = 0.7) -> Tuple[List[List[int]], List[List[bool]]]:
    """The random draws of a random forest (Section 5's regressor), made here so that whoever grows
    the forest is handed them as data: per tree a bootstrap sample of the tuple indices (n_tuples
    draws with repetition) and the subset of the inputs open to it (each with probability
    `open_fraction`; the last two inputs, the workgroup size, always)."""
    rng = np.random.default_rng(seed)
    bootstrap = rng.integers(0, n_tuples, size=(n_trees, n_tuples)).tolist()
    masks = rng.random((n_trees, n_inputs)) < open_fraction
    masks[:, n_inputs - 2:] = True
    return bootstrap, masks.tolist()


def canny_stage(kernel: str, rows: int, cols: int, border: str = "clamp", level: float = 0.5) -> Workload:
    """One stencil of the Canny edge detector (Table 2: sobel and nms with border region 1/1/1/1,
    threshold with none) on a seeded U[0,1) image."""
    halo = (0, 0, 0, 0) if kernel == THRESHOLD else (1, 1, 1, 1)
    seed = BASE_SEED + 300 + {SOBEL: 0, NMS: 1, THRESHOLD: 2}[kernel]
    return Workload("%s %dx%d" % (kernel, rows, cols), rows, cols, "f32", halo, border, 0.0, kernel, 1, seed, "pow2",
                    scalars=(level,) if kernel == THRESHOLD else ())


def image_blur(rows: int, cols: int, radius: int = 2, border: str = "clamp") -> Workload:
    """The Canny detector's first stage on an 8-bit image: Gaussian blur, bytes in, floats out."""
    side = 2 * radius + 1
    return Workload("gaussian%dx%d u8->f32 %dx%d" % (side, side, rows, cols), rows, cols, "u8", (radius,) * 4, border,
                    0.0, WEIGHTED_SUM, 1, BASE_SEED + 310 + radius, "pow2", weights=gaussian_weights(radius, 1.0))


def real_scenarios() -> List[Workload]:
    """The reference applications of Section 5 (Gaussian blur, Game of Life, heat equation, and
    the sobel / nms / threshold stencils of the Canny detector) on the paper's four matrix sizes."""
    out = []
    for side in (512, 1024, 2048, 4096):
        for radius in (1, 2):
            w = config(1 if radius == 2 else 0, rows=side, cols=side)
            w.name = "gaussian%dx%d %dx%d" % (2 * radius + 1, 2 * radius + 1, side, side)
            w.sweep = "pow2"
            out.append(w)
        g = config(2, rows=side, cols=side, iters=10)
        g.name = "gol %dx%d" % (side, side)
        out.append(g)
        h = config(3, rows=side, cols=side, iters=10)
        h.name = "he %dx%d" % (side, side)
        out.append(h)
        for kernel in (SOBEL, NMS, THRESHOLD):
            out.append(canny_stage(kernel, side, side))
    return out

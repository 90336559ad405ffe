"""Pins for the CPU oracle: each check below is something other than the oracle itself -
hand-worked fixtures, closed forms, invariants, library routines on the special cases they
cover, brute force on tiny grids.  None of these needs a GPU."""
import math

import numpy as np
import pytest
import scipy.ndimage as ndi
import torch
import torch.nn.functional as F

from oracle import stencil as oracle
from paper_1511_02490_amd import workloads as wl

from conftest import read_golden_sections

BORDERS = ("clamp", "wrap", "constant")


def rng(seed):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------------------------------
# weighted sum: orientation, borders, library cross-checks
# ---------------------------------------------------------------------------------------

def test_impulse_reveals_orientation_fig1_shape():
    """Figure 1's border region (1 south, 2 north / east / west) with distinct weights: an
    impulse at (r0,c0) must appear at out[r0-dr][c0-dc] = w[dr+N][dc+W] (correlation, north =
    smaller row, west = smaller column).  A transposed, flipped or mis-centred table fails."""
    N, S, E, W = 2, 1, 2, 2
    w = np.arange(1, (N + S + 1) * (E + W + 1) + 1, dtype=np.float32).reshape(N + S + 1, E + W + 1)
    g = np.zeros((11, 13), np.float32)
    r0, c0 = 5, 6
    g[r0, c0] = 1.0
    out = oracle.apply(g, "weighted_sum", (N, S, E, W), "constant", 0.0, w)
    expect = np.zeros_like(g)
    for dr in range(-N, S + 1):
        for dc in range(-W, E + 1):
            expect[r0 - dr, c0 - dc] = w[dr + N, dc + W]
    np.testing.assert_array_equal(out, expect)
    # the cell 2 rows *below* the impulse sees it through its *north* extent (dr = -2)
    assert out[r0 + 2, c0] == w[0, W]
    # nothing 2 rows above: south extent is only 1
    assert out[r0 - 2, c0] == 0.0


@pytest.mark.parametrize("border", BORDERS)
def test_corner_impulse_hand_worked(border):
    exp = np.array(read_golden_sections("corner_impulse_4x5.txt")[border], dtype=np.float32)
    g = np.zeros((4, 5), np.float32)
    g[0, 0] = 1.0
    w = np.arange(1, 10, dtype=np.float32).reshape(3, 3)
    out = oracle.apply(g, "weighted_sum", (1, 1, 1, 1), border, 0.0, w)
    np.testing.assert_array_equal(out, exp)


def _torch_correlate(g, w, halo, border, pad):
    """Library route for any rectangular region: torch's own padding modes (constant /
    replicate / circular) followed by a valid cross-correlation, in float64."""
    N, S, E, W = halo
    x = torch.from_numpy(g.astype(np.float64))[None, None]
    if border == "constant":
        xp = F.pad(x, (W, E, N, S), mode="constant", value=float(pad))
    else:
        xp = F.pad(x, (W, E, N, S), mode="replicate" if border == "clamp" else "circular")
    k = torch.from_numpy(w.astype(np.float64))[None, None]
    return F.conv2d(xp, k)[0, 0].numpy()


@pytest.mark.parametrize("border", BORDERS)
@pytest.mark.parametrize("halo", [(1, 1, 1, 1), (2, 2, 2, 2), (2, 1, 2, 2), (1, 5, 3, 0), (0, 0, 0, 0),
                                  (0, 3, 0, 0), (0, 0, 4, 1)])
def test_weighted_sum_matches_library_correlation(border, halo):
    N, S, E, W = halo
    r = rng(1234 + N * 1000 + S * 100 + E * 10 + W)
    g = r.random((19, 23), dtype=np.float32) - np.float32(0.3)
    w = r.random((N + S + 1, E + W + 1), dtype=np.float32)
    pad = 0.75
    out = oracle.apply(g, "weighted_sum", halo, border, pad, w)
    ref = _torch_correlate(g, w, halo, border, pad)
    np.testing.assert_allclose(out, ref.astype(np.float32), rtol=2e-7, atol=1e-7)


@pytest.mark.parametrize("border,mode", [("clamp", "nearest"), ("wrap", "grid-wrap"), ("constant", "constant")])
def test_weighted_sum_matches_scipy_symmetric(border, mode):
    r = rng(77)
    g = r.random((33, 29), dtype=np.float32)
    w = wl.gaussian_weights(2, 1.0)
    out = oracle.apply(g, "weighted_sum", (2, 2, 2, 2), border, 0.5, w)
    ref = ndi.correlate(g.astype(np.float64), w.astype(np.float64), mode=mode, cval=0.5)
    np.testing.assert_allclose(out, ref.astype(np.float32), rtol=2e-7, atol=0)


def test_halo_larger_than_matrix():
    """Wrap is a true modulo and clamp saturates even when the border region is larger than
    the matrix (torch's padding modes stop at the matrix extent, so pad by index here)."""
    g = rng(5).random((3, 4), dtype=np.float32)
    halo = (5, 4, 6, 7)
    w = rng(6).random((10, 14), dtype=np.float32)
    ri, ci = np.arange(-5, 3 + 4), np.arange(-7, 4 + 6)
    for border in BORDERS:
        out = oracle.apply(g, "weighted_sum", halo, border, 0.25, w)
        g64 = g.astype(np.float64)
        if border == "clamp":
            xp = g64[np.clip(ri, 0, 2)][:, np.clip(ci, 0, 3)]
        elif border == "wrap":
            xp = g64[np.mod(ri, 3)][:, np.mod(ci, 4)]
        else:
            xp = np.pad(g64, ((5, 4), (7, 6)), constant_values=0.25)
        ref = F.conv2d(torch.from_numpy(xp)[None, None],
                       torch.from_numpy(w.astype(np.float64))[None, None])[0, 0].numpy()
        np.testing.assert_allclose(out, ref.astype(np.float32), rtol=2e-7)


@pytest.mark.parametrize("border", ("clamp", "wrap"))
def test_normalised_kernel_keeps_constant_field(border):
    g = np.full((40, 37), 1.0, np.float32)
    out = oracle.apply(g, "weighted_sum", (1, 1, 1, 1), border, 0.0, wl.binomial3_weights())
    np.testing.assert_array_equal(out, g)                      # dyadic weights: exact
    g5 = np.full((40, 37), 3.25, np.float32)
    out5 = oracle.apply(g5, "weighted_sum", (2, 2, 2, 2), border, 0.0, wl.gaussian_weights(2, 1.0))
    np.testing.assert_allclose(out5, g5, rtol=3e-7)


def test_symmetric_kernel_reproduces_linear_ramp_in_interior():
    rows, cols = 24, 31
    rr, cc = np.meshgrid(np.arange(rows), np.arange(cols), indexing="ij")
    g = (0.5 * rr - 0.25 * cc + 3.0).astype(np.float32)        # exactly representable
    out = oracle.apply(g, "weighted_sum", (2, 2, 2, 2), "clamp", 0.0, wl.gaussian_weights(2, 1.0))
    np.testing.assert_allclose(out[2:-2, 2:-2], g[2:-2, 2:-2], rtol=1e-6)
    # a one-sided region shifts the ramp by its centre of mass instead
    w = np.full((1, 3), 1.0 / 3.0, np.float32)
    out2 = oracle.apply(g, "weighted_sum", (0, 0, 2, 0), "clamp", 0.0, w)   # cells c, c+1, c+2
    np.testing.assert_allclose(out2[:, :-2], g[:, :-2] - 0.25, rtol=1e-6)


def test_weight_tables_of_the_workloads():
    w3 = wl.binomial3_weights()
    assert w3.dtype == np.float32 and w3.shape == (3, 3)
    np.testing.assert_array_equal(w3 * 16, np.array([[1, 2, 1], [2, 4, 2], [1, 2, 1]], np.float32))
    w5 = wl.gaussian_weights(2, 1.0).astype(np.float64)
    assert abs(w5.sum() - 1.0) < 1e-7
    np.testing.assert_allclose(w5, w5.T, rtol=0)
    np.testing.assert_allclose(w5, w5[::-1, ::-1], rtol=0)
    # sigma = 1: neighbouring taps differ by exp(-1/2) and exp(-3/2)
    assert abs(w5[2, 1] / w5[2, 2] - math.exp(-0.5)) < 1e-6
    assert abs(w5[2, 0] / w5[2, 1] - math.exp(-1.5)) < 1e-6
    assert abs(w5[0, 0] / w5[2, 2] - math.exp(-4.0)) < 1e-6


def test_weighted_sum_on_double_and_int32_matrices():
    """The other element types of the paper's template.  double: against torch's float64
    correlation; int32: exact integers, reduced modulo 2^32 (checked with Python integers)."""
    r = rng(31)
    halo = (2, 1, 2, 2)
    g = r.random((17, 21))
    w = r.random((4, 5), dtype=np.float32)
    for border in BORDERS:
        out = oracle.apply(g, "weighted_sum", halo, border, 0.75, w)
        assert out.dtype == np.float64
        ref = _torch_correlate(g, w, halo, border, 0.75)
        np.testing.assert_allclose(out, ref, rtol=1e-14, atol=1e-15)
    # an impulse keeps all 53 bits: out = w * x exactly when w is a power of two
    gi = np.zeros((5, 5)); gi[2, 2] = 1.0 / 3.0
    oi = oracle.apply(gi, "weighted_sum", (1, 1, 1, 1), "constant", 0.0, np.full((3, 3), 0.25, np.float32))
    assert oi[1, 1] == (1.0 / 3.0) * 0.25
    gi32 = r.integers(-50, 51, size=(9, 11), dtype=np.int32)
    wi = r.integers(-4, 5, size=(4, 5)).astype(np.float32)
    for border in BORDERS:
        out = oracle.apply(gi32, "weighted_sum", halo, border, 7, wi)
        assert out.dtype == np.int32
        ref = _torch_correlate(gi32.astype(np.float64), wi, halo, border, 7.0)
        np.testing.assert_array_equal(out, np.rint(ref).astype(np.int32))
    # wrap-around: 2^20 * 2^20 * 9 = 9 * 2^40 = 0 (mod 2^32); (2^20 + 1)^2 * 9 leaves 9 * (2^21 + 1)
    big = np.full((3, 3), 1 << 20, np.int32)
    wb = np.full((3, 3), float(1 << 20), np.float32)
    assert oracle.apply(big, "weighted_sum", (1, 1, 1, 1), "wrap", 0, wb)[1, 1] == 0
    big1 = np.full((3, 3), (1 << 20) + 1, np.int32)
    wb1 = np.full((3, 3), float((1 << 20) + 1), np.float32)
    want = (9 * ((1 << 20) + 1) ** 2) % (1 << 32)
    want = want - (1 << 32) if want >= (1 << 31) else want
    assert int(oracle.apply(big1, "weighted_sum", (1, 1, 1, 1), "wrap", 0, wb1)[1, 1]) == want
    with pytest.raises(ValueError):
        oracle.apply(gi32, "weighted_sum", halo, "clamp", 0, wi + 0.5)


def test_weighted_sum_of_a_byte_matrix_into_floats():
    """Bytes in, floats out (the kernel whose input and output types differ): torch's float64
    correlation of the same integers for every border mode; an impulse of 255 under distinct
    weights by hand (orientation, and no wrap-around at the top of the byte range); a byte padding
    value; integer weights give exact integers; one application only."""
    r = rng(77)
    halo = (2, 1, 2, 2)
    g = r.integers(0, 256, size=(17, 21), dtype=np.uint8)
    w = r.random((4, 5), dtype=np.float32)
    for border in BORDERS:
        out = oracle.apply(g, "weighted_sum", halo, border, 200, w)
        assert out.dtype == np.float32 and out.shape == g.shape
        ref = _torch_correlate(g.astype(np.float64), w, halo, border, 200.0)
        np.testing.assert_array_equal(out, ref.astype(np.float32))     # fp64 sums of <= 20 products, rounded once
    N, S, E, W = halo
    wd = np.arange(1, 21, dtype=np.float32).reshape(4, 5)
    gi = np.zeros((9, 9), np.uint8)
    gi[4, 4] = 255
    oi = oracle.apply(gi, "weighted_sum", halo, "constant", 0, wd)
    expect = np.zeros((9, 9), np.float32)
    for dr in range(-N, S + 1):
        for dc in range(-W, E + 1):
            expect[4 - dr, 4 - dc] = 255.0 * wd[dr + N, dc + W]
    np.testing.assert_array_equal(oi, expect)
    # all-255 image, weights 1: every cell 20 * 255 (a byte sum would have wrapped)
    full = np.full((6, 7), 255, np.uint8)
    np.testing.assert_array_equal(oracle.apply(full, "weighted_sum", halo, "clamp", 0, np.ones((4, 5), np.float32)),
                                  np.full((6, 7), 5100.0, np.float32))
    # the padding value is a byte: a 1x1 matrix of 10 with pad 3 under a 3x3 box sums to 10 + 8 * 3
    one = np.array([[10]], np.uint8)
    assert oracle.apply(one, "weighted_sum", (1, 1, 1, 1), "constant", 3, np.ones((3, 3), np.float32))[0, 0] == 34.0
    with pytest.raises(ValueError):
        oracle.apply(g, "weighted_sum", halo, "clamp", 0, w, iters=2)


def test_iterations_compose():
    g = rng(9).random((12, 15), dtype=np.float32)
    w = wl.binomial3_weights()
    a = oracle.apply(g, "weighted_sum", (1, 1, 1, 1), "wrap", 0.0, w, iters=3)
    b = g
    for _ in range(3):
        b = oracle.apply(b, "weighted_sum", (1, 1, 1, 1), "wrap", 0.0, w, iters=1)
    np.testing.assert_array_equal(a, b)
    np.testing.assert_array_equal(oracle.apply(g, "weighted_sum", (1, 1, 1, 1), "wrap", 0.0, w, iters=0), g)


def test_thread_count_does_not_change_values():
    g = rng(10).random((64, 50), dtype=np.float32)
    w = wl.gaussian_weights(2, 1.0)
    a = oracle.apply(g, "weighted_sum", (2, 2, 2, 2), "clamp", 0.0, w, threads=1)
    b = oracle.apply(g, "weighted_sum", (2, 2, 2, 2), "clamp", 0.0, w, threads=4)
    np.testing.assert_array_equal(a, b)


# ---------------------------------------------------------------------------------------
# Game of Life
# ---------------------------------------------------------------------------------------

def _pattern(sections, name):
    return np.array([[1 if ch == "O" else 0 for ch in row[0]] for row in sections[name]], np.uint8)


def _embed(pat, shape, top, left):
    g = np.zeros(shape, np.uint8)
    idx_r = (np.arange(pat.shape[0]) + top) % shape[0]
    idx_c = (np.arange(pat.shape[1]) + left) % shape[1]
    g[np.ix_(idx_r, idx_c)] = pat
    return g


def _life_roll(g):
    """Independent torus step: neighbour count by eight whole-array rotations."""
    n = sum(np.roll(np.roll(g.astype(np.int32), dr, 0), dc, 1)
            for dr in (-1, 0, 1) for dc in (-1, 0, 1) if (dr, dc) != (0, 0))
    return ((n == 3) | ((g == 1) & (n == 2))).astype(np.uint8)


def life(g, iters=1, border="wrap"):
    return oracle.apply(g, "life", (1, 1, 1, 1), border, 0, iters=iters)


def test_life_glider_phases_and_translation():
    sec = read_golden_sections("life_glider.txt")
    shape = (9, 11)
    for k in range(5):
        start = _embed(_pattern(sec, "glider_gen0"), shape, 2, 3)
        expect = _embed(_pattern(sec, "glider_gen%d" % k), shape, 2, 3)
        np.testing.assert_array_equal(life(start, k), expect)
    # 4 generations = one cell south-east; 4*9*11 generations on the 9x11 torus come home
    g0 = _embed(_pattern(sec, "glider_gen0"), shape, 2, 3)
    np.testing.assert_array_equal(life(g0, 4), np.roll(np.roll(g0, 1, 0), 1, 1))
    np.testing.assert_array_equal(life(g0, 4 * 99), g0)


def test_life_glider_crosses_the_wrap_edge():
    sec = read_golden_sections("life_glider.txt")
    shape = (8, 8)
    g0 = _embed(_pattern(sec, "glider_gen0"), shape, 5, 5)      # straddles bottom/right edges soon
    g = g0
    for step in range(1, 33):
        g = life(g, 1)
        assert int(g.sum()) == 5
        if step % 4 == 0:
            np.testing.assert_array_equal(g, np.roll(np.roll(g0, step // 4, 0), step // 4, 1))
    np.testing.assert_array_equal(g, g0)                         # 32 generations: 8 cells each way


def test_life_blinker_block_and_empty():
    sec = read_golden_sections("life_glider.txt")
    b0 = _embed(_pattern(sec, "blinker_gen0"), (7, 6), 1, 0)
    b1 = _embed(_pattern(sec, "blinker_gen1"), (7, 6), 1, 0)
    np.testing.assert_array_equal(life(b0, 1), b1)
    np.testing.assert_array_equal(life(b0, 2), b0)
    block = np.zeros((6, 6), np.uint8)
    block[2:4, 2:4] = 1
    np.testing.assert_array_equal(life(block, 5), block)
    dead = np.zeros((5, 9), np.uint8)
    np.testing.assert_array_equal(life(dead, 3), dead)


@pytest.mark.parametrize("shape", [(3, 3), (4, 6), (6, 5), (1, 7), (2, 2)])
def test_life_brute_force_tiny_tori(shape):
    r = rng(shape[0] * 10 + shape[1])
    for _ in range(20):
        g = (r.random(shape) < 0.4).astype(np.uint8)
        np.testing.assert_array_equal(life(g, 1), _life_roll(g))


def test_life_random_torus_many_steps():
    g = (rng(3).random((37, 41)) < 0.3).astype(np.uint8)
    ref = g
    for _ in range(25):
        ref = _life_roll(ref)
    np.testing.assert_array_equal(life(g, 25), ref)


@pytest.mark.parametrize("border", ("clamp", "constant"))
def test_life_non_periodic_borders(border):
    g = (rng(4).random((9, 8)) < 0.5).astype(np.uint8)
    gp = np.pad(g.astype(np.int32), 1, mode="edge" if border == "clamp" else "constant")
    n = sum(gp[1 + dr:1 + dr + 9, 1 + dc:1 + dc + 8] for dr in (-1, 0, 1) for dc in (-1, 0, 1)
            if (dr, dc) != (0, 0))
    ref = ((n == 3) | ((g == 1) & (n == 2))).astype(np.uint8)
    np.testing.assert_array_equal(life(g, 1, border), ref)


def test_life_rejects_non_binary_cells():
    with pytest.raises(ValueError):
        life(np.full((3, 3), 2, np.uint8))


# ---------------------------------------------------------------------------------------
# heat equation
# ---------------------------------------------------------------------------------------

def heat(g, iters, border="wrap", alpha=0.2, precision="native"):
    return oracle.apply(g, "heat", (1, 1, 1, 1), border, 0.0, scalars=(alpha,), iters=iters,
                        precision=precision)


def test_heat_conserves_total_under_wrap():
    w = wl.config(3, rows=96, cols=80)
    g = w.grid()
    out64 = heat(g, 200, precision="f64")
    s0 = g.astype(np.float64).sum()
    assert abs(out64.sum() - s0) / s0 < 1e-12
    out32 = heat(g, 200)
    assert abs(out32.astype(np.float64).sum() - s0) / s0 < 1e-6


def test_heat_eigenfunction_decay_closed_form():
    """cos(2 pi k r / rows) is an eigenfunction of the periodic 5-point step with eigenvalue
    1 + 2 alpha (cos(2 pi k / rows) - 1): checks the coefficient, the sign of the Laplacian and
    the iteration count at once."""
    rows, cols, k, alpha, n = 64, 48, 3, 0.2, 37
    r = np.arange(rows)[:, None] * np.ones((1, cols))
    mode_r = np.cos(2 * np.pi * k * r / rows)
    lam = 1.0 + 2.0 * alpha * (math.cos(2 * math.pi * k / rows) - 1.0)
    out = heat(mode_r, n, precision="f64")
    np.testing.assert_allclose(out, (lam ** n) * mode_r, atol=1e-12)
    c = np.ones((rows, 1)) * np.arange(cols)[None, :]
    mode_c = np.sin(2 * np.pi * 5 * c / cols)
    lam_c = 1.0 + 2.0 * alpha * (math.cos(2 * math.pi * 5 / cols) - 1.0)
    np.testing.assert_allclose(heat(mode_c, n, precision="f64"), (lam_c ** n) * mode_c, atol=1e-12)
    # both directions at once: the eigenvalue offsets add
    both = mode_r * np.cos(2 * np.pi * 5 * c / cols)
    lam_b = 1.0 + 2.0 * alpha * ((math.cos(2 * math.pi * k / rows) - 1.0) + (math.cos(2 * math.pi * 5 / cols) - 1.0))
    np.testing.assert_allclose(heat(both, n, precision="f64"), (lam_b ** n) * both, atol=1e-12)
    # the fp32 path follows the same closed form to fp32 accuracy
    out32 = heat(mode_r.astype(np.float32), n)
    np.testing.assert_allclose(out32, ((lam ** n) * mode_r).astype(np.float32), atol=5e-6)


def test_heat_constant_is_fixed_point_and_max_principle():
    g = np.full((17, 19), 42.5, np.float32)
    for border in ("wrap", "clamp"):
        np.testing.assert_array_equal(heat(g, 10, border), g)
    h = wl.config(3, rows=160, cols=160).grid()
    out = heat(h, 50)
    assert out.min() >= h.min() and out.max() <= h.max()
    assert out.min() > h.min() + 1.0                 # the coldest cell must warm up


def test_heat_single_step_by_hand():
    g = np.zeros((4, 4), np.float32)
    g[1, 2] = 10.0
    out = heat(g, 1, "constant")
    exp = np.zeros_like(g)
    exp[1, 2] = 10.0 + 0.2 * (-40.0)
    for (r, c) in ((0, 2), (2, 2), (1, 1), (1, 3)):
        exp[r, c] = 2.0
    np.testing.assert_allclose(out, exp, rtol=1e-6)
    # wrap: an impulse in the corner reaches the opposite edges
    g2 = np.zeros((4, 5), np.float32)
    g2[0, 0] = 5.0
    out2 = heat(g2, 1, "wrap")
    assert out2[3, 0] == out2[1, 0] == out2[0, 4] == out2[0, 1] == np.float32(1.0)
    assert out2[0, 0] == np.float32(5.0 + 0.2 * -20.0)
    # clamp: the corner's missing neighbours are itself
    out3 = heat(g2, 1, "clamp")
    assert out3[0, 0] == np.float32(5.0 + np.float32(0.2) * np.float32(10.0 - 20.0))


def test_heat_fp32_path_rounds_every_operation():
    """The parity reference is strict fp32 in a fixed order: reproduce one step with numpy
    float32 scalars (each numpy op rounds to fp32) on a wrap grid."""
    g = wl.config(3, rows=16, cols=12).grid()
    n_, s_ = np.roll(g, 1, 0), np.roll(g, -1, 0)
    w_, e_ = np.roll(g, 1, 1), np.roll(g, -1, 1)
    t = ((n_ + s_) + (e_ + w_)) - np.float32(4.0) * g
    exp = g + np.float32(0.2) * t
    assert exp.dtype == np.float32
    np.testing.assert_array_equal(heat(g, 1), exp)


def test_heat_fp32_tracks_fp64():
    g = wl.config(3, rows=48, cols=48).grid()
    a = heat(g, 300).astype(np.float64)
    b = heat(g, 300, precision="f64")
    assert np.max(np.abs(a - b) / np.abs(b)) < 1e-5


# ---------------------------------------------------------------------------------------
# synthetic sin/cos stencil
# ---------------------------------------------------------------------------------------

C5_HALO = (1, 5, 3, 0)


def test_sincos_zero_field_counts_the_region():
    """x = 0 everywhere and pad 0: every term is w*0 + 1, so each cell equals the number of
    cells in its region, 7 * 4 = 28, including cells whose region hangs over the edge."""
    w = wl.sincos_weights(C5_HALO, 1)
    out = oracle.apply(np.zeros((9, 10), np.float32), "sincos", C5_HALO, "constant", 0.0, w)
    np.testing.assert_array_equal(out, np.full((9, 10), 28.0, np.float32))


def test_sincos_impulse_closed_form():
    """One cell at pi/2 (sin = 1, cos = 0) in a zero field: the cells that see it through
    offset (dr, dc) read 27 + w[dr+N][dc+W]; all others read 28."""
    N, S, E, W = C5_HALO
    w = wl.sincos_weights(C5_HALO, 2)
    g = np.zeros((16, 14), np.float32)
    r0, c0 = 8, 7
    g[r0, c0] = np.float32(np.pi / 2)
    out = oracle.apply(g, "sincos", C5_HALO, "constant", 0.0, w)
    x = float(np.float32(np.pi / 2))
    exp = np.full(g.shape, 28.0)
    for dr in range(-N, S + 1):
        for dc in range(-W, E + 1):
            exp[r0 - dr, c0 - dc] = 27.0 + w[dr + N, dc + W] * math.sin(x) + math.cos(x)
    np.testing.assert_allclose(out, exp.astype(np.float32), rtol=1e-7)
    assert out[r0 + 1, c0] != 28.0 and out[r0 - 5, c0 - 3] != 28.0      # N = 1 and S = 5, E = 3
    assert out[r0 + 2, c0] == 28.0 and out[r0, c0 + 1] == 28.0          # W = 0


@pytest.mark.parametrize("border", BORDERS)
def test_sincos_matches_library_route(border):
    """sum(w sin x + cos x) = correlate(sin x, w) + correlate(cos x, ones): two library
    correlations of elementwise-transformed fields (padding applied to x first)."""
    N, S, E, W = C5_HALO
    r = rng(21)
    g = (r.random((20, 17), dtype=np.float32) * 2 - 1).astype(np.float32)
    w = wl.sincos_weights(C5_HALO, 3)
    pad = 0.4
    out = oracle.apply(g, "sincos", C5_HALO, border, pad, w)
    rows, cols = g.shape
    ri, ci = np.arange(-N, rows + S), np.arange(-W, cols + E)
    if border == "clamp":
        xp = g[np.clip(ri, 0, rows - 1)][:, np.clip(ci, 0, cols - 1)]
    elif border == "wrap":
        xp = g[ri % rows][:, ci % cols]
    else:
        xp = np.pad(g, ((N, S), (W, E)), constant_values=np.float32(pad))
    xs = torch.from_numpy(np.sin(xp.astype(np.float64)))[None, None]
    xc = torch.from_numpy(np.cos(xp.astype(np.float64)))[None, None]
    k = torch.from_numpy(w.astype(np.float64))[None, None]
    ref = (F.conv2d(xs, k) + F.conv2d(xc, torch.ones_like(k)))[0, 0].numpy()
    np.testing.assert_allclose(out, ref.astype(np.float32), rtol=2e-7)


def test_sincos_pad_is_substituted_before_the_function():
    w = np.full((1, 2), 0.5, np.float32)          # region: the cell and its east neighbour
    g = np.zeros((1, 3), np.float32)
    out = oracle.apply(g, "sincos", (0, 0, 1, 0), "constant", float(np.float32(np.pi / 2)), w)
    x = float(np.float32(np.pi / 2))
    last = (0.5 * 0 + 1.0) + (0.5 * math.sin(x) + math.cos(x))
    np.testing.assert_allclose(out, np.array([[2.0, 2.0, last]], np.float32), rtol=1e-7)


# ---------------------------------------------------------------------------------------
# workload recipes
# ---------------------------------------------------------------------------------------

def test_workload_recipes():
    c = wl.all_configs()
    assert [(w.rows, w.cols) for w in c.values()] == [(256, 256), (2048, 2048), (4096, 4096),
                                                      (4096, 4096), (8192, 8192)]
    assert len(c["C2"].wg_sizes()) == 66 and len(c["C5"].wg_sizes()) == 590
    g1 = wl.config(0).grid()
    assert g1.dtype == np.float32 and 0.0 <= g1.min() and g1.max() < 1.0
    np.testing.assert_array_equal(g1, wl.config(0).grid())       # seeded
    g3 = wl.config(2, rows=512, cols=512).grid()
    assert g3.dtype == np.uint8 and set(np.unique(g3)) == {0, 1} and abs(g3.mean() - 0.3) < 0.01
    g4 = wl.config(3, rows=512, cols=512).grid()
    assert g4.max() == 1000.0 and (g4 == 1000.0).sum() >= 32 * 32 and g4.min() >= 0.0
    g5 = wl.config(4, rows=256, cols=256).grid()
    assert -1.0 <= g5.min() and g5.max() < 1.0 and abs(g5.mean()) < 0.02
    assert wl.config(4).weights.shape == (7, 4)


# ---- the Canny detector's stencils (Table 2: sobel, nms, threshold) ---------------------------

_NP_MODE = {"clamp": "edge", "wrap": "wrap", "constant": "constant"}
_NDI_MODE = {"clamp": "nearest", "wrap": "wrap", "constant": "constant"}


def test_sobel_closed_forms():
    """The Sobel operator answers a ramp a*c + b*r with (8a, 8b), so the magnitude is
    8*sqrt(a^2 + b^2) in the interior; a constant field has no gradient anywhere under clamp."""
    r, c = np.meshgrid(np.arange(9), np.arange(11), indexing="ij")
    for a, b in [(1.0, 0.0), (0.0, 1.0), (3.0, 4.0), (-2.0, 0.5)]:
        g = (a * c + b * r).astype(np.float32)
        out = oracle.apply(g, "sobel", (1, 1, 1, 1), "clamp")
        np.testing.assert_allclose(out[1:-1, 1:-1], 8.0 * math.hypot(a, b), rtol=1e-6)
    assert np.all(oracle.apply(np.full((5, 6), 7.5, np.float32), "sobel", (1, 1, 1, 1), "clamp") == 0.0)
    # orientation by hand: one bright cell; its west neighbour sees it to the east (gx = 2), the
    # cell north-west of it sees it to the south-east (gx = gy = 1)
    g = np.zeros((5, 5), np.float32)
    g[2, 2] = 1.0
    out = oracle.apply(g, "sobel", (1, 1, 1, 1), "constant")
    assert out[2, 1] == 2.0 and out[2, 3] == 2.0 and out[1, 2] == 2.0 and out[2, 2] == 0.0
    assert out[1, 1] == np.float32(math.sqrt(2.0)) and out[0, 0] == 0.0


@pytest.mark.parametrize("border", ["clamp", "wrap", "constant"])
def test_sobel_matches_library_operator(border):
    g = wl.config(0, rows=23, cols=31).grid() * np.float32(10.0)
    out = oracle.apply(g, "sobel", (1, 1, 1, 1), border, pad=2.5)
    g64 = g.astype(np.float64)
    kx = np.array([[-1.0, 0.0, 1.0], [-2.0, 0.0, 2.0], [-1.0, 0.0, 1.0]])
    gx = ndi.correlate(g64, kx, mode=_NDI_MODE[border], cval=2.5)
    gy = ndi.correlate(g64, kx.T, mode=_NDI_MODE[border], cval=2.5)
    np.testing.assert_allclose(out, np.hypot(gx, gy), rtol=2e-6, atol=2e-5)
    if border != "constant":      # the library's own (separable) Sobel filter pads its passes one by one
        np.testing.assert_allclose(np.hypot(ndi.sobel(g64, axis=1, mode=_NDI_MODE[border]),
                                            ndi.sobel(g64, axis=0, mode=_NDI_MODE[border])), np.hypot(gx, gy), rtol=1e-12)


@pytest.mark.parametrize("border", ["clamp", "wrap", "constant"])
def test_nms_by_hand_and_by_shifted_arrays(border):
    # by hand: a ridge along a row survives (maximal north-south), its flanks do not
    g = np.array([[1, 1, 1, 1], [5, 6, 5, 6], [2, 4, 2, 3], [0, 3, 0, 0]], np.float32)
    out = oracle.apply(g, "nms", (1, 1, 1, 1), "constant")            # padding 0 around the matrix
    np.testing.assert_array_equal(out[0], g[0])                       # a row of equals: none smaller than west / east
    np.testing.assert_array_equal(out[1], g[1])                       # every ridge cell tops its column neighbours
    np.testing.assert_array_equal(out[2], [0, 4, 0, 3])               # below the ridge only west-east maxima survive
    np.testing.assert_array_equal(out[3], [0, 3, 0, 0])
    # whole arrays at once: neighbours as padded, shifted copies
    x = wl.config(0, rows=17, cols=29).grid()
    p = np.pad(x, 1, mode=_NP_MODE[border], **({"constant_values": 0.25} if border == "constant" else {}))
    u, n, s, w, e = p[1:-1, 1:-1], p[:-2, 1:-1], p[2:, 1:-1], p[1:-1, :-2], p[1:-1, 2:]
    expect = np.where(((u >= w) & (u >= e)) | ((u >= n) & (u >= s)), u, np.float32(0.0))
    np.testing.assert_array_equal(oracle.apply(x, "nms", (1, 1, 1, 1), border, pad=0.25), expect)
    # a strict minimum of its four neighbours never survives; survivors keep their value
    out = oracle.apply(x, "nms", (1, 1, 1, 1), "wrap")
    assert set(np.unique(out[out != x])) <= {0.0}


def test_threshold_bytes_out():
    x = np.array([[0.1, 0.5, 0.49999997], [np.nan, np.inf, -1.0]], np.float32)
    out = oracle.apply(x, "threshold", (0, 0, 0, 0), "clamp", scalars=(0.5,))
    assert out.dtype == np.uint8
    np.testing.assert_array_equal(out, [[0, 1, 0], [0, 1, 0]])
    g = wl.config(0, rows=40, cols=33).grid()
    np.testing.assert_array_equal(oracle.apply(g, "threshold", (0, 0, 0, 0), "wrap", scalars=(0.3,)),
                                  (g >= np.float32(0.3)).astype(np.uint8))
    with pytest.raises(ValueError):
        oracle.apply(g, "threshold", (0, 0, 0, 0), "wrap", scalars=(0.3,), iters=2)

"""Host-side logic of the C-ABI library, checked without a GPU: the library loads and exports
every declared symbol; enumeration, legality (Eq. 1), sweep reductions (Eq. 3, Section 7) and
prediction (Algorithm 1) agree with the oracle's definitions and with hand-worked cases."""
import math
import os
import re

import numpy as np
import pytest

from oracle import tuning
from paper_1511_02490_amd import libstencil as ls
from paper_1511_02490_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "libstencil.h")).read()
    declared = set(re.findall(r"\b(stencil_[a-z_]+)\s*\(", header))
    declared -= {"stencil_t", "stencil_predictor_t"}
    assert declared == set(ls.EXPORTS)
    import ctypes
    lib = ctypes.CDLL(ls.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def test_plain_cpp_example_builds_against_the_header():
    """examples/heat_sweep.cpp uses nothing but include/libstencil.h and the HIP runtime: it
    compiles as C++ and links with the library (running it needs a GPU: test_gpu_parity)."""
    from paper_1511_02490_amd import build
    path = build.build_example()
    assert os.path.exists(path) and os.access(path, os.X_OK)


@pytest.mark.parametrize("mode,count", [("pow2", 66), ("even", 590)])
def test_enumeration_matches_definition(mode, count):
    got = ls.enumerate_wg(mode, 1024)
    assert len(got) == count
    assert got == tuning.enumerate_sizes(mode, 1024) == wl.enumerate_wg(mode, 1024)
    assert ls.enumerate_wg(mode, 256) == tuning.enumerate_sizes(mode, 256)


def test_create_validates_arguments():
    for bad in [dict(rows=0, cols=4), dict(rows=4, cols=-1), dict(rows=1 << 20, cols=1 << 20)]:
        with pytest.raises(ls.StencilError) as e:
            ls.Stencil(bad["rows"], bad["cols"])
        assert e.value.code == ls.E_INVALID
    with pytest.raises(ls.StencilError):
        ls.Stencil(8, 8, halo=(1, 1, 33, 1))
    with pytest.raises(ls.StencilError):
        ls.Stencil(8, 8, halo=(1, -1, 1, 1))
    with pytest.raises(ls.StencilError):
        ls.Stencil(8, 8, border=7)
    st = ls.Stencil(8, 8, "u8")
    for bad_pad in (-1.0, 256.0, 0.5):
        with pytest.raises(ls.StencilError):
            st.set_border_value(bad_pad)
    st.set_border_value(1.0)
    with pytest.raises(ls.StencilError):
        st.set_kernel("heat", scalars=(0.2,))            # heat needs f32
    with pytest.raises(ls.StencilError):
        ls.Stencil(8, 8, "f32", (2, 2, 2, 2)).set_kernel("heat", scalars=(0.2,))   # 5-point only
    with pytest.raises(ls.StencilError):
        ls.Stencil(8, 8, "f32", (1, 1, 1, 1)).set_kernel("weighted_sum", np.ones((3, 2), np.float32))
    assert "weights" in ls.last_error()


def test_life_rejects_cells_that_are_not_0_or_1_and_streaming_rejects_4gib_rows():
    st = ls.Stencil(8, 8, "u8", (1, 1, 1, 1), "constant")
    st.set_border_value(3.0)                              # fine for a byte matrix as such ...
    with pytest.raises(ls.StencilError) as e:
        st.set_kernel("life")                             # ... but not for the packed-byte Life kernels
    assert e.value.code == ls.E_INVALID and "0 or 1" in ls.last_error()
    st.set_border_value(1.0)
    st.set_kernel("life")
    with pytest.raises(ls.StencilError):
        st.set_border_value(2.0)
    st.set_border_value(0.0)
    # a near-one-row matrix whose rows are 4 GiB long: the streaming kernels' 32-bit offsets would wrap
    st = ls.Stencil(1, 1 << 30, "f32", (1, 1, 1, 1), "wrap")
    st.set_kernel("heat", scalars=(0.2,))
    st.set_mapping("direct", 1, 4)
    with pytest.raises(ls.StencilError):
        st.set_mapping("stream", 8, 4)
    st = ls.Stencil(1, (1 << 30) - 4, "f32", (1, 1, 1, 1), "wrap")
    st.set_kernel("heat", scalars=(0.2,))
    st.set_mapping("stream", 8, 4)


def test_marching_kernel_serves_run_time_regions_within_its_largest():
    """Weighted sums of floats: a region given at run time is marched if it lies within N5 S5 E4 W4."""
    for halo, ok in [((1, 5, 3, 0), True), ((0, 0, 0, 0), True), ((5, 5, 4, 4), True), ((2, 1, 2, 2), True),
                     ((6, 0, 1, 1), False), ((0, 6, 1, 1), False), ((1, 1, 5, 0), False), ((1, 1, 0, 5), False)]:
        n, s, e, w = halo
        st = ls.Stencil(64, 300, "f32", halo, "wrap")
        st.set_kernel("weighted_sum", np.ones((n + s + 1, e + w + 1), np.float32))
        if ok:
            st.set_mapping("stream", 16, 4)
            assert st.max_wg_size() == 256 and st.is_legal(4, 64) and not st.is_legal(4, 4)
        else:
            with pytest.raises(ls.StencilError):
                st.set_mapping("stream", 16, 4)
    st = ls.Stencil(64, 300, "f64", (1, 1, 1, 1), "wrap")             # floats only
    st.set_kernel("weighted_sum", np.ones((3, 3), np.float32))
    with pytest.raises(ls.StencilError):
        st.set_mapping("stream", 16, 4)


def test_sweep_rotation_is_validated_and_used_by_the_sweeps():
    """Matrix pairs for the sweeps to go round: pointers are checked for overlap (an output may not touch any
    other matrix of the rotation), the number of pairs is bounded, an empty list clears; with every launch made
    to fail, a sweep over a rotation still visits every size (nothing is launched, so no GPU is needed)."""
    import ctypes
    w = wl.config(1, rows=256, cols=256)
    st = ls.Stencil.from_workload(w)
    nbytes = 256 * 256 * 4
    base = 1 << 30
    vp = ctypes.c_void_p

    def rotation(ins, outs):
        n = len(ins)
        return ls._lib.stencil_set_sweep_rotation(st._h, (vp * max(n, 1))(*ins), (vp * max(n, 1))(*outs), n)

    m = [base + k * nbytes for k in range(8)]
    assert rotation([m[0], m[2], m[4]], [m[1], m[3], m[5]]) == ls.OK
    assert rotation([m[0], m[0]], [m[1], m[2]]) == ls.OK                    # a shared input is fine
    assert rotation([m[0], m[1]], [m[1], m[2]]) == ls.E_INVALID             # pair 0 writes what pair 1 reads
    assert "overlaps" in ls.last_error()
    assert rotation([m[0], m[2]], [m[1], m[1] + 64]) == ls.E_INVALID        # two outputs overlap
    assert rotation([m[0]], [m[0] + 128]) == ls.E_INVALID                   # in and out of one pair overlap
    assert rotation([m[0]], [0]) == ls.E_INVALID
    assert rotation([m[0]] * 65, [m[1]] * 65) == ls.E_INVALID               # too many
    assert ls._lib.stencil_set_sweep_rotation(st._h, None, None, 2) == ls.E_INVALID
    assert rotation([m[0], m[2], m[4]], [m[1], m[3], m[5]]) == ls.OK
    st.set_option(ls.OPT_FAIL_LAUNCH, -1)
    sizes = [(4, 4), (8, 8), (16, 16)]
    n = len(sizes)
    mean = (ctypes.c_double * n)(*([7.0] * n))
    status = (ctypes.c_int * n)(*([9] * n))
    best = ctypes.c_int(5)
    a, b = _fake_device_pointers()
    rc = ls._lib.stencil_sweep_wg(st._h, a, b, 4, ls._ints([r for r, _ in sizes]), ls._ints([c for _, c in sizes]), n,
                                  0, 0, 5, mean, None, None, None, status, ctypes.byref(best), None, None)
    assert rc == ls.OK and list(status) == [ls.E_REFUSED] * n and best.value == -1
    assert rotation([], []) == ls.OK
    st.close()


def test_segment_heights_that_fill_whole_wavefront_slots():
    """8192^2, region N1 S5 E3 W0: 63 vectors of 4 cells per strip -> 33 strips; 1024 SIMDs x 3 slots hold 93
    segments per strip, i.e. segments of 89 rows (the height the sweeps find fastest for the sin/cos stencil)."""
    st = ls.Stencil.from_workload(wl.config(4))
    with pytest.raises(ls.StencilError):
        st.stream_segment_rows(3)                         # not on the streaming mapping
    st.set_mapping("stream", 64, 4)
    assert [st.stream_segment_rows(k) for k in (1, 2, 3, 4, 6)] == [265, 133, 89, 67, 45]
    with pytest.raises(ls.StencilError):
        st.stream_segment_rows(0)
    # a 7x7 sum (3/3/3/3: one rim lane each side, 62 vectors): 34 strips; six slots -> 46 rows
    g7 = ls.Stencil(8192, 8192, "f32", (3, 3, 3, 3), "clamp")
    g7.set_kernel("weighted_sum", np.ones((7, 7), np.float32))
    g7.set_mapping("stream", 64, 4)
    assert g7.stream_segment_rows(6) == 46 and g7.stream_segment_rows(2) == 137
    # fewer rows than slots: one row per segment; one narrow tall strip: the kernels' limit
    small = ls.Stencil(8, 100, "f32", (3, 3, 3, 3), "clamp")
    small.set_kernel("weighted_sum", np.ones((7, 7), np.float32))
    small.set_mapping("stream", 4, 4)
    assert small.stream_segment_rows(2) == 1
    tall = ls.Stencil(1 << 24, 16, "f32", (3, 3, 3, 3), "clamp")
    tall.set_kernel("weighted_sum", np.ones((7, 7), np.float32))
    tall.set_mapping("stream", 4, 4)
    with pytest.raises(ls.StencilError) as e:
        tall.stream_segment_rows(1)
    assert e.value.code == ls.E_REFUSED


def test_legality_eq1():
    st = ls.Stencil.from_workload(wl.config(1))          # 5x5 gaussian, halo 2
    assert st.max_wg_size() == 1024
    cands = tuning.enumerate_sizes("pow2", 2048)
    for w in cands:
        tile_ok = st.tile_bytes(*w) <= 160 * 1024
        assert st.is_legal(*w) == (tuning.is_legal(w, 1024) and tile_ok)
    assert not st.is_legal(0, 4) and not st.is_legal(4, 0) and not st.is_legal(-2, 2)
    # the tile of Section 2: (w_r + N + S) x (w_c + E + W) elements of 4 bytes
    assert st.tile_bytes(16, 16) == tuning.tile_elements((16, 16), (2, 2, 2, 2)) * 4
    # a refused parameter: inside W_max, but the tile does not fit local memory
    big = ls.Stencil(4096, 4096, "f32", (30, 30, 30, 30), "clamp")
    big.set_kernel("weighted_sum", np.zeros((61, 61), np.float32))
    assert 32 * 32 <= big.max_wg_size()
    assert big.tile_bytes(32, 32) == (32 + 60) * (32 + 60) * 4 and big.is_legal(32, 32)
    assert big.tile_bytes(64, 16) == (64 + 60) * (16 + 60) * 4 and big.is_legal(64, 16)
    assert big.tile_bytes(8, 128) == (8 + 60) * (128 + 60) * 4 and big.is_legal(8, 128)
    with pytest.raises(ls.StencilError):
        big.set_mapping("direct", 1, 4)                  # no cache-staged variant for a 30-cell region
    big.set_blocking(4, 4)
    assert big.tile_bytes(32, 32) == (128 + 60) * (128 + 64) * 4 and big.is_legal(32, 32)
    assert big.tile_bytes(128, 8) == (512 + 60) * (32 + 64) * 4 and not big.is_legal(128, 8)   # > 160 KiB
    assert "refused" in ls.last_error()


def test_blocking_changes_tile_and_per_kernel_limit():
    st = ls.Stencil.from_workload(wl.config(4))          # sincos N1 S5 E3 W0
    assert st.get_blocking() == (1, 1)
    assert st.tile_bytes(32, 8) == tuning.tile_elements((32, 8), (1, 5, 3, 0)) * 8   # (sin, cos) pairs
    st.set_blocking(8, 4)
    assert st.get_blocking() == (8, 4)
    assert st.max_wg_size() == 256                       # register-heavy variant: lower per-kernel limit
    assert st.is_legal(2, 64) and not st.is_legal(8, 64)          # 512 work-items > 256
    assert st.tile_bytes(4, 64) == 38 * 260 * 8 and st.is_legal(4, 64)   # sine plane + cosine plane
    with pytest.raises(ls.StencilError):
        st.set_blocking(3, 4)
    # cache-staged mapping: no tile in local memory, nothing refused below W_max
    heat = ls.Stencil.from_workload(wl.config(3))
    heat.set_mapping("direct", 1, 4)
    assert heat.get_mapping() == (ls.STAGING_DIRECT, 1, 4)
    assert heat.tile_bytes(32, 32) == 0 and heat.is_legal(1, 1024) and not heat.is_legal(2, 1024)
    heat.set_mapping("local", 8, 4)
    assert heat.tile_bytes(32, 32) == (256 + 2) * (128 + 8) * 4 and heat.is_legal(32, 32)
    assert heat.tile_bytes(128, 8) == (1024 + 2) * (32 + 8) * 4 and not heat.is_legal(128, 8)   # > 160 KiB


def test_kernels_whose_output_type_differs_from_the_input():
    """Section 3.3 lists input and output element types among a kernel's features."""
    blur = ls.Stencil.from_workload(wl.image_blur(512, 512))        # bytes in, floats out
    assert blur.output_dtype() == ls.F32
    f = blur.features()
    assert f[2] == 1.0 and f[12] == 4.0
    assert blur.tile_bytes(16, 16) == (16 + 4) * (16 + 4) * 4           # the tile holds the cells as floats
    blur.set_blocking(1, 16)
    assert blur.tile_bytes(4, 16) == (4 + 4) * (256 + 32) * 4           # extents widened to whole 16-cell vectors
    blur.set_blocking(2, 16)
    assert blur.max_wg_size() == 256
    with pytest.raises(ls.StencilError):
        blur.set_mapping("direct", 1, 16)
    edges = ls.Stencil.from_workload(wl.canny_stage(wl.THRESHOLD, 512, 512))   # floats in, bytes out
    assert edges.output_dtype() == ls.U8
    f = edges.features()
    assert f[2] == 4.0 and f[12] == 1.0
    heat = ls.Stencil.from_workload(wl.config(3))
    assert heat.output_dtype() == ls.F32


def test_sweep_reduce_matches_definitions():
    rng = np.random.default_rng(0)
    for trial in range(20):
        sizes = tuning.enumerate_sizes("pow2", 1024)
        ms = rng.choice([0.5, 1.0, 2.0, 3.0, 7.5], size=len(sizes)).tolist()
        ok = (rng.random(len(sizes)) > 0.2).tolist()
        status = [ls.OK if o else ls.E_REFUSED for o in ok]
        ms = [m if o else float("nan") for m, o in zip(ms, ok)]
        fixed_ms = float(rng.choice([4.0, float("nan")]))
        best, perf, sp = ls.sweep_reduce(sizes, ms, status, fixed_ms)
        assert best == tuning.oracle_size(sizes, ms, ok)
        ref_perf = tuning.performance(ms, ok, best)
        for a, b in zip(perf, ref_perf):
            assert (math.isnan(a) and math.isnan(b)) or a == b
        if math.isnan(fixed_ms):
            assert math.isnan(sp)
        else:
            assert sp == tuning.speedup(fixed_ms, ms[best])
    # by inspection
    best, perf, sp = ls.sweep_reduce([(4, 4), (8, 8), (64, 4)], [4.0, 2.0, 1.0], [0, 0, 0], 4.0)
    assert best == 2 and perf == [0.25, 0.5, 1.0] and sp == 4.0
    best, perf, sp = ls.sweep_reduce([(4, 4)], [float("nan")], [ls.E_REFUSED], 1.0)
    assert best == -1 and math.isnan(sp)


def test_features_and_prediction_algorithm1():
    scen = [ls.Stencil.from_workload(wl.config(i)) for i in range(5)]
    feats = [s.features() for s in scen]
    assert feats[1][:9] == [2048.0, 2048.0, 4.0, 2.0, 2.0, 2.0, 2.0, 25.0, 0.0]
    assert feats[2][2] == 1.0 and feats[4][8] == 1.0 and feats[4][7] == 28.0
    # kernel descriptors (operations per cell stated by the customising function, of which on the
    # transcendental unit) and the border mode tell apart scenarios whose dataset features coincide
    assert len(feats[0]) == ls.N_FEATURES == 16
    assert feats[0][13:16] == [17.0, 0.0, 0.0] and feats[1][13:16] == [49.0, 0.0, 0.0]
    assert feats[2][13:16] == [11.0, 0.0, 1.0] and feats[3][13:16] == [7.0, 0.0, 1.0] and feats[4][13:16] == [85.0, 2.0, 2.0]
    same_data = []
    for kernel in ("weighted_sum", "heat", "sobel", "nms"):
        st = ls.Stencil(1024, 1024, "f32", (1, 1, 1, 1), "clamp")
        st.set_kernel(kernel, np.zeros((3, 3), np.float32), scalars=(0.2,))
        same_data.append(tuple(st.features()))
    assert len(set(same_data)) == 4 and len({f[:13] for f in same_data}) == 1
    if not _gpu_visible():
        # no GPU has been asked: the device features are the header's constants
        assert feats[0][9:12] == [256.0, 163840.0, 1024.0]
    labels = [(8, 8), (4, 64), (16, 16), (2, 128), (64, 32)]      # the last is above any W_max
    pred = ls.Predictor()
    for f, w in zip(feats, labels):
        pred.add(f, w)
    probe = ls.Stencil(2000, 2100, "f32", (2, 2, 2, 2), "clamp")
    probe.set_kernel("weighted_sum", np.zeros((5, 5), np.float32))
    assert pred.classify(probe.features()) == tuning.classify_1nn(feats, labels, probe.features()) == (4, 64)
    cands = tuning.enumerate_sizes("pow2", 1024)
    assert probe.predict(pred, cands) == (4, 64)                  # legal: returned as classified
    # a scenario whose nearest training label is illegal falls back to the closest legal size
    probe2 = ls.Stencil(8000, 8000, "f32", (1, 5, 3, 0), "constant")
    probe2.set_kernel("sincos", np.zeros((7, 4), np.float32))
    assert pred.classify(probe2.features()) == (64, 32)
    legal = [c for c in cands if probe2.is_legal(*c)]
    expect = tuning.predict_nearest_neighbour((64, 32), legal, 1024)
    assert probe2.predict(pred, cands) == expect == (64, 16)      # distance 16; (32,32) is 32 away
    # the other two handlers of Algorithm 1
    refused = [c for c in cands if not probe2.is_legal(*c)]
    assert probe2.predict(pred, cands, "baseline", baseline=(4, 4)) == tuning.predict_baseline((64, 32), (4, 4), 1024, refused) == (4, 4)
    assert probe.predict(pred, cands, "baseline", baseline=(4, 4)) == (4, 64)      # legal prediction is kept
    with pytest.raises(ls.Refused):
        probe2.predict(pred, cands, "baseline", baseline=(64, 64))
    for draw in (0, 7, 12345678901234567):
        got = probe2.predict(pred, cands, "random", random=draw)
        assert got == tuning.predict_random((64, 32), cands, 1024, refused, draw) and probe2.is_legal(*got)
    assert probe.predict(pred, cands, "random", random=99) == (4, 64)
    with pytest.raises(ls.Refused):
        probe2.predict(pred, [(2048, 1)])
    with pytest.raises(ls.StencilError):
        ls.Predictor().classify(feats[0])


def _gpu_visible():
    try:
        import torch
        return torch.cuda.is_available()
    except ImportError:
        return False


def _fake_device_pointers():
    import ctypes
    return ctypes.c_void_p(0x10000000), ctypes.c_void_p(0x30000000)     # never dereferenced: no launch is made


def test_sweep_records_launch_failures_as_refused_and_finishes():
    """Section 3.1: some sizes are refused only when launched; Section 4.2: the tuner strikes them and
    goes on.  With every launch made to fail (STENCIL_OPT_FAIL_LAUNCH, a testing aid that puts the
    runtime's out-of-resources error in the launch's place) the sweep still visits every size,
    records each as refused and returns; no GPU is needed since nothing is launched."""
    import ctypes
    w = wl.config(1, rows=256, cols=256)
    st = ls.Stencil.from_workload(w)
    st.set_option(ls.OPT_FAIL_LAUNCH, -1)
    sizes = [(4, 4), (8, 8), (64, 32), (16, 16)]            # the third is beyond W_max anyway
    n = len(sizes)
    a, b = _fake_device_pointers()
    mean = (ctypes.c_double * n)(*([7.0] * n))
    status = (ctypes.c_int * n)(*([9] * n))
    best, sp = ctypes.c_int(5), ctypes.c_double(1.0)
    rc = ls._lib.stencil_sweep_wg(st._h, a, b, 1, ls._ints([r for r, _ in sizes]), ls._ints([c for _, c in sizes]), n,
                                  4, 4, 5, mean, None, None, None, status, ctypes.byref(best), ctypes.byref(sp), None)
    assert rc == ls.OK
    assert list(status) == [ls.E_REFUSED] * n and all(math.isnan(x) for x in mean)
    assert best.value == -1 and math.isnan(sp.value)
    assert "refused at launch" in ls.last_error() and "16x16" in ls.last_error()
    # the same failure from a plain run is the refusal code, with the runtime's text
    assert ls._lib.stencil_run(st._h, a, b, 1, 8, 8, None) == ls.E_REFUSED
    assert "8x8 refused at launch" in ls.last_error()
    # only one size made to fail: the others are no longer touched by the aid (they would launch)
    st.set_option(ls.OPT_FAIL_LAUNCH, (8 << 16) | 8)
    assert ls._lib.stencil_run(st._h, a, b, 1, 8, 8, None) == ls.E_REFUSED
    with pytest.raises(ls.StencilError):
        st.set_option(ls.OPT_FAIL_LAUNCH, -7)
    st.set_option(ls.OPT_FAIL_LAUNCH, 0)
    st.close()


def test_predictor_from_a_text_file_and_inside_the_librarys_own_choice(tmp_path):
    """stencil_predictor_load reads (f(s), size) pairs from text; an attached classifier decides
    what stencil_run(0, 0) launches when the handle has no sweep to go by (Section 2: choosing the
    size is the implementation's job).  The chosen size shows in the text of a launch made to fail."""
    scen = [ls.Stencil.from_workload(wl.config(i)) for i in range(5)]
    labels = [(8, 8), (4, 64), (16, 16), (2, 128), (64, 32)]
    path = tmp_path / "pairs.txt"
    with open(path, "w") as fh:
        fh.write("# five pairs\n\nfeatures %d\n" % ls.N_FEATURES)
        for st, (r, c) in zip(scen, labels):
            fh.write("# a comment between the pairs\n" + " ".join(repr(x) for x in st.features()) + " %d %d\n" % (r, c))
    by_hand = ls.Predictor("nearest")
    for st, lab in zip(scen, labels):
        by_hand.add(st.features(), lab)
    for kind in ("nearest", "tree", "zeror"):
        pred = ls.Predictor.load(str(path), kind)
        for st, lab in zip(scen, labels):
            assert pred.classify(st.features()) == (lab if kind != "zeror" else (8, 8))
        pred.close()
    pred = ls.Predictor.load(str(path), "nearest")
    probe = ls.Stencil(2000, 2100, "f32", (2, 2, 2, 2), "clamp")
    probe.set_kernel("weighted_sum", np.zeros((5, 5), np.float32))
    assert pred.classify(probe.features()) == by_hand.classify(probe.features()) == (4, 64)
    a, b = _fake_device_pointers()

    def chosen(st):
        # the size shows in the text of a launch made to fail, and stencil_default_wg names the same
        st.set_option(ls.OPT_FAIL_LAUNCH, -1)
        assert ls._lib.stencil_run(st._h, a, b, 1, 0, 0, None) == ls.E_REFUSED
        st.set_option(ls.OPT_FAIL_LAUNCH, 0)
        seen = tuple(int(x) for x in re.search(r"workgroup size (\d+)x(\d+) refused at launch", ls.last_error()).groups())
        assert st.default_wg() == seen
        return seen

    assert chosen(probe) == (4, 64)                         # nothing attached: the built-in default (also 4x64)
    probe2 = ls.Stencil(300, 300, "f32", (1, 1, 1, 1), "clamp")
    probe2.set_kernel("weighted_sum", np.zeros((3, 3), np.float32))
    assert chosen(probe2) == (4, 64)
    probe2.attach_predictor(pred)
    assert chosen(probe2) == pred.classify(probe2.features()) == (8, 8)      # nearest: C1
    # an illegal prediction is repaired by the attached handler (Algorithm 1)
    probe3 = ls.Stencil(8000, 8000, "f32", (1, 5, 3, 0), "constant")
    probe3.set_kernel("sincos", np.zeros((7, 4), np.float32))
    probe3.attach_predictor(pred, "nearest")
    assert pred.classify(probe3.features()) == (64, 32) and chosen(probe3) == (64, 16)
    probe3.attach_predictor(pred, "baseline")
    assert chosen(probe3) == (4, 64)                        # the baseline handler falls back to the built-in default
    probe3.attach_predictor(None)
    assert chosen(probe3) == (4, 64)
    # files that do not parse
    for text in ("", "features 3\n", "1 2 3 4 5\n", "features 3\n1 2 3 4\n", "features 3\n1 2 3 0 4\n", "features 2\n1 x 3 4\n"):
        bad = tmp_path / "bad.txt"
        bad.write_text(text)
        with pytest.raises(ls.StencilError):
            ls.Predictor.load(str(bad))
    with pytest.raises(ls.StencilError):
        ls.Predictor.load(str(tmp_path / "missing.txt"))


def test_pretrained_predictor_ships_with_the_library():
    """The (f(s), oracle size) pairs recorded on the device are loaded into a classifier; what it
    predicts, repaired by Algorithm 1's fallback, is a legal size for every benchmark workload."""
    sizes = ls.enumerate_wg("pow2", 1024)
    for mapping in ("local,1,1", "local,2,4"):
        for kind in ("tree", "nearest", "zeror"):
            pred = ls.pretrained_predictor(mapping, kind)
            for i in range(5):
                st = ls.Stencil.from_workload(wl.config(i))
                m = mapping.split(",")
                try:
                    st.set_mapping(m[0], int(m[1]), int(m[2]))
                except ls.StencilError:
                    continue                                  # Life has no 2x4 blocking
                wr, wc = st.predict(pred, sizes)
                assert (wr, wc) in sizes and st.is_legal(wr, wc)
                st.close()
            pred.close()
    # the study's most common oracle size under the paper's mapping is what ZeroR answers
    st = ls.Stencil.from_workload(wl.config(3))
    assert st.predict(ls.pretrained_predictor("local,1,1", "zeror"), sizes) == (16, 32)
    with pytest.raises(ValueError):
        ls.pretrained_predictor("direct,2,4")


def test_baseline_handler_matches_definition():
    sizes = [(4, 4), (8, 8), (64, 4)]
    nan = float("nan")
    perf = [[0.5, 1.0, nan], [0.5, 0.16, 1.0]]
    # (64,4) is not safe; geometric means 0.5 vs 0.4
    assert ls.baseline_wg(perf) == 0
    dicts = [{w: p for w, p in zip(sizes, row) if not math.isnan(p)} for row in perf]
    safe = tuning.safe_set([list(d) for d in dicts])
    assert sizes[ls.baseline_wg(perf)] == tuning.baseline_size(dicts, safe)
    perf[1][1] = 0.36
    assert ls.baseline_wg(perf) == 1
    assert ls.baseline_wg([[nan, 1.0], [1.0, nan]]) == -1
    rng = np.random.default_rng(3)
    for _ in range(20):
        table = rng.uniform(0.05, 1.0, size=(6, 9))
        table[rng.random(table.shape) < 0.1] = np.nan
        dicts = [{j: p for j, p in enumerate(row) if not np.isnan(p)} for row in table]
        safe = tuning.safe_set([list(d) for d in dicts])
        expect = tuning.baseline_size(dicts, safe)
        got = ls.baseline_wg(table.tolist())
        assert (got == -1 and expect is None) or got == expect


def test_tree_and_zeror_classifiers_match_definitions():
    rng = np.random.default_rng(11)
    labels_pool = [(64, 4), (8, 8), (16, 16), (4, 64), (32, 32)]
    for trial in range(10):
        n, nf = int(rng.integers(3, 40)), int(rng.integers(1, 6))
        X = rng.integers(0, 6, size=(n, nf)).astype(float).tolist()      # repeated values and ties
        W = [labels_pool[int(k)] for k in rng.integers(0, len(labels_pool), size=n)]
        tree = tuning.grow_tree(X, W)
        pt, pz = ls.Predictor("tree"), ls.Predictor("zeror")
        for x, w in zip(X, W):
            pt.add(x, w)
            pz.add(x, w)
        probes = rng.uniform(-1, 7, size=(30, nf)).tolist() + X
        for x in probes:
            assert pt.classify(x) == tuning.classify_tree(tree, x)
            assert pz.classify(x) == tuning.classify_zeror(W)
    with pytest.raises(ls.StencilError):
        ls.Predictor("tree").classify([1.0])


def test_algorithm2_regression_matches_definition():
    scen = [ls.Stencil.from_workload(wl.config(i)) for i in range(5)]
    feats = [s.features() for s in scen]
    cands = tuning.enumerate_sizes("pow2", 2048)
    rng = np.random.default_rng(17)
    reg = ls.Regressor()
    X, W, Y = [], [], []
    for f in feats[:4]:
        for w in cands:
            if rng.random() < 0.8:
                y = float(rng.uniform(0.1, 5.0))
                reg.add(f, w, y)
                X.append(f); W.append(w); Y.append(y)
    big = ls.Stencil(4096, 4096, "f32", (30, 30, 30, 30), "clamp")      # many refused sizes (tile > local memory)
    big.set_kernel("weighted_sum", np.zeros((61, 61), np.float32))
    big.set_mapping("local", 4, 4)
    for st in (scen[4], big):
        f = st.features()
        for w in cands[::7]:
            a, b = reg.predict(f, w), tuning.regress_1nn(X, W, Y, f, w)
            assert (math.isnan(a) and math.isnan(b)) or a == b
        refused = [c for c in cands if c[0] * c[1] <= st.max_wg_size() and not st.is_legal(*c)]
        for fitness, fn in (("reciprocal", lambda y: 1.0 / y), ("identity", lambda y: y)):
            got, struck = st.predict_regression(reg, cands, fitness)
            exp, exp_struck = tuning.predict_by_regression(lambda w: tuning.regress_1nn(X, W, Y, f, w), cands,
                                                           st.max_wg_size(), refused, fn)
            assert got == exp and struck == exp_struck and st.is_legal(*got)
    assert len([c for c in cands if c[0] * c[1] <= 1024 and not big.is_legal(*c)]) > 5
    with pytest.raises(ls.StencilError):
        scen[0].predict_regression(ls.Regressor(), cands)


def test_random_forest_regressor_matches_definition():
    """The library's forest against the oracle's, given the same bootstrap rows and input masks:
    the same cuts, so the same predictions to the last bit, on training tuples and elsewhere."""
    rng = np.random.default_rng(23)
    nf = 5
    scen_f = rng.random((9, nf)) * np.array([4096.0, 4096.0, 8.0, 30.0, 1.0])
    sizes = tuning.enumerate_sizes("pow2", 256)
    reg = ls.Regressor()
    xs, ys, fs, ws = [], [], [], []
    for f in scen_f.tolist():
        for w in sizes:
            if rng.random() < 0.7:
                y = float(math.log(f[0] * f[1]) / (w[0] * w[1]) ** 0.5 + 0.3 * abs(math.log2(w[1]) - 5) + 0.05 * rng.random())
                reg.add(f, w, y)
                xs.append(list(f) + [float(w[0]), float(w[1])]); ys.append(y); fs.append(f); ws.append(w)
    n, ni = len(ys), nf + 2
    probes = [(f, w) for f in (rng.random((6, nf)) * np.array([4096.0, 4096.0, 8.0, 30.0, 1.0])).tolist() for w in sizes[::3]]
    probes += list(zip(fs, ws))[::5]
    for n_trees, n_rows, min_leaf, max_depth in [(1, 0, 1, 64), (5, n, 2, 6), (8, n // 2, 1, 64), (3, n, 7, 2)]:
        bootstrap = rng.integers(0, n, size=(n_trees, n_rows)).tolist() if n_rows else None
        masks = (rng.random((n_trees, ni)) < 0.6)
        masks[:, ni - 1] = True                                  # never a tree without an open input
        masks = masks.tolist() if n_rows else None
        reg.fit_forest(bootstrap, masks, n_trees=n_trees, min_leaf=min_leaf, max_depth=max_depth)
        forest = tuning.grow_forest(xs, ys, bootstrap if bootstrap else [list(range(n))] * n_trees,
                                    masks if masks else [[True] * ni] * n_trees, min_leaf, max_depth)
        for f, w in probes:
            assert reg.predict(f, w) == tuning.predict_forest(forest, list(f) + [float(w[0]), float(w[1])])
    # a fully grown single tree on all tuples reproduces its training targets (the tuples are distinct)
    reg.fit_forest(None, None, n_trees=1)
    assert all(abs(reg.predict(f, w) - y) < 1e-12 for f, w, y in zip(fs, ws, ys))
    # adding a tuple discards the forest: back to the nearest-neighbour rule
    reg.add(fs[0], (3, 3), 42.0)
    assert reg.predict(fs[0], (3, 3)) == 42.0 and math.isnan(reg.predict(fs[0], (5, 5)))
    with pytest.raises(ls.StencilError):
        reg.fit_forest([[0, n + 5]], None)                       # bootstrap index out of range
    with pytest.raises(ls.StencilError):
        reg.fit_forest(None, [[False] * ni])                     # a tree with no input
    with pytest.raises(ls.StencilError):
        ls.Regressor().fit_forest(None, None, n_trees=2)         # nothing to grow on


def test_study_evaluates_a_fabricated_landscape(tmp_path, capsys, monkeypatch):
    """The autotuning study's evaluation stage (Section 7's metrics over Algorithms 1 and 2, all
    through the C ABI) on sweeps made up so that prediction matters: the best size is 4x64 on
    matrices up to 1024^2 and 8x64 above.  A decision tree and a forest on speedups learn that
    from the other scenarios; the best fixed size is right for half of them."""
    import json
    import sys
    from paper_1511_02490_amd import autotune_study
    sizes = ls.enumerate_wg("pow2", 1024)
    scen = wl.real_scenarios()
    times, status, feats = [], [], []
    for w in scen:
        st = ls.Stencil.from_workload(w)
        feats.append(st.features())
        legal = [st.is_legal(r, c) for r, c in sizes]
        tall = 4 if w.rows <= 1024 else 8
        times.append([(abs(r - tall) + 1) * (abs(c - 64) + 32) * w.rows * 1e-6 if ok else float("nan")
                      for (r, c), ok in zip(sizes, legal)])
        status.append([0 if ok else ls.E_REFUSED for ok in legal])
        st.close()
    path = tmp_path / "sweeps.json"
    path.write_text(json.dumps({"sizes": sizes, "scenarios": [w.name for w in scen], "times_ms": times, "status": status,
                                "features": feats, "mapping": "local,1,1", "reps": 3, "sweep_seconds": 1.0}))
    monkeypatch.setattr(sys, "argv", ["autotune_study", "--synthetic", "0", "--mapping", "local,1,1", "--from-json", str(path)])
    autotune_study.main()
    report = capsys.readouterr().out
    rows = {line.split("|")[1].strip(): [c.strip() for c in line.split("|")[2:-1]]
            for line in report.splitlines() if line.startswith("| leave-one-out") or line.startswith("| ZeroR")}
    assert rows["leave-one-out, decision tree + NearestNeighbour"][1] == "100 %"        # accuracy
    assert rows["leave-one-out, decision tree + NearestNeighbour"][3] == "100 %"        # performance
    assert int(rows["leave-one-out, random forest on speedups (Algorithm 2)"][1].split()[0]) >= 90
    assert rows["ZeroR (always the baseline size)"][1] == "50 %"
    assert all(r[2] == "100 %" for r in rows.values())                                  # every first answer legal
    # sweeps taken under the fastest mapping of each scenario carry that mapping with them
    path.write_text(json.dumps({"sizes": sizes, "scenarios": [w.name for w in scen], "times_ms": times, "status": status,
                                "features": feats, "mapping": "best", "mappings": [["local", 2, 4]] * len(scen), "reps": 3,
                                "sweep_seconds": 1.0}))
    monkeypatch.setattr(sys, "argv", ["autotune_study", "--synthetic", "0", "--mapping", "best", "--from-json", str(path)])
    autotune_study.main()
    report = capsys.readouterr().out
    assert "fastest mapping: local for %d scenarios" % len(scen) in report
    assert sum("| local 2x4 |" in line for line in report.splitlines()) == len(scen)


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU: asked for more it says so and exits before touching a device."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    out = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], cwd=root, capture_output=True,
                         text=True, timeout=120)
    assert out.returncode != 0 and "one GPU" in out.stderr and out.stdout.strip() == ""

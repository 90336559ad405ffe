"""Pins for the host-side definitions (legality, oracle size, metrics, fallback handlers):
hand-made tables whose answers can be read off by inspection, and closed counts."""
import math

import pytest

from oracle import tuning


def test_enumeration_closed_counts():
    """Powers of two with product <= 2^10: pairs (a, b) of exponents with a + b <= 10 ->
    11 * 12 / 2 = 66.  Even sizes 2..64 = 2i, 2j with i*j <= 256, i, j <= 32: 590."""
    p2 = tuning.enumerate_sizes("pow2", 1024)
    assert len(p2) == 66 and len(set(p2)) == 66
    assert (1, 1) in p2 and (1024, 1) in p2 and (1, 1024) in p2 and (32, 32) in p2 and (64, 32) not in p2
    ev = tuning.enumerate_sizes("even", 1024)
    assert len(ev) == sum(1 for i in range(1, 33) for j in range(1, 33) if i * j <= 256) == 590
    assert all(r % 2 == 0 and c % 2 == 0 and 2 <= r <= 64 and 2 <= c <= 64 and r * c <= 1024 for r, c in ev)
    # the strict reading of Eq. 1 (w < W_max) would drop the three sizes with exactly 1024 items
    assert sum(1 for r, c in ev if r * c == 1024) == 3
    assert len(tuning.enumerate_sizes("pow2", 256)) == 9 * 10 // 2


def test_tile_elements_fig1():
    # Figure 1: 1 south, 2 north / east / west around a w_r x w_c workgroup
    assert tuning.tile_elements((4, 8), (2, 1, 2, 2)) == (4 + 3) * (8 + 4)
    assert tuning.tile_elements((16, 16), (2, 2, 2, 2)) == 400
    assert tuning.tile_elements((32, 8), (1, 5, 3, 0)) == 38 * 11


def test_legality_eq1_and_safe_set_eq2():
    refused = [(32, 4)]
    assert tuning.is_legal((32, 32), 1024)
    assert not tuning.is_legal((64, 32), 1024)
    assert not tuning.is_legal((32, 4), 1024, refused)
    assert tuning.is_legal((4, 32), 1024, refused)
    assert not tuning.is_legal((0, 4), 1024) and not tuning.is_legal((4, -1), 1024)
    assert tuning.is_legal((16, 16), 256) and not tuning.is_legal((16, 32), 256)
    cands = [(4, 4), (32, 4), (16, 16), (32, 32)]
    s1 = tuning.legal_set(cands, 1024, refused)          # loses (32,4)
    s2 = tuning.legal_set(cands, 256)                    # loses (32,32)
    assert s1 == [(4, 4), (16, 16), (32, 32)] and s2 == [(4, 4), (32, 4), (16, 16)]
    assert tuning.safe_set([s1, s2]) == [(4, 4), (16, 16)]


def test_oracle_size_and_metrics_by_inspection():
    sizes = [(4, 4), (8, 8), (64, 4), (32, 32), (2, 2)]
    ms = [4.0, 2.0, 1.0, float("nan"), 8.0]
    ok = [True, True, True, False, True]
    best = tuning.oracle_size(sizes, ms, ok)
    assert sizes[best] == (64, 4)
    perf = tuning.performance(ms, ok, best)
    assert perf[:3] == [0.25, 0.5, 1.0] and math.isnan(perf[3]) and perf[4] == 0.125
    red = tuning.sweep_reduce(sizes, ms, ok, fixed=(4, 4))
    assert red["best_index"] == 2 and red["speedup_over_fixed"] == 4.0 and red["best_over_worst"] == 8.0
    # fixed size not in the list: its runtime is supplied separately
    red2 = tuning.sweep_reduce(sizes, ms, ok, fixed=(32, 4), fixed_ms=3.0)
    assert red2["speedup_over_fixed"] == 3.0
    # fixed size refused -> no speedup
    red3 = tuning.sweep_reduce(sizes, ms, ok, fixed=(32, 32))
    assert math.isnan(red3["speedup_over_fixed"])
    # a refused size never wins even with a tiny recorded time
    assert tuning.oracle_size([(4, 4), (8, 8)], [5.0, 0.1], [True, False]) == 0
    assert tuning.oracle_size([(4, 4)], [float("nan")], [False]) == -1


def test_oracle_size_tie_break():
    sizes = [(16, 16), (8, 8), (4, 16), (16, 4)]
    ms = [1.0, 1.0, 1.0, 1.0]
    ok = [True] * 4
    # fewer work-items first -> 64-item sizes; among them the smaller w_r
    assert sizes[tuning.oracle_size(sizes, ms, ok)] == (4, 16)


def test_baseline_handler_geometric_mean():
    perf = [{(4, 4): 0.5, (8, 8): 1.0}, {(4, 4): 0.5, (8, 8): 0.16}]
    # geometric means: 0.5 vs 0.4
    assert tuning.baseline_size(perf, [(4, 4), (8, 8)]) == (4, 4)
    perf[1][(8, 8)] = 0.36   # 0.5 vs 0.6
    assert tuning.baseline_size(perf, [(4, 4), (8, 8)]) == (8, 8)


def test_nearest_neighbour_fallback_by_hand():
    cands = [(4, 4), (32, 4), (16, 64)]
    # prediction legal -> returned unchanged, even if it is not one of the candidates
    assert tuning.predict_nearest_neighbour((8, 8), cands, 1024) == (8, 8)
    # (64, 32) has 2048 items: distances to candidates are
    #   (4,4): sqrt(60^2+28^2)=66.2   (32,4): sqrt(32^2+28^2)=42.5   (16,64): sqrt(48^2+32^2)=57.7
    assert tuning.predict_nearest_neighbour((64, 32), cands, 1024) == (32, 4)
    # ... and if (32,4) is a refused parameter the next closest wins
    assert tuning.predict_nearest_neighbour((64, 32), cands, 1024, refused=[(32, 4)]) == (16, 64)
    # a legal-looking prediction that is known to be refused is moved as well
    assert tuning.predict_nearest_neighbour((32, 4), cands, 1024, refused=[(32, 4)]) == (4, 4)
    # candidates above W_max are not eligible
    assert tuning.predict_nearest_neighbour((64, 32), cands, 127) == (4, 4)
    assert tuning.predict_nearest_neighbour((64, 32), [], 1024) is None
    # ties keep the first candidate
    assert tuning.nearest_legal((10, 10), [(8, 10), (12, 10)]) == (8, 10)


def test_1nn_classifier_by_hand():
    # features: (rows, halo area); the first feature spans 1000, the second spans 10
    X = [(1000.0, 9.0), (2000.0, 9.0), (2000.0, 19.0)]
    W = [(8, 8), (64, 4), (16, 16)]
    assert tuning.classify_1nn(X, W, (1900.0, 10.0)) == (64, 4)     # 0.1^2+0.1^2 beats 0.1^2+0.9^2
    assert tuning.classify_1nn(X, W, (1900.0, 18.0)) == (16, 16)
    assert tuning.classify_1nn(X, W, (0.0, 9.0)) == (8, 8)
    # a feature that is constant over the training set carries no distance
    X2 = [(5.0, 1.0), (5.0, 2.0)]
    assert tuning.classify_1nn(X2, [(4, 4), (8, 8)], (500.0, 1.9)) == (8, 8)


def test_baseline_and_random_handlers_by_hand():
    cands = [(4, 4), (32, 4), (16, 64)]
    assert tuning.predict_baseline((8, 8), (4, 4), 1024) == (8, 8)
    assert tuning.predict_baseline((64, 32), (4, 4), 1024) == (4, 4)
    assert tuning.predict_baseline((64, 32), (4, 4), 1024, refused=[(4, 4)]) is None
    assert tuning.predict_random((8, 8), cands, 1024, [], 5) == (8, 8)
    # legal pool in list order: (4,4), (16,64) once (32,4) is refused; draw 3 -> index 1
    assert tuning.predict_random((64, 32), cands, 1024, [(32, 4)], 3) == (16, 64)
    assert tuning.predict_random((64, 32), cands, 1024, [(32, 4)], 4) == (4, 4)
    assert tuning.predict_random((64, 32), [], 1024, [], 4) is None


def test_decision_tree_by_hand():
    """Four scenarios, two features.  Feature 0 separates {A, A} from {B, C} with gain 1 bit (the
    parent has entropy 1.5 bits, the children 0 and 1); feature 1 cannot do better, so the root
    splits on feature 0 at the midpoint 15; the right child then splits on feature 1 at 2.5."""
    X = [(10.0, 1.0), (10.0, 9.0), (20.0, 2.0), (20.0, 3.0)]
    A, B, C = (64, 4), (8, 8), (16, 16)
    W = [A, A, B, C]
    tree = tuning.grow_tree(X, W)
    assert tree == ("split", 0, 15.0, ("leaf", A), ("split", 1, 2.5, ("leaf", B), ("leaf", C)))
    assert tuning.classify_tree(tree, (12.0, 100.0)) == A
    assert tuning.classify_tree(tree, (15.0, 0.0)) == A          # x <= t goes left
    assert tuning.classify_tree(tree, (99.0, 2.5)) == B
    assert tuning.classify_tree(tree, (99.0, 2.6)) == C
    # identical features with different labels cannot be split: majority, first among equals
    tree2 = tuning.grow_tree([(1.0,), (1.0,), (1.0,)], [B, A, A])
    assert tree2 == ("leaf", A)
    assert tuning.grow_tree([(1.0,), (1.0,)], [B, A]) == ("leaf", B)
    # a training set is always classified back correctly when its features are distinct
    import random
    rnd = random.Random(5)
    X3 = [(rnd.random(), rnd.random(), float(rnd.randrange(4))) for _ in range(40)]
    W3 = [rnd.choice([A, B, C, (4, 64)]) for _ in range(40)]
    t3 = tuning.grow_tree(X3, W3)
    assert all(tuning.classify_tree(t3, x) == w for x, w in zip(X3, W3))
    assert tuning.classify_zeror([B, A, A, B, C]) == B and tuning.classify_zeror([C, A, A]) == A


def test_algorithm2_regression_by_hand():
    # two training scenarios (feature 10 and 20), runtimes per size
    X = [(10.0,), (10.0,), (10.0,), (20.0,), (20.0,), (20.0,)]
    W = [(4, 4), (8, 8), (64, 4)] * 2
    Y = [4.0, 2.0, 1.0, 9.0, 3.0, 5.0]
    assert tuning.regress_1nn(X, W, Y, (11.0,), (8, 8)) == 2.0
    assert tuning.regress_1nn(X, W, Y, (19.0,), (8, 8)) == 3.0
    assert math.isnan(tuning.regress_1nn(X, W, Y, (19.0,), (2, 2)))
    cands = [(4, 4), (8, 8), (64, 4), (2, 2), (64, 32)]
    near10 = lambda w: tuning.regress_1nn(X, W, Y, (11.0,), w)
    recip = lambda y: 1.0 / y
    # fastest predicted runtime wins; (2,2) has no tuple, (64,32) is above W_max
    assert tuning.predict_by_regression(near10, cands, 1024, [], recip) == ((64, 4), 0)
    # a refused parameter is struck and the next best taken
    assert tuning.predict_by_regression(near10, cands, 1024, [(64, 4)], recip) == ((8, 8), 1)
    assert tuning.predict_by_regression(near10, cands, 1024, [(64, 4), (8, 8), (4, 4)], recip) == (None, 3)
    # speedups: identity fitness picks the largest
    assert tuning.predict_by_regression(near10, cands, 1024, [], lambda y: y) == ((4, 4), 0)

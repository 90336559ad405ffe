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


def test_regression_tree_by_hand_and_by_brute_force():
    # a step in input 0, input 1 is noise: one split, midway between the two points next to the step
    X = [(0.1, 5.0), (0.2, 1.0), (0.4, 3.0), (0.7, 2.0), (0.8, 4.0), (0.9, 0.0)]
    Y = [1.0, 1.0, 1.0, 3.0, 3.0, 3.0]
    tree = tuning.grow_regression_tree(X, Y, [True, True])
    assert tree == ("node", 0, (0.4 + 0.7) / 2.0, ("leaf", 1.0), ("leaf", 3.0))
    assert tuning.predict_regression_tree(tree, (0.55, 9.0)) == 1.0
    assert tuning.predict_regression_tree(tree, (0.5500001, -9.0)) == 3.0
    # input 0 closed to the tree: it has to make do with the noise input
    blind = tuning.grow_regression_tree(X, Y, [False, True])
    assert blind[0] == "node" and blind[1] == 1
    # equal targets, too few tuples for two leaves, depth 0: a leaf with the mean
    assert tuning.grow_regression_tree(X, [2.0] * 6, [True, True]) == ("leaf", 2.0)
    assert tuning.grow_regression_tree(X, Y, [True, True], min_leaf=4) == ("leaf", 2.0)
    assert tuning.grow_regression_tree(X, Y, [True, True], max_depth=0) == ("leaf", 2.0)
    # brute force: the root split minimises the summed squared error over every (input, cut)
    import random
    rnd = random.Random(11)
    for trial in range(20):
        n = rnd.randrange(4, 9)
        Xr = [(rnd.random(), float(rnd.randrange(3)), rnd.random()) for _ in range(n)]
        Yr = [rnd.random() * 10 for _ in range(n)]
        min_leaf = rnd.choice([1, 2])
        root = tuning.grow_regression_tree(Xr, Yr, [True] * 3, min_leaf=min_leaf, max_depth=1)
        sse = lambda ys: sum((y - sum(ys) / len(ys)) ** 2 for y in ys) if ys else 0.0
        cuts = {}
        for j in range(3):
            vals = sorted(set(x[j] for x in Xr))
            for a, b in zip(vals, vals[1:]):
                thr = (a + b) / 2.0
                left = [y for x, y in zip(Xr, Yr) if x[j] <= thr]
                right = [y for x, y in zip(Xr, Yr) if x[j] > thr]
                if len(left) >= min_leaf and len(right) >= min_leaf:
                    cuts[(j, thr)] = sse(left) + sse(right)
        if not cuts:
            assert root[0] == "leaf"
        else:
            # (two cuts that part the tuples the same way tie: either is the minimum)
            assert root[0] == "node" and cuts[(root[1], root[2])] <= min(cuts.values()) * (1 + 1e-12)
            assert root[3][0] == "leaf" and root[4][0] == "leaf"
            side = [y for x, y in zip(Xr, Yr) if x[root[1]] <= root[2]]
            assert abs(root[3][1] - sum(side) / len(side)) < 1e-12


def test_regression_tree_and_forest_against_a_library_cart():
    """scikit-learn's DecisionTreeRegressor is an independent implementation of CART with the same
    conventions (squared error, midpoint thresholds, x <= threshold goes left; it holds the inputs
    in float32, so the data here is float32-exact).  Where no two cuts tie it must predict what the
    oracle's trees predict: continuous random data, and leaves of three or more tuples or shallow
    trees (two inputs order a handful of tuples the same way too often, and CART does not say which
    of two equally good cuts to take).  The forest is checked as the mean of library trees grown on
    the same bootstrap rows and columns."""
    np = pytest.importorskip("numpy")
    sk = pytest.importorskip("sklearn.tree")
    rng = np.random.default_rng(17)
    X = rng.random((70, 4)).astype(np.float32).astype(np.float64)
    y = np.sin(3 * X[:, 0]) + X[:, 1] ** 2 + 0.1 * rng.random(70)
    Q = rng.random((200, 4)).astype(np.float32).astype(np.float64)
    for min_leaf, max_depth, tie_free in [(3, 64, True), (1, 3, True), (2, 3, True), (4, 6, True), (5, 64, True),
                                          (8, 2, True), (1, 64, False), (2, 5, False)]:
        mine = tuning.grow_regression_tree(X.tolist(), y.tolist(), [True] * 4, min_leaf, max_depth)
        ref = sk.DecisionTreeRegressor(min_samples_leaf=min_leaf, max_depth=min(max_depth, 60)).fit(X, y)
        # the training tuples are parted the same way whichever of two tied cuts is taken
        got = np.array([tuning.predict_regression_tree(mine, q) for q in X.tolist()])
        assert np.max(np.abs(got - ref.predict(X))) < 1e-12
        if tie_free:
            got = np.array([tuning.predict_regression_tree(mine, q) for q in Q.tolist()])
            assert np.max(np.abs(got - ref.predict(Q))) < 1e-12
    n_trees = 7
    bootstrap = rng.integers(0, 70, size=(n_trees, 70))
    masks = np.array([[True, True, False, True], [True, False, True, True], [False, True, True, True],
                      [True, True, True, False], [True, True, True, True], [True, False, False, True],
                      [False, True, True, False]])
    forest = tuning.grow_forest(X.tolist(), y.tolist(), bootstrap.tolist(), masks.tolist(), 5, 4)
    expect = np.zeros(len(Q))
    for rows, mask in zip(bootstrap, masks):
        t = sk.DecisionTreeRegressor(min_samples_leaf=5, max_depth=4).fit(X[rows][:, mask], y[rows])
        expect += t.predict(Q[:, mask])
    got = np.array([tuning.predict_forest(forest, q) for q in Q.tolist()])
    assert np.max(np.abs(got - expect / n_trees)) < 1e-12
    # a forest of identical full samples with every input open is the single tree
    same = tuning.grow_forest(X.tolist(), y.tolist(), [list(range(70))] * 3, [[True] * 4] * 3)
    one = tuning.grow_regression_tree(X.tolist(), y.tolist(), [True] * 4)
    assert all(abs(tuning.predict_forest(same, q) - tuning.predict_regression_tree(one, q)) < 1e-15 for q in Q.tolist())

"""Host-side definitions around the workgroup-size sweep (TEST INFRASTRUCTURE ONLY).

Written from the paper's definitions, in plain Python, one function per definition:
legality (Section 3.1, Eq. 1-2), oracle workgroup size (Section 4.1, Eq. 3), the evaluation
metrics `performance` and `speedup` (Section 7), the fallback handlers of Algorithm 1 and a
nearest-neighbour classifier standing in for `classify(f(s))`.

A workgroup size is a pair (w_r, w_c).  Eq. 1's comparison `w < W_max(s)` is read on the
number of work-items, non-strictly: w_r * w_c <= W_max(s).
"""
from __future__ import annotations

import math
from typing import Dict, Iterable, List, Optional, Sequence, Tuple

WG = Tuple[int, int]


# ---- enumeration (Section 5) ------------------------------------------------------------

def enumerate_sizes(mode: str, max_threads: int) -> List[WG]:
    """All (w_r, w_c) with w_r * w_c <= max_threads, both drawn from
    "pow2": {1, 2, 4, ...};  "even": {2, 4, ..., 64} (multiples of two)."""
    if mode == "pow2":
        vals = [1 << k for k in range(0, 32) if (1 << k) <= max_threads]
    elif mode == "even":
        vals = [2 * k for k in range(1, 33)]
    else:
        raise ValueError(mode)
    out = []
    for r in vals:
        for c in vals:
            if r * c <= max_threads:
                out.append((r, c))
    return out


# ---- legality (Section 3.1) ---------------------------------------------------------------

def tile_elements(w: WG, halo: Sequence[int]) -> int:
    """Elements of the local-memory tile of Section 2: the workgroup plus its perimeter
    border region, (w_r + north + south) * (w_c + east + west)."""
    n, s, e, we = halo
    return (w[0] + n + s) * (w[1] + e + we)


def is_legal(w: WG, w_max: int, refused: Iterable[WG] = ()) -> bool:
    """Eq. 1: w in W_legal(s) iff it satisfies the size constraint and is not refused."""
    wr, wc = w
    if wr < 1 or wc < 1:
        return False
    if wr * wc > w_max:
        return False
    return (wr, wc) not in set(refused)


def legal_set(candidates: Iterable[WG], w_max: int, refused: Iterable[WG] = ()) -> List[WG]:
    ref = set(refused)
    return [w for w in candidates if is_legal(w, w_max, ref)]


def safe_set(legal_sets: Sequence[Iterable[WG]]) -> List[WG]:
    """Eq. 2: sizes legal for every scenario."""
    sets = [set(s) for s in legal_sets]
    if not sets:
        return []
    common = set.intersection(*sets)
    return sorted(common)


# ---- sweep reductions (Eq. 3 and Section 7 metrics) ---------------------------------------

def oracle_size(sizes: Sequence[WG], mean_ms: Sequence[float], ok: Sequence[bool]) -> int:
    """Eq. 3: index of the legal size with the lowest mean runtime.  Ties: fewer work-items,
    then smaller w_r, then first in the list.  -1 when nothing is legal."""
    best = -1
    for i, (w, t, good) in enumerate(zip(sizes, mean_ms, ok)):
        if not good or t is None or math.isnan(t):
            continue
        if best < 0:
            best = i
            continue
        tb, wb = mean_ms[best], sizes[best]
        key_i = (t, w[0] * w[1], w[0])
        key_b = (tb, wb[0] * wb[1], wb[0])
        if key_i < key_b:
            best = i
    return best


def performance(mean_ms: Sequence[float], ok: Sequence[bool], best: int) -> List[float]:
    """p(s, w) = t(s, Omega(s)) / t(s, w), in (0, 1]; NaN for refused sizes."""
    out = []
    for t, good in zip(mean_ms, ok):
        out.append(mean_ms[best] / t if (good and best >= 0) else float("nan"))
    return out


def speedup(t_fixed: float, t_w: float) -> float:
    """Speedup of size w over a fixed size: t(s, fixed) / t(s, w)."""
    return t_fixed / t_w


def sweep_reduce(sizes: Sequence[WG], mean_ms: Sequence[float], ok: Sequence[bool],
                 fixed: WG, fixed_ms: Optional[float] = None) -> Dict[str, object]:
    """What a sweep reports: the oracle size, its speedup over the fixed size (NaN if the
    fixed size was refused) and the oracle/worst ratio."""
    best = oracle_size(sizes, mean_ms, ok)
    t_fixed = fixed_ms
    if t_fixed is None:
        for w, t, good in zip(sizes, mean_ms, ok):
            if tuple(w) == tuple(fixed) and good:
                t_fixed = t
    res = {"best_index": best, "speedup_over_fixed": float("nan"), "best_over_worst": float("nan")}
    if best >= 0:
        if t_fixed is not None and not math.isnan(t_fixed):
            res["speedup_over_fixed"] = speedup(t_fixed, mean_ms[best])
        worst = max(t for t, good in zip(mean_ms, ok) if good)
        res["best_over_worst"] = worst / mean_ms[best]
    return res


def baseline_size(perf_by_scenario: Sequence[Dict[WG, float]], safe: Sequence[WG]) -> Optional[WG]:
    """Algorithm 1, Baseline handler: the safe size with the highest geometric mean of
    p(s, w) over the training scenarios."""
    best_w, best_g = None, -1.0
    for w in safe:
        logs = [math.log(p[w]) for p in perf_by_scenario]
        g = math.exp(sum(logs) / len(logs))
        if g > best_g:
            best_w, best_g = w, g
    return best_w


# ---- Algorithm 1: classification with the NearestNeighbour fallback ------------------------

def nearest_legal(w: WG, candidates: Sequence[WG]) -> Optional[WG]:
    """The candidate with the lowest Euclidean distance to w (first one wins ties, as the
    strict `d < d_min` of Algorithm 1 implies)."""
    d_min, closest = math.inf, None
    for c in candidates:
        d = math.sqrt((c[0] - w[0]) ** 2 + (c[1] - w[1]) ** 2)
        if d < d_min:
            d_min, closest = d, c
    return closest


def predict_nearest_neighbour(predicted: WG, candidates: Sequence[WG], w_max: int,
                              refused: Iterable[WG] = ()) -> Optional[WG]:
    """Algorithm 1, NearestNeighbour: keep the classifier's size if legal, else move to the
    closest size that satisfies the constraints and is not known to be refused."""
    ref = set(refused)
    w = tuple(predicted)
    pool = [c for c in candidates if c[0] >= 1 and c[1] >= 1 and c[0] * c[1] <= w_max and c not in ref]
    while not is_legal(w, w_max, ref):
        if not pool:
            return None
        w = nearest_legal(w, pool)
    return w


def predict_baseline(predicted: WG, baseline: WG, w_max: int, refused: Iterable[WG] = ()) -> Optional[WG]:
    """Algorithm 1, Baseline: keep a legal prediction, else fall back to the baseline size."""
    ref = set(refused)
    if is_legal(tuple(predicted), w_max, ref):
        return tuple(predicted)
    return tuple(baseline) if is_legal(tuple(baseline), w_max, ref) else None


def predict_random(predicted: WG, candidates: Sequence[WG], w_max: int, refused: Iterable[WG], random: int) -> Optional[WG]:
    """Algorithm 1, Random: keep a legal prediction, else a random size among those expected to be
    legal; the draw is passed in (`random` modulo the number of legal candidates, in list order)."""
    ref = set(refused)
    if is_legal(tuple(predicted), w_max, ref):
        return tuple(predicted)
    pool = [c for c in candidates if is_legal(c, w_max, ref)]
    return pool[random % len(pool)] if pool else None


def classify_1nn(train_x: Sequence[Sequence[float]], train_w: Sequence[WG],
                 x: Sequence[float]) -> WG:
    """classify(f(s)): label of the nearest training scenario.  Each feature is scaled by its
    range over the training set (a constant feature carries no distance); Euclidean metric;
    the first nearest wins ties."""
    nf = len(x)
    lo = [min(row[j] for row in train_x) for j in range(nf)]
    hi = [max(row[j] for row in train_x) for j in range(nf)]
    best, d_best = -1, math.inf
    for i, row in enumerate(train_x):
        d = 0.0
        for j in range(nf):
            span = hi[j] - lo[j]
            if span > 0.0:
                z = (row[j] - x[j]) / span
                d += z * z
        if d < d_best:
            best, d_best = i, d
    return tuple(train_w[best])


# ---- decision tree and ZeroR classifiers ---------------------------------------------------------

def _label_counts(labels: Sequence[WG]):
    """(label, count) in order of first appearance."""
    out: List[List] = []
    for w in labels:
        for entry in out:
            if entry[0] == w:
                entry[1] += 1
                break
        else:
            out.append([w, 1])
    return out


def _entropy(labels: Sequence[WG]) -> float:
    h = 0.0
    for _, c in _label_counts(labels):
        p = c / len(labels)
        h -= p * math.log2(p)
    return h


def _majority(labels: Sequence[WG]) -> WG:
    counts = _label_counts(labels)
    best = counts[0]
    for entry in counts[1:]:
        if entry[1] > best[1]:
            best = entry
    return best[0]


def classify_zeror(train_w: Sequence[WG]) -> WG:
    """The dummy classifier of Section 7: the most frequent training label (first among equals)."""
    return _majority([tuple(w) for w in train_w])


def grow_tree(train_x: Sequence[Sequence[float]], train_w: Sequence[WG]):
    """Decision tree in the manner of the paper's J48 classifier: binary splits `x[j] <= t` chosen
    by information gain, t over the midpoints between consecutive distinct values of feature j;
    features in order, thresholds ascending, the first best split wins; grown until a node is
    pure or no split gains.  Returns nested tuples: ("leaf", label) or ("split", j, t, left, right)."""
    labels = [tuple(w) for w in train_w]

    def grow(idx):
        here = [labels[i] for i in idx]
        h = _entropy(here)
        if h <= 0:
            return ("leaf", _majority(here))
        best = None
        best_gain = 0.0
        for j in range(len(train_x[0])):
            vals = sorted({train_x[i][j] for i in idx})
            for a, b in zip(vals, vals[1:]):
                t = 0.5 * (a + b)
                left = [i for i in idx if train_x[i][j] <= t]
                right = [i for i in idx if not train_x[i][j] <= t]
                n = float(len(idx))
                gain = h - (len(left) / n) * _entropy([labels[i] for i in left]) \
                         - (len(right) / n) * _entropy([labels[i] for i in right])
                if gain > best_gain:
                    best_gain, best = gain, (j, t, left, right)
        if best is None:
            return ("leaf", _majority(here))
        j, t, left, right = best
        return ("split", j, t, grow(left), grow(right))

    return grow(list(range(len(labels))))


def classify_tree(tree, x: Sequence[float]) -> WG:
    while tree[0] == "split":
        _, j, t, left, right = tree
        tree = left if x[j] <= t else right
    return tree[1]


# ---- Algorithm 2: classification by regression --------------------------------------------------

def regress_1nn(train_x: Sequence[Sequence[float]], train_w: Sequence[WG], train_y: Sequence[float],
                x: Sequence[float], w: WG) -> float:
    """R(f(s), w): the y of the training tuple with the same w whose scenario is nearest to x
    (features scaled by their range over all tuples; first nearest wins ties); NaN if none has w."""
    nf = len(x)
    lo = [min(row[j] for row in train_x) for j in range(nf)]
    hi = [max(row[j] for row in train_x) for j in range(nf)]
    best_y, d_best = float("nan"), math.inf
    for row, wi, y in zip(train_x, train_w, train_y):
        if tuple(wi) != tuple(w):
            continue
        d = 0.0
        for j in range(nf):
            span = hi[j] - lo[j]
            if span > 0.0:
                z = (row[j] - x[j]) / span
                d += z * z
        if d < d_best:
            d_best, best_y = d, y
    return best_y


# Regression trees and their bagged ensemble (Section 5: "a Random Forest with regression trees";
# the trees are CART regression trees, the forest averages trees grown on bootstrap samples, each
# with a random subset of the inputs).  The random draws are arguments: `bootstrap[t]` lists the
# tuple indices tree t is grown on (with repetition), `masks[t][j]` says whether input j is open
# to tree t.

def grow_regression_tree(xs: Sequence[Sequence[float]], ys: Sequence[float], mask: Sequence[bool],
                         min_leaf: int = 1, max_depth: int = 64):
    """CART: a node splits on the (input, threshold) pair that minimises the summed squared error
    of the two sides' means, thresholds midway between consecutive distinct values, each side
    keeping at least `min_leaf` tuples; x <= threshold goes left.  Among equal scores the first
    input, then the lowest threshold, is kept.  A node is a leaf when its targets are all equal, no split is admissible
    or `max_depth` is reached; it predicts the mean of its targets."""
    nf = len(xs[0])

    def build(idx, depth):
        ysub = [ys[i] for i in idx]
        mean = sum(ysub) / len(ysub)
        if depth >= max_depth or len(idx) < 2 * min_leaf or min(ysub) == max(ysub):
            return ("leaf", mean)
        best = None            # (score, input, threshold)
        for j in range(nf):
            if not mask[j]:
                continue
            order = sorted(idx, key=lambda i: xs[i][j])        # stable: ties keep index order
            total = sum(ys[i] for i in order)
            left_sum = 0.0
            for pos in range(len(order) - 1):
                left_sum += ys[order[pos]]
                a, b = xs[order[pos]][j], xs[order[pos + 1]][j]
                n_l, n_r = pos + 1, len(order) - pos - 1
                if a == b or n_l < min_leaf or n_r < min_leaf:
                    continue
                right_sum = total - left_sum
                # minimising SSE = maximising sum_l^2 / n_l + sum_r^2 / n_r
                score = left_sum * left_sum / n_l + right_sum * right_sum / n_r
                if best is None or score > best[0]:
                    best = (score, j, (a + b) / 2.0)
        if best is None:
            return ("leaf", mean)
        _, j, thr = best
        left = [i for i in idx if xs[i][j] <= thr]
        right = [i for i in idx if xs[i][j] > thr]
        return ("node", j, thr, build(left, depth + 1), build(right, depth + 1))

    return build(list(range(len(xs))), 0)


def predict_regression_tree(tree, x: Sequence[float]) -> float:
    while tree[0] == "node":
        _, j, thr, left, right = tree
        tree = left if x[j] <= thr else right
    return tree[1]


def grow_forest(xs: Sequence[Sequence[float]], ys: Sequence[float], bootstrap: Sequence[Sequence[int]],
                masks: Sequence[Sequence[bool]], min_leaf: int = 1, max_depth: int = 64):
    """One CART tree per bootstrap sample, each restricted to its own subset of the inputs."""
    forest = []
    for rows, mask in zip(bootstrap, masks):
        forest.append(grow_regression_tree([xs[i] for i in rows], [ys[i] for i in rows], mask, min_leaf, max_depth))
    return forest


def predict_forest(forest, x: Sequence[float]) -> float:
    """The mean of the trees' predictions."""
    return sum(predict_regression_tree(t, x) for t in forest) / len(forest)


def predict_by_regression(predict, candidates: Sequence[WG], w_max: int, refused: Iterable[WG],
                          fitness) -> Tuple[Optional[WG], int]:
    """Algorithm 2.  `predict(w)` is R(f(s), w) for the scenario at hand, `fitness` the function
    Delta (reciprocal for runtimes, identity for speedups).  Candidates are the sizes within
    W_max; the best one by fitness is returned unless it is a refused parameter, in which case it
    is struck from the pool and the next best taken.  Returns (size, number struck)."""
    ref = set(refused)
    pool = []
    for c in candidates:
        if c[0] >= 1 and c[1] >= 1 and c[0] * c[1] <= w_max:
            y = predict(c)
            if not math.isnan(y):
                pool.append((c, fitness(y)))
    struck = 0
    while pool:
        best = 0
        for i in range(1, len(pool)):
            if pool[i][1] > pool[best][1]:
                best = i
        w = pool[best][0]
        if w not in ref:
            return w, struck
        struck += 1
        del pool[best]
    return None, struck

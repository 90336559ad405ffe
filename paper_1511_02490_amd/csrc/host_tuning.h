// Host-side arithmetic around the workgroup-size sweep: the enumeration of Section 5, the
// oracle size of Eq. 3, the performance / speedup metrics of Section 7, sample statistics, the
// classifiers behind classify(f(s)) in Algorithm 1 (nearest neighbour, decision tree, ZeroR) and
// the regressors behind R(f(s), w) in Algorithm 2 (nearest neighbour, random forest).
#pragma once
#include <algorithm>
#include <cmath>
#include <limits>
#include <vector>

namespace host_tuning {

// The values w_r and w_c are drawn from.  mode 0: powers of two up to max_threads;
// mode 1: multiples of two, 2..64.
inline bool size_values(int mode, int max_threads, std::vector<int> &vals) {
    vals.clear();
    if (mode == 0) {
        for (long long v = 1; v <= max_threads; v *= 2) vals.push_back((int)v);
        return true;
    }
    if (mode == 1) {
        for (int v = 2; v <= 64; v += 2) vals.push_back(v);
        return true;
    }
    return false;
}

struct SampleStats {
    double mean, min, median, stddev;
};

inline SampleStats summarise(std::vector<double> s) {
    SampleStats r{0, 0, 0, 0};
    const size_t n = s.size();
    if (n == 0) return r;
    double sum = 0;
    for (double x : s) sum += x;
    r.mean = sum / (double)n;
    std::sort(s.begin(), s.end());
    r.min = s.front();
    r.median = (n % 2) ? s[n / 2] : 0.5 * (s[n / 2 - 1] + s[n / 2]);
    double ss = 0;
    for (double x : s) ss += (x - r.mean) * (x - r.mean);
    r.stddev = n > 1 ? std::sqrt(ss / (double)(n - 1)) : 0.0;
    return r;
}

// Eq. 3 and the metrics of Section 7.  status[i] == 0 marks a legal, measured size.
inline void reduce(const int *wr, const int *wc, int n, const double *mean_ms, const int *status,
                   double fixed_ms, int *best_index, double *performance, double *speedup) {
    int best = -1;
    for (int i = 0; i < n; ++i) {
        if (status[i] != 0 || std::isnan(mean_ms[i])) continue;
        if (best < 0) {
            best = i;
            continue;
        }
        const long long ti = (long long)wr[i] * wc[i], tb = (long long)wr[best] * wc[best];
        bool better = mean_ms[i] < mean_ms[best];
        if (mean_ms[i] == mean_ms[best]) better = ti < tb || (ti == tb && wr[i] < wr[best]);
        if (better) best = i;
    }
    const double nan = std::numeric_limits<double>::quiet_NaN();
    if (best_index) *best_index = best;
    if (performance)
        for (int i = 0; i < n; ++i)
            performance[i] = (best >= 0 && status[i] == 0) ? mean_ms[best] / mean_ms[i] : nan;
    if (speedup) *speedup = (best >= 0 && !std::isnan(fixed_ms)) ? fixed_ms / mean_ms[best] : nan;
}

// Algorithm 1's Baseline handler: among the sizes legal for every scenario (W_safe, Eq. 2), the
// one with the highest geometric mean of p(s, w).  perf is n_scen x n_sizes, row-major, NaN
// where a size is not legal for a scenario.  Returns -1 if no size is safe.
inline int baseline_index(const double *perf, int n_scen, int n_sizes) {
    int best = -1;
    double best_log = 0;
    for (int j = 0; j < n_sizes; ++j) {
        double sum_log = 0;
        bool safe = n_scen > 0;
        for (int i = 0; i < n_scen && safe; ++i) {
            const double p = perf[(size_t)i * n_sizes + j];
            if (std::isnan(p) || p <= 0) safe = false; else sum_log += std::log(p);
        }
        if (safe && (best < 0 || sum_log > best_log)) {
            best = j;
            best_log = sum_log;
        }
    }
    return best;
}

// classify(f(s)) of Algorithm 1 over (f(s), Omega(s)) training pairs, three ways:
//   kNearest - the label of the nearest training scenario (each feature scaled by its range
//              over the training set, Euclidean distance, first nearest wins ties);
//   kTree    - a decision tree in the manner of the paper's J48: binary splits `feature <=
//              threshold` chosen by information gain over the midpoints between consecutive
//              distinct values (features in order, thresholds ascending, first best wins), grown
//              until a node is pure or nothing gains; a leaf answers with its most frequent
//              label (the one seen first among equals);
//   kZeroR   - always the most frequent label of the training set (the paper's dummy classifier).
class Classifier {
public:
    enum Kind { kNearest = 0, kTree = 1, kZeroR = 2 };
    explicit Classifier(int kind) : kind_(kind) {}

    bool add(const double *f, int nf, int wr, int wc) {
        if (nf_ == 0) nf_ = nf;
        if (nf != nf_) return false;
        x_.insert(x_.end(), f, f + nf);
        wr_.push_back(wr);
        wc_.push_back(wc);
        built_ = false;
        return true;
    }

    bool classify(const double *f, int nf, int *wr, int *wc) const {
        const size_t n = wr_.size();
        if (n == 0 || nf != nf_) return false;
        size_t pick = 0;
        if (kind_ == kNearest) {
            pick = nearest(f);
        } else {
            if (!built_) build();
            int node = 0;
            while (kind_ == kTree && nodes_[node].feature >= 0)
                node = f[nodes_[node].feature] <= nodes_[node].threshold ? nodes_[node].left : nodes_[node].right;
            pick = (size_t)nodes_[node].label_of;
        }
        *wr = wr_[pick];
        *wc = wc_[pick];
        return true;
    }

private:
    struct Node {
        int feature;        // -1: leaf
        double threshold;
        int left, right;
        int label_of;       // a training pair carrying the leaf's label
    };

    size_t nearest(const double *f) const {
        const size_t n = wr_.size();
        std::vector<double> lo(nf_), hi(nf_);
        for (int j = 0; j < nf_; ++j) {
            lo[j] = hi[j] = x_[j];
            for (size_t i = 1; i < n; ++i) {
                lo[j] = std::min(lo[j], x_[i * nf_ + j]);
                hi[j] = std::max(hi[j], x_[i * nf_ + j]);
            }
        }
        size_t best = 0;
        double d_best = std::numeric_limits<double>::infinity();
        for (size_t i = 0; i < n; ++i) {
            double d = 0;
            for (int j = 0; j < nf_; ++j) {
                const double span = hi[j] - lo[j];
                if (span > 0) {
                    const double z = (x_[i * nf_ + j] - f[j]) / span;
                    d += z * z;
                }
            }
            if (d < d_best) {
                d_best = d;
                best = i;
            }
        }
        return best;
    }

    bool same_label(int a, int b) const { return wr_[a] == wr_[b] && wc_[a] == wc_[b]; }

    // label counts of a set of training pairs, labels in order of first appearance
    void count(const std::vector<int> &idx, std::vector<int> &first, std::vector<int> &cnt) const {
        first.clear();
        cnt.clear();
        for (int i : idx) {
            size_t c = 0;
            while (c < first.size() && !same_label(first[c], i)) ++c;
            if (c == first.size()) {
                first.push_back(i);
                cnt.push_back(0);
            }
            ++cnt[c];
        }
    }

    double entropy(const std::vector<int> &idx) const {
        std::vector<int> first, cnt;
        count(idx, first, cnt);
        double h = 0;
        for (int c : cnt) {
            const double p = (double)c / (double)idx.size();
            h -= p * std::log2(p);
        }
        return h;
    }

    int majority(const std::vector<int> &idx) const {
        std::vector<int> first, cnt;
        count(idx, first, cnt);
        size_t best = 0;
        for (size_t c = 1; c < cnt.size(); ++c)
            if (cnt[c] > cnt[best]) best = c;
        return first[best];
    }

    int grow(const std::vector<int> &idx) const {
        const int me = (int)nodes_.size();
        nodes_.push_back(Node{-1, 0.0, -1, -1, majority(idx)});
        if (kind_ != kTree) return me;
        const double h = entropy(idx);
        if (h <= 0) return me;
        double best_gain = 0;
        int best_f = -1;
        double best_t = 0;
        std::vector<int> l, r;
        for (int j = 0; j < nf_; ++j) {
            std::vector<double> vals;
            for (int i : idx) vals.push_back(x_[(size_t)i * nf_ + j]);
            std::sort(vals.begin(), vals.end());
            vals.erase(std::unique(vals.begin(), vals.end()), vals.end());
            for (size_t k = 0; k + 1 < vals.size(); ++k) {
                const double t = 0.5 * (vals[k] + vals[k + 1]);
                l.clear();
                r.clear();
                for (int i : idx) (x_[(size_t)i * nf_ + j] <= t ? l : r).push_back(i);
                const double n = (double)idx.size();
                const double gain = h - ((double)l.size() / n) * entropy(l) - ((double)r.size() / n) * entropy(r);
                if (gain > best_gain) {
                    best_gain = gain;
                    best_f = j;
                    best_t = t;
                }
            }
        }
        if (best_f < 0) return me;
        l.clear();
        r.clear();
        for (int i : idx) (x_[(size_t)i * nf_ + best_f] <= best_t ? l : r).push_back(i);
        const int left = grow(l);
        const int right = grow(r);
        nodes_[me].feature = best_f;
        nodes_[me].threshold = best_t;
        nodes_[me].left = left;
        nodes_[me].right = right;
        return me;
    }

    void build() const {
        nodes_.clear();
        std::vector<int> all(wr_.size());
        for (size_t i = 0; i < all.size(); ++i) all[i] = (int)i;
        grow(all);
        built_ = true;
    }

    int kind_;
    int nf_ = 0;
    std::vector<double> x_;
    std::vector<int> wr_, wc_;
    mutable std::vector<Node> nodes_;
    mutable bool built_ = false;
};

// R(f(s), w) of Algorithm 2 over (f(s), w, y) tuples.  Without a fitted forest: the y of the
// tuple with the same w whose scenario is nearest to f (features scaled by their range over all
// tuples, Euclidean distance, first nearest wins ties); NaN if no tuple has this w.  With one (Section 5: a random forest of regression trees):
// the mean of CART trees over the inputs (f(s), w_r, w_c), each grown on its own bootstrap sample
// with its own subset of the inputs; the random draws are the caller's.
class Regressor {
public:
    bool add(const double *f, int nf, int wr, int wc, double y) {
        if (nf_ == 0) nf_ = nf;
        if (nf != nf_) return false;
        x_.insert(x_.end(), f, f + nf);
        wr_.push_back(wr);
        wc_.push_back(wc);
        y_.push_back(y);
        trees_.clear();     // a forest describes the tuples it was grown on
        return true;
    }
    int n_features() const { return nf_; }
    size_t n_tuples() const { return y_.size(); }
    int n_inputs() const { return nf_ + 2; }
    bool has_forest() const { return !trees_.empty(); }

    // bootstrap: n_trees x n_rows tuple indices (NULL: every tree sees every tuple once);
    // masks: n_trees x n_inputs() flags (NULL: every input open).  False on a bad index or a tree
    // with no open input.
    bool fit_forest(int n_trees, int n_rows, const int *bootstrap, const unsigned char *masks, int min_leaf,
                    int max_depth) {
        const int n = (int)y_.size(), ni = n_inputs();
        if (n_trees < 1 || n < 1 || min_leaf < 1 || max_depth < 0) return false;
        if (bootstrap && n_rows < 1) return false;
        std::vector<Tree> trees((size_t)n_trees);
        for (int t = 0; t < n_trees; ++t) {
            std::vector<int> rows;
            if (bootstrap) {
                rows.assign(bootstrap + (size_t)t * n_rows, bootstrap + (size_t)(t + 1) * n_rows);
                for (int r : rows)
                    if (r < 0 || r >= n) return false;
            } else {
                rows.resize((size_t)n);
                for (int i = 0; i < n; ++i) rows[(size_t)i] = i;
            }
            std::vector<unsigned char> open((size_t)ni, 1);
            if (masks) open.assign(masks + (size_t)t * ni, masks + (size_t)(t + 1) * ni);
            bool any = false;
            for (unsigned char o : open) any = any || o;
            if (!any) return false;
            std::vector<std::vector<int>> sorted((size_t)ni);
            for (int j = 0; j < ni; ++j) {
                if (!open[(size_t)j]) continue;
                sorted[(size_t)j] = rows;
                std::stable_sort(sorted[(size_t)j].begin(), sorted[(size_t)j].end(),
                                 [&](int a, int b) { return input(a, j) < input(b, j); });
            }
            grow(trees[(size_t)t], rows, sorted, open, min_leaf, max_depth, 0);
        }
        trees_.swap(trees);
        return true;
    }

    double predict(const double *f, int wr, int wc) const {
        if (!trees_.empty()) {
            double sum = 0.0;
            for (const Tree &t : trees_) {
                int k = 0;
                while (t[(size_t)k].input >= 0) {
                    const Node &nd = t[(size_t)k];
                    const double v = nd.input < nf_ ? f[nd.input] : (nd.input == nf_ ? (double)wr : (double)wc);
                    k = v <= nd.threshold ? nd.left : nd.right;
                }
                sum += t[(size_t)k].value;
            }
            return sum / (double)trees_.size();
        }
        const size_t n = y_.size();
        std::vector<double> lo(nf_), hi(nf_);
        for (int j = 0; j < nf_; ++j) {
            lo[j] = hi[j] = n ? x_[j] : 0.0;
            for (size_t i = 1; i < n; ++i) {
                lo[j] = std::min(lo[j], x_[i * nf_ + j]);
                hi[j] = std::max(hi[j], x_[i * nf_ + j]);
            }
        }
        double best_y = std::numeric_limits<double>::quiet_NaN();
        double d_best = std::numeric_limits<double>::infinity();
        for (size_t i = 0; i < n; ++i) {
            if (wr_[i] != wr || wc_[i] != wc) continue;
            double d = 0;
            for (int j = 0; j < nf_; ++j) {
                const double span = hi[j] - lo[j];
                if (span > 0) {
                    const double z = (x_[i * nf_ + j] - f[j]) / span;
                    d += z * z;
                }
            }
            if (d < d_best) {
                d_best = d;
                best_y = y_[i];
            }
        }
        return best_y;
    }

private:
    struct Node {
        int input = -1;         // -1: leaf
        double threshold = 0.0;
        int left = -1, right = -1;
        double value = 0.0;     // leaf: mean of the targets
    };
    using Tree = std::vector<Node>;

    double input(int tuple, int j) const {
        return j < nf_ ? x_[(size_t)tuple * nf_ + j] : (j == nf_ ? (double)wr_[(size_t)tuple] : (double)wc_[(size_t)tuple]);
    }

    // CART: the cut that minimises the two sides' summed squared error (= maximises
    // sum_l^2 / n_l + sum_r^2 / n_r), thresholds midway between consecutive distinct values,
    // at least min_leaf tuples a side, x <= threshold to the left; first best cut kept.
    // `rows` are the node's tuples in the order they were drawn; `sorted[j]` holds the same tuples
    // ordered by input j (equal values in drawing order) for every open input - sorted once per
    // tree and split stably from node to node, which is what sorting each node afresh would give.
    int grow(Tree &tree, const std::vector<int> &rows, const std::vector<std::vector<int>> &sorted,
             const std::vector<unsigned char> &open, int min_leaf, int max_depth, int depth) const {
        const int me = (int)tree.size();
        tree.push_back(Node());
        double sum = 0.0, lo = y_[(size_t)rows[0]], hi = lo;
        for (int r : rows) {
            sum += y_[(size_t)r];
            lo = std::min(lo, y_[(size_t)r]);
            hi = std::max(hi, y_[(size_t)r]);
        }
        tree[(size_t)me].value = sum / (double)rows.size();
        if (depth >= max_depth || (int)rows.size() < 2 * min_leaf || lo == hi) return me;
        bool found = false;
        double best_score = 0.0, best_thr = 0.0;
        int best_input = -1;
        for (int j = 0; j < n_inputs(); ++j) {
            if (!open[(size_t)j]) continue;
            const std::vector<int> &order = sorted[(size_t)j];
            double total = 0.0;
            for (int r : order) total += y_[(size_t)r];
            double left_sum = 0.0;
            for (size_t pos = 0; pos + 1 < order.size(); ++pos) {
                left_sum += y_[(size_t)order[pos]];
                const double a = input(order[pos], j), b = input(order[pos + 1], j);
                const double n_l = (double)(pos + 1), n_r = (double)(order.size() - pos - 1);
                if (a == b || (int)(pos + 1) < min_leaf || (int)(order.size() - pos - 1) < min_leaf) continue;
                const double right_sum = total - left_sum;
                const double score = left_sum * left_sum / n_l + right_sum * right_sum / n_r;
                if (!found || score > best_score) {
                    found = true;
                    best_score = score;
                    best_input = j;
                    best_thr = (a + b) / 2.0;
                }
            }
        }
        if (!found) return me;
        auto goes_left = [&](int r) { return input(r, best_input) <= best_thr; };
        std::vector<int> left, right;
        for (int r : rows) (goes_left(r) ? left : right).push_back(r);
        std::vector<std::vector<int>> sorted_l(sorted.size()), sorted_r(sorted.size());
        for (size_t j = 0; j < sorted.size(); ++j)
            for (int r : sorted[j]) (goes_left(r) ? sorted_l[j] : sorted_r[j]).push_back(r);
        tree[(size_t)me].input = best_input;
        tree[(size_t)me].threshold = best_thr;
        const int l = grow(tree, left, sorted_l, open, min_leaf, max_depth, depth + 1);
        const int r = grow(tree, right, sorted_r, open, min_leaf, max_depth, depth + 1);
        tree[(size_t)me].left = l;
        tree[(size_t)me].right = r;
        return me;
    }

    int nf_ = 0;
    std::vector<double> x_, y_;
    std::vector<int> wr_, wc_;
    std::vector<Tree> trees_;
};

}  // namespace host_tuning

// Offline tuner, host only (paper Sections II-A, III, III-A, IV): normalise a timing table,
// prune the family with a leaf-limited multi-output regression tree, score the kept set,
// fit the decision-tree selector and score it.  Plain C++; deterministic.
//
// Both trees are CART over integer features.  A candidate split "x[f] <= t" uses
// t = floor(midpoint) of two consecutive distinct values.  With per-row target vectors y_s
// (normalised performance for the regression tree, weighted one-hot labels for the Gini
// classifier) and row weights w_s, the impurity a split removes is
//     gain = |S_L|^2 / W_L + |S_R|^2 / W_R - |S|^2 / W,     S = sum_s w_s y_s,  W = sum_s w_s
// which is the drop in summed squared error, and for one-hot targets the drop in n * Gini.
#include "../../include/ks_gemm.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <numeric>
#include <limits>
#include <vector>

namespace {

constexpr double kRelEps = 1e-9;   // a candidate must beat the incumbent by this relative margin
constexpr double kMinGain = 1e-12;

inline bool better(double gain, double best) { return gain > best + kRelEps * std::fabs(best); }

struct Split {
    bool ok = false;
    double gain = 0.0;
    int feature = -1;
    int64_t threshold = 0;
};

struct Table {
    const int64_t *X;
    int nf;
    const double *Y;      // rows x cols targets
    int cols;
    const double *w;      // per-row weight or nullptr
};

double weight_of(const Table &t, int row) { return t.w ? t.w[row] : 1.0; }

Split best_split(const Table &t, const std::vector<int> &rows, int minLeaf) {
    Split best;
    const int n = (int)rows.size();
    if (n < 2 * minLeaf || n < 2) return best;
    std::vector<double> tot(t.cols, 0.0), left(t.cols);
    double W = 0.0;
    for (int r : rows) {
        const double w = weight_of(t, r);
        W += w;
        for (int c = 0; c < t.cols; ++c) tot[c] += w * t.Y[(size_t)r * t.cols + c];
    }
    if (!(W > 0.0)) return best;
    double base = 0.0;
    for (int c = 0; c < t.cols; ++c) base += tot[c] * tot[c];
    base /= W;
    std::vector<int> order(rows);
    for (int f = 0; f < t.nf; ++f) {
        std::stable_sort(order.begin(), order.end(), [&](int a, int b) {
            const int64_t xa = t.X[(size_t)a * t.nf + f], xb = t.X[(size_t)b * t.nf + f];
            return xa != xb ? xa < xb : a < b;
        });
        std::fill(left.begin(), left.end(), 0.0);
        double WL = 0.0;
        for (int i = 0; i + 1 < n; ++i) {
            const int r = order[i];
            const double w = weight_of(t, r);
            WL += w;
            for (int c = 0; c < t.cols; ++c) left[c] += w * t.Y[(size_t)r * t.cols + c];
            const int64_t xa = t.X[(size_t)r * t.nf + f], xb = t.X[(size_t)order[i + 1] * t.nf + f];
            if (xa == xb) continue;
            if (i + 1 < minLeaf || n - (i + 1) < minLeaf) continue;
            const double WR = W - WL;
            if (!(WL > 0.0) || !(WR > 0.0)) continue;
            double sl = 0.0, sr = 0.0;
            for (int c = 0; c < t.cols; ++c) {
                const double l = left[c], r2 = tot[c] - left[c];
                sl += l * l;
                sr += r2 * r2;
            }
            const double gain = sl / WL + sr / WR - base;
            if (gain <= kMinGain) continue;
            if (!best.ok || better(gain, best.gain)) {
                best.ok = true;
                best.gain = gain;
                best.feature = f;
                // floor of the midpoint, also for negative values
                const int64_t sum = xa + xb;
                best.threshold = sum >= 0 ? sum / 2 : -((-sum + 1) / 2);
            }
        }
    }
    return best;
}

void partition(const Table &t, const std::vector<int> &rows, const Split &s, std::vector<int> &l,
               std::vector<int> &r) {
    for (int row : rows) (t.X[(size_t)row * t.nf + s.feature] <= s.threshold ? l : r).push_back(row);
}

int argmax_mean(const Table &t, const std::vector<int> &rows) {
    int best = 0;
    double bestV = -1.0;
    for (int c = 0; c < t.cols; ++c) {
        double s = 0.0;
        for (int r : rows) s += t.Y[(size_t)r * t.cols + c];
        s /= (double)rows.size();
        if (s > bestV) { bestV = s; best = c; }
    }
    return best;
}

struct Grow {
    const Table &t;
    const std::vector<int> &label;     // class index per row
    const std::vector<int32_t> &classId;
    int maxDepth, minLeaf, cap;
    std::vector<ks_tree_node_t> nodes;
    bool overflow = false;

    int grow(const std::vector<int> &rows, int depth) {
        if ((int)nodes.size() >= cap) { overflow = true; return -1; }
        const int me = (int)nodes.size();
        nodes.push_back(ks_tree_node_t{-1, -1, -1, 0, 0});
        // majority by weight, lowest kernel id on ties (classId is ascending)
        std::vector<double> mass(classId.size(), 0.0);
        bool pure = true;
        for (int r : rows) {
            mass[label[r]] += weight_of(t, r);
            pure = pure && label[r] == label[rows[0]];
        }
        int top = 0;
        for (size_t k = 1; k < mass.size(); ++k) if (mass[k] > mass[top]) top = (int)k;
        nodes[me].value = classId[top];
        if (pure || depth >= maxDepth) return me;
        const Split s = best_split(t, rows, minLeaf);
        if (!s.ok) return me;
        std::vector<int> l, r;
        partition(t, rows, s, l, r);
        const int li = grow(l, depth + 1);
        const int ri = overflow ? -1 : grow(r, depth + 1);
        if (overflow) return me;
        nodes[me].feature = s.feature;
        nodes[me].threshold = s.threshold;
        nodes[me].left = li;
        nodes[me].right = ri;
        return me;
    }
};

}  // namespace

extern "C" int ks_tune_performance(const int64_t *sizes, const double *seconds, int rows, int cols, double *out) {
    if (!sizes || !seconds || !out || rows < 0 || cols <= 0) return KS_ERR_INVALID_ARG;
    for (int s = 0; s < rows; ++s) {
        const int64_t *z = sizes + (size_t)s * 4;
        if (z[0] < 0 || z[1] < 0 || z[2] < 0 || z[3] < 0) return KS_ERR_INVALID_ARG;
        const double flops = 2.0 * (double)z[0] * (double)z[1] * (double)z[2] * (double)z[3];
        for (int c = 0; c < cols; ++c) {
            const double t = seconds[(size_t)s * cols + c];
            if (!(t > 0.0)) return KS_ERR_INVALID_ARG;
            out[(size_t)s * cols + c] = flops / t;
        }
    }
    return KS_OK;
}

extern "C" int ks_tune_normalise(const double *perf, int rows, int cols, double *out) {
    if (!perf || !out || rows < 0 || cols <= 0) return KS_ERR_INVALID_ARG;
    for (int s = 0; s < rows; ++s) {
        double m = perf[(size_t)s * cols];
        for (int c = 1; c < cols; ++c) m = std::max(m, perf[(size_t)s * cols + c]);
        if (!(m > 0.0)) return KS_ERR_INVALID_ARG;
        for (int c = 0; c < cols; ++c) out[(size_t)s * cols + c] = perf[(size_t)s * cols + c] / m;
    }
    return KS_OK;
}

extern "C" int ks_tune_prune_tree(const int64_t *features, int n_features, const double *normalised,
                                  int rows, int cols, int max_leaves, int min_samples_leaf,
                                  int32_t *kept_out, ks_tree_node_t *tree_out, int *tree_nodes_out) {
    if (!features || !normalised || !kept_out || rows <= 0 || cols <= 0 || n_features <= 0 ||
        max_leaves < 1 || min_samples_leaf < 1)
        return KS_ERR_INVALID_ARG;
    const Table t{features, n_features, normalised, cols, nullptr};
    struct Node {
        std::vector<int> rows;
        Split split;
        int feature = -1, left = -1, right = -1;
        int64_t threshold = 0;
    };
    std::vector<Node> nodes(1);
    nodes[0].rows.resize(rows);
    std::iota(nodes[0].rows.begin(), nodes[0].rows.end(), 0);
    nodes[0].split = best_split(t, nodes[0].rows, min_samples_leaf);
    int leaves = 1;
    while (leaves < max_leaves) {
        int pick = -1;
        for (int i = 0; i < (int)nodes.size(); ++i) {
            if (nodes[i].feature != -1 || !nodes[i].split.ok) continue;
            if (pick < 0 || better(nodes[i].split.gain, nodes[pick].split.gain)) pick = i;
        }
        if (pick < 0) break;
        Node l, r;
        partition(t, nodes[pick].rows, nodes[pick].split, l.rows, r.rows);
        l.split = best_split(t, l.rows, min_samples_leaf);
        r.split = best_split(t, r.rows, min_samples_leaf);
        nodes[pick].feature = nodes[pick].split.feature;
        nodes[pick].threshold = nodes[pick].split.threshold;
        nodes[pick].left = (int)nodes.size();
        nodes[pick].right = (int)nodes.size() + 1;
        nodes.push_back(std::move(l));
        nodes.push_back(std::move(r));
        ++leaves;
    }
    std::vector<int32_t> kept;
    for (size_t i = 0; i < nodes.size(); ++i) {
        int value = 0;
        if (nodes[i].feature == -1) {
            value = argmax_mean(t, nodes[i].rows);
            kept.push_back(value);
        }
        if (tree_out)
            tree_out[i] = ks_tree_node_t{nodes[i].feature, nodes[i].left, nodes[i].right, value,
                                         nodes[i].threshold};
    }
    if (tree_nodes_out) *tree_nodes_out = (int)nodes.size();
    std::sort(kept.begin(), kept.end());
    kept.erase(std::unique(kept.begin(), kept.end()), kept.end());
    std::copy(kept.begin(), kept.end(), kept_out);
    return (int)kept.size();
}

extern "C" int ks_tune_achievable(const double *normalised, int rows, int cols, const int32_t *kept,
                                  int n_kept, double *score_out) {
    if (!normalised || !kept || !score_out || rows <= 0 || cols <= 0 || n_kept <= 0)
        return KS_ERR_INVALID_ARG;
    for (int k = 0; k < n_kept; ++k) if (kept[k] < 0 || kept[k] >= cols) return KS_ERR_INVALID_ARG;
    double logSum = 0.0;
    for (int s = 0; s < rows; ++s) {
        double m = 0.0;
        for (int k = 0; k < n_kept; ++k) m = std::max(m, normalised[(size_t)s * cols + kept[k]]);
        logSum += std::log(m);
    }
    *score_out = std::exp(logSum / rows);
    return KS_OK;
}

extern "C" int ks_tune_fit_selector(const int64_t *features, int n_features, const double *perf,
                                    int rows, int cols, const int32_t *kept, int n_kept, int max_depth,
                                    int min_samples_leaf, const double *row_weight,
                                    ks_tree_node_t *tree_out, int cap) {
    if (!features || !perf || !kept || !tree_out || rows <= 0 || cols <= 0 || n_features <= 0 ||
        n_kept <= 0 || max_depth < 0 || min_samples_leaf < 1 || cap < 1)
        return KS_ERR_INVALID_ARG;
    std::vector<int32_t> classId(kept, kept + n_kept);
    std::sort(classId.begin(), classId.end());
    classId.erase(std::unique(classId.begin(), classId.end()), classId.end());
    for (int32_t c : classId) if (c < 0 || c >= cols) return KS_ERR_INVALID_ARG;
    const int nc = (int)classId.size();
    // label = fastest kept configuration of the row (lowest id on ties); targets = one-hot labels
    std::vector<int> label(rows);
    std::vector<double> onehot((size_t)rows * nc, 0.0);
    for (int s = 0; s < rows; ++s) {
        int best = 0;
        for (int k = 1; k < nc; ++k)
            if (perf[(size_t)s * cols + classId[k]] > perf[(size_t)s * cols + classId[best]]) best = k;
        label[s] = best;
        onehot[(size_t)s * nc + best] = 1.0;
        if (row_weight && !(row_weight[s] >= 0.0)) return KS_ERR_INVALID_ARG;
    }
    const Table t{features, n_features, onehot.data(), nc, row_weight};
    Grow g{t, label, classId, max_depth, min_samples_leaf, cap, {}, false};
    std::vector<int> all(rows);
    std::iota(all.begin(), all.end(), 0);
    g.grow(all, 0);
    if (g.overflow) return KS_ERR_INVALID_ARG;
    std::copy(g.nodes.begin(), g.nodes.end(), tree_out);
    return (int)g.nodes.size();
}

extern "C" int ks_tune_predict(const ks_tree_node_t *tree, int n_nodes, const int64_t *features,
                               int n_features, int rows, int32_t *chosen_out) {
    if (!tree || !features || !chosen_out || n_nodes <= 0 || rows < 0 || n_features <= 0)
        return KS_ERR_INVALID_ARG;
    for (int s = 0; s < rows; ++s) {
        int i = 0, steps = 0;
        while (tree[i].feature >= 0) {
            if (tree[i].feature >= n_features || ++steps > n_nodes) return KS_ERR_INVALID_ARG;
            const int next = features[(size_t)s * n_features + tree[i].feature] <= tree[i].threshold
                                 ? tree[i].left : tree[i].right;
            if (next <= i || next >= n_nodes) return KS_ERR_INVALID_ARG;
            i = next;
        }
        chosen_out[s] = tree[i].value;
    }
    return KS_OK;
}

extern "C" int ks_tune_selector_score(const double *normalised, int rows, int cols,
                                      const int32_t *chosen, double *score_out) {
    if (!normalised || !chosen || !score_out || rows <= 0 || cols <= 0) return KS_ERR_INVALID_ARG;
    double logSum = 0.0;
    for (int s = 0; s < rows; ++s) {
        if (chosen[s] < 0 || chosen[s] >= cols) return KS_ERR_INVALID_ARG;
        logSum += std::log(normalised[(size_t)s * cols + chosen[s]]);
    }
    *score_out = std::exp(logSum / rows);
    return KS_OK;
}

// ------------------------------------------------------------------------------------------------
// The paper's other pruning methods (Section III) and the PCA variance spectrum (Section II-B).
// k-means is Lloyd's algorithm with deterministic maximin seeding (first centre: the row nearest
// to the mean of all rows; each further centre: the row farthest from its nearest centre so far;
// lowest row on ties).  A centre that loses all its rows stays where it is.
namespace {

double dist2(const double *a, const double *b, int d) {
    double s = 0.0;
    for (int j = 0; j < d; ++j) {
        const double t = a[j] - b[j];
        s += t * t;
    }
    return s;
}

// Z: rows x d.  centres: k x d (k <= rows).  Returns the assignment of every row.
std::vector<int> lloyd(const std::vector<double> &Z, int rows, int d, int k, int maxIter,
                       std::vector<double> &centres) {
    std::vector<double> mean(d, 0.0);
    for (int s = 0; s < rows; ++s)
        for (int j = 0; j < d; ++j) mean[j] += Z[(size_t)s * d + j];
    for (int j = 0; j < d; ++j) mean[j] /= rows;
    int first = 0;
    double best = dist2(&Z[0], mean.data(), d);
    for (int s = 1; s < rows; ++s) {
        const double v = dist2(&Z[(size_t)s * d], mean.data(), d);
        if (v < best) { best = v; first = s; }
    }
    std::vector<int> seeds{first};
    std::vector<double> nearest(rows);
    for (int s = 0; s < rows; ++s) nearest[s] = dist2(&Z[(size_t)s * d], &Z[(size_t)first * d], d);
    while ((int)seeds.size() < k) {
        int far = 0;
        for (int s = 1; s < rows; ++s) if (nearest[s] > nearest[far]) far = s;
        seeds.push_back(far);
        for (int s = 0; s < rows; ++s)
            nearest[s] = std::min(nearest[s], dist2(&Z[(size_t)s * d], &Z[(size_t)far * d], d));
    }
    centres.assign((size_t)k * d, 0.0);
    for (int c = 0; c < k; ++c)
        std::copy(&Z[(size_t)seeds[c] * d], &Z[(size_t)seeds[c] * d] + d, &centres[(size_t)c * d]);
    std::vector<int> assign(rows, -1);
    std::vector<double> sum((size_t)k * d);
    std::vector<int> count(k);
    for (int it = 0; it < maxIter; ++it) {
        bool changed = false;
        for (int s = 0; s < rows; ++s) {
            int arg = 0;
            double bd = dist2(&Z[(size_t)s * d], &centres[0], d);
            for (int c = 1; c < k; ++c) {
                const double v = dist2(&Z[(size_t)s * d], &centres[(size_t)c * d], d);
                if (v < bd) { bd = v; arg = c; }
            }
            if (arg != assign[s]) { assign[s] = arg; changed = true; }
        }
        if (!changed) break;
        std::fill(sum.begin(), sum.end(), 0.0);
        std::fill(count.begin(), count.end(), 0);
        for (int s = 0; s < rows; ++s) {
            ++count[assign[s]];
            for (int j = 0; j < d; ++j) sum[(size_t)assign[s] * d + j] += Z[(size_t)s * d + j];
        }
        for (int c = 0; c < k; ++c)
            if (count[c] > 0)
                for (int j = 0; j < d; ++j) centres[(size_t)c * d + j] = sum[(size_t)c * d + j] / count[c];
    }
    return assign;
}

// Eigen-decomposition of the covariance of the rows by cyclic Jacobi rotations.
// w: eigenvalues descending; V: cols x cols, eigenvector i in column i.
void covariance_eigen(const double *X, int rows, int cols, std::vector<double> &mean,
                      std::vector<double> &w, std::vector<double> &V) {
    mean.assign(cols, 0.0);
    for (int s = 0; s < rows; ++s)
        for (int j = 0; j < cols; ++j) mean[j] += X[(size_t)s * cols + j];
    for (int j = 0; j < cols; ++j) mean[j] /= rows;
    std::vector<double> A((size_t)cols * cols, 0.0);
    for (int s = 0; s < rows; ++s)
        for (int i = 0; i < cols; ++i) {
            const double xi = X[(size_t)s * cols + i] - mean[i];
            for (int j = i; j < cols; ++j) A[(size_t)i * cols + j] += xi * (X[(size_t)s * cols + j] - mean[j]);
        }
    const double denom = rows > 1 ? rows - 1 : 1;
    for (int i = 0; i < cols; ++i)
        for (int j = i; j < cols; ++j) A[(size_t)j * cols + i] = A[(size_t)i * cols + j] /= denom;
    V.assign((size_t)cols * cols, 0.0);
    for (int i = 0; i < cols; ++i) V[(size_t)i * cols + i] = 1.0;
    for (int sweep = 0; sweep < 100; ++sweep) {
        double off = 0.0, diag = 0.0;
        for (int i = 0; i < cols; ++i) {
            diag += A[(size_t)i * cols + i] * A[(size_t)i * cols + i];
            for (int j = i + 1; j < cols; ++j) off += A[(size_t)i * cols + j] * A[(size_t)i * cols + j];
        }
        if (off <= 1e-30 * (diag + off) || off == 0.0) break;
        for (int p = 0; p < cols; ++p)
            for (int q = p + 1; q < cols; ++q) {
                const double apq = A[(size_t)p * cols + q];
                if (apq == 0.0) continue;
                const double theta = (A[(size_t)q * cols + q] - A[(size_t)p * cols + p]) / (2.0 * apq);
                const double t = (theta >= 0 ? 1.0 : -1.0) / (std::fabs(theta) + std::sqrt(theta * theta + 1.0));
                const double c = 1.0 / std::sqrt(t * t + 1.0), sn = t * c;
                for (int k = 0; k < cols; ++k) {
                    const double akp = A[(size_t)k * cols + p], akq = A[(size_t)k * cols + q];
                    A[(size_t)k * cols + p] = c * akp - sn * akq;
                    A[(size_t)k * cols + q] = sn * akp + c * akq;
                }
                for (int k = 0; k < cols; ++k) {
                    const double apk = A[(size_t)p * cols + k], aqk = A[(size_t)q * cols + k];
                    A[(size_t)p * cols + k] = c * apk - sn * aqk;
                    A[(size_t)q * cols + k] = sn * apk + c * aqk;
                }
                for (int k = 0; k < cols; ++k) {
                    const double vkp = V[(size_t)k * cols + p], vkq = V[(size_t)k * cols + q];
                    V[(size_t)k * cols + p] = c * vkp - sn * vkq;
                    V[(size_t)k * cols + q] = sn * vkp + c * vkq;
                }
            }
    }
    std::vector<int> order(cols);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(),
                     [&](int a, int b) { return A[(size_t)a * cols + a] > A[(size_t)b * cols + b]; });
    w.resize(cols);
    std::vector<double> Vs((size_t)cols * cols);
    for (int i = 0; i < cols; ++i) {
        w[i] = std::max(A[(size_t)order[i] * cols + order[i]], 0.0);
        for (int k = 0; k < cols; ++k) Vs[(size_t)k * cols + i] = V[(size_t)k * cols + order[i]];
    }
    V.swap(Vs);
}

int keep_argmax_rows(const std::vector<double> &reps, int k, int cols, int32_t *kept_out) {
    std::vector<int32_t> kept;
    for (int c = 0; c < k; ++c) {
        int best = 0;
        for (int j = 1; j < cols; ++j)
            if (reps[(size_t)c * cols + j] > reps[(size_t)c * cols + best]) best = j;
        kept.push_back(best);
    }
    std::sort(kept.begin(), kept.end());
    kept.erase(std::unique(kept.begin(), kept.end()), kept.end());
    std::copy(kept.begin(), kept.end(), kept_out);
    return (int)kept.size();
}

}  // namespace

extern "C" int ks_tune_prune_top_n(const double *normalised, int rows, int cols, int n,
                                   int32_t *kept_out) {
    if (!normalised || !kept_out || rows <= 0 || cols <= 0 || n < 1) return KS_ERR_INVALID_ARG;
    std::vector<int> wins(cols, 0);
    for (int s = 0; s < rows; ++s) {
        int best = 0;
        for (int c = 1; c < cols; ++c)
            if (normalised[(size_t)s * cols + c] > normalised[(size_t)s * cols + best]) best = c;
        ++wins[best];
    }
    std::vector<int> order(cols);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return wins[a] > wins[b]; });
    std::vector<int32_t> kept;
    for (int i = 0; i < cols && (int)kept.size() < n; ++i)
        if (wins[order[i]] > 0) kept.push_back(order[i]);
    std::sort(kept.begin(), kept.end());
    std::copy(kept.begin(), kept.end(), kept_out);
    return (int)kept.size();
}

extern "C" int ks_tune_prune_kmeans(const double *normalised, int rows, int cols, int n, int pca_dims,
                                    int max_iter, int32_t *kept_out) {
    if (!normalised || !kept_out || rows <= 0 || cols <= 0 || n < 1 || pca_dims < 0 || pca_dims > cols ||
        max_iter < 1)
        return KS_ERR_INVALID_ARG;
    const int k = std::min(n, rows);
    std::vector<double> centres;
    if (pca_dims == 0) {
        std::vector<double> Z(normalised, normalised + (size_t)rows * cols);
        lloyd(Z, rows, cols, k, max_iter, centres);
        return keep_argmax_rows(centres, k, cols, kept_out);
    }
    std::vector<double> mean, w, V;
    covariance_eigen(normalised, rows, cols, mean, w, V);
    const int d = pca_dims;
    std::vector<double> Z((size_t)rows * d, 0.0);
    for (int s = 0; s < rows; ++s)
        for (int i = 0; i < d; ++i) {
            double acc = 0.0;
            for (int j = 0; j < cols; ++j) acc += (normalised[(size_t)s * cols + j] - mean[j]) * V[(size_t)j * cols + i];
            Z[(size_t)s * d + i] = acc;
        }
    lloyd(Z, rows, d, k, max_iter, centres);
    std::vector<double> back((size_t)k * cols);
    for (int c = 0; c < k; ++c)
        for (int j = 0; j < cols; ++j) {
            double acc = mean[j];
            for (int i = 0; i < d; ++i) acc += centres[(size_t)c * d + i] * V[(size_t)j * cols + i];
            back[(size_t)c * cols + j] = acc;
        }
    return keep_argmax_rows(back, k, cols, kept_out);
}

// ---------------------------------------------------------------- HDBSCAN (Section III)
// Density-based clustering of the rows (Campello, Moulavi, Sander 2013; McInnes, Healy, Astels
// 2017): core distances, mutual reachability, minimum spanning tree, single-linkage hierarchy,
// condensed tree, excess-of-mass selection.  The number of clusters is a result, not a parameter.
namespace {

struct CondensedCluster {
    int parent = -1;
    double birth = 0.0;
    double stability = 0.0;
    std::vector<int> children;
    std::vector<int> fellPoints;          // rows that left this cluster as single points
    bool selected = false;
};

constexpr double kHdbscanDmin = 1e-12;

// labels[i] = cluster of row i (numbered by first member row) or -1; returns the cluster count
int hdbscan_cluster(const double *Z, int n, int d, int minClusterSize, int minSamples, std::vector<int> &labels) {
    labels.assign((size_t)n, -1);
    if (n < 2) return 0;
    const int k = std::min(std::max(minSamples, 1), n);
    std::vector<double> D((size_t)n * n);
    for (int i = 0; i < n; ++i)
        for (int j = i; j < n; ++j) {
            double acc = 0.0;
            for (int c = 0; c < d; ++c) {
                const double t = Z[(size_t)i * d + c] - Z[(size_t)j * d + c];
                acc += t * t;
            }
            D[(size_t)i * n + j] = D[(size_t)j * n + i] = std::sqrt(acc);
        }
    std::vector<double> core((size_t)n), row((size_t)n);
    for (int i = 0; i < n; ++i) {
        std::copy(D.begin() + (size_t)i * n, D.begin() + (size_t)(i + 1) * n, row.begin());
        std::nth_element(row.begin(), row.begin() + (k - 1), row.end());
        core[i] = row[k - 1];
    }
    // minimum spanning tree under the mutual reachability distance (Prim from row 0)
    struct Edge { double w; int a, b, order; };
    std::vector<Edge> edges;
    std::vector<char> inTree((size_t)n, 0);
    std::vector<double> key((size_t)n, std::numeric_limits<double>::infinity());
    std::vector<int> from((size_t)n, -1);
    key[0] = 0.0;
    for (int step = 0; step < n; ++step) {
        int v = -1;
        for (int i = 0; i < n; ++i)
            if (!inTree[i] && (v < 0 || key[i] < key[v])) v = i;
        inTree[v] = 1;
        if (from[v] >= 0) edges.push_back(Edge{key[v], from[v], v, (int)edges.size()});
        for (int i = 0; i < n; ++i) {
            if (inTree[i]) continue;
            const double w = std::max(std::max(core[v], core[i]), D[(size_t)v * n + i]);
            if (w < key[i]) { key[i] = w; from[i] = v; }
        }
    }
    std::sort(edges.begin(), edges.end(), [](const Edge &x, const Edge &y) {
        return x.w != y.w ? x.w < y.w : x.order < y.order;
    });
    // single-linkage hierarchy: nodes 0 .. n-1 are rows, n .. 2n-2 merges
    const int total = 2 * n - 1;
    std::vector<int> left((size_t)total, -1), right((size_t)total, -1), size((size_t)total, 1), uf((size_t)n), nodeOf((size_t)n);
    std::vector<double> dist((size_t)total, 0.0);
    for (int i = 0; i < n; ++i) { uf[i] = i; nodeOf[i] = i; }
    auto find = [&](int x) {
        while (uf[x] != x) { uf[x] = uf[uf[x]]; x = uf[x]; }
        return x;
    };
    int next = n;
    for (const Edge &e : edges) {
        const int ra = find(e.a), rb = find(e.b);
        const int na = nodeOf[ra], nb = nodeOf[rb];
        left[next] = na; right[next] = nb; dist[next] = e.w; size[next] = size[na] + size[nb];
        uf[rb] = ra;
        nodeOf[ra] = next++;
    }
    const int root = next - 1;
    auto collect = [&](int node, std::vector<int> &out) {
        std::vector<int> stack{node};
        while (!stack.empty()) {
            const int y = stack.back();
            stack.pop_back();
            if (y < n) out.push_back(y);
            else { stack.push_back(left[y]); stack.push_back(right[y]); }
        }
    };
    // condensed tree, breadth first from the root; cluster 0 is the root cluster
    std::vector<CondensedCluster> cl(1);
    std::vector<double> fellLambdaSum(1, 0.0);       // sum over leaving points / child clusters of lambda_leave
    std::vector<double> leaveCount(1, 0.0);
    std::vector<std::pair<int, int>> queue{{root, 0}};
    for (size_t head = 0; head < queue.size(); ++head) {
        const int node = queue[head].first, c = queue[head].second;
        if (node < n) { cl[c].fellPoints.push_back(node); continue; }
        const double lam = 1.0 / std::max(dist[node], kHdbscanDmin);
        const int sides[2] = {left[node], right[node]};
        const bool big[2] = {size[sides[0]] >= minClusterSize, size[sides[1]] >= minClusterSize};
        if (big[0] && big[1]) {
            for (int t = 0; t < 2; ++t) {
                const int id = (int)cl.size();
                cl.emplace_back();
                fellLambdaSum.push_back(0.0);
                leaveCount.push_back(0.0);
                cl[id].parent = c;
                cl[id].birth = lam;
                cl[c].children.push_back(id);
                fellLambdaSum[c] += lam * size[sides[t]];
                leaveCount[c] += size[sides[t]];
                queue.push_back({sides[t], id});
            }
        } else {
            for (int t = 0; t < 2; ++t) {
                if (big[t]) { queue.push_back({sides[t], c}); continue; }
                std::vector<int> pts;
                collect(sides[t], pts);
                for (int p : pts) cl[c].fellPoints.push_back(p);
                fellLambdaSum[c] += lam * (double)pts.size();
                leaveCount[c] += (double)pts.size();
            }
        }
    }
    const int nc = (int)cl.size();
    for (int c = 0; c < nc; ++c) cl[c].stability = fellLambdaSum[c] - cl[c].birth * leaveCount[c];
    // excess of mass, children before parents (children have larger ids)
    std::vector<double> best((size_t)nc);
    for (int c = nc - 1; c >= 0; --c) {
        best[c] = cl[c].stability;
        if (cl[c].children.empty()) { cl[c].selected = c != 0; continue; }
        double below = 0.0;
        for (int ch : cl[c].children) below += best[ch];
        if (c == 0 || cl[c].stability < below) {
            best[c] = below;
        } else {
            cl[c].selected = true;
            std::vector<int> todo(cl[c].children);
            while (!todo.empty()) {
                const int x = todo.back();
                todo.pop_back();
                cl[x].selected = false;
                for (int ch : cl[x].children) todo.push_back(ch);
            }
        }
    }
    std::vector<int> raw((size_t)n, -1);
    for (int c = 0; c < nc; ++c) {
        int a = c;
        while (a != -1 && !cl[a].selected) a = cl[a].parent;
        if (a == -1) continue;
        for (int p : cl[c].fellPoints) raw[p] = a;
    }
    std::vector<int> remap((size_t)nc, -1);
    int count = 0;
    for (int i = 0; i < n; ++i)
        if (raw[i] >= 0) {
            if (remap[raw[i]] < 0) remap[raw[i]] = count++;
            labels[i] = remap[raw[i]];
        }
    return count;
}

}  // namespace

extern "C" int ks_tune_prune_hdbscan(const double *normalised, int rows, int cols, int min_cluster_size,
                                     int min_samples, int32_t *kept_out, int kept_cap, int32_t *labels_out) {
    if (!normalised || !kept_out || rows <= 0 || cols <= 0 || min_cluster_size < 2 || min_samples < 1 || kept_cap < 1)
        return KS_ERR_INVALID_ARG;
    if ((double)rows * rows * sizeof(double) > 4e9) return KS_ERR_UNSUPPORTED;
    std::vector<int> labels;
    const int count = hdbscan_cluster(normalised, rows, cols, min_cluster_size, min_samples, labels);
    if (labels_out)
        for (int i = 0; i < rows; ++i) labels_out[i] = labels[i];
    std::vector<char> keep((size_t)cols, 0);
    auto best_of_mean = [&](int cluster) {
        std::vector<double> mean((size_t)cols, 0.0);
        int members = 0;
        for (int i = 0; i < rows; ++i)
            if (cluster < 0 || labels[i] == cluster) {
                ++members;
                for (int c = 0; c < cols; ++c) mean[c] += normalised[(size_t)i * cols + c];
            }
        int arg = 0;
        for (int c = 1; c < cols; ++c)
            if (mean[c] / members > mean[arg] / members) arg = c;
        return arg;
    };
    if (count == 0) keep[best_of_mean(-1)] = 1;
    for (int k = 0; k < count; ++k) keep[best_of_mean(k)] = 1;
    int n = 0;
    for (int c = 0; c < cols; ++c)
        if (keep[c]) {
            if (n >= kept_cap) return KS_ERR_INVALID_ARG;
            kept_out[n++] = c;
        }
    return n;
}

extern "C" int ks_tune_pca_variance(const double *normalised, int rows, int cols, double *ratio_out) {
    if (!normalised || !ratio_out || rows <= 0 || cols <= 0) return KS_ERR_INVALID_ARG;
    std::vector<double> mean, w, V;
    covariance_eigen(normalised, rows, cols, mean, w, V);
    double total = 0.0;
    for (double v : w) total += v;
    if (!(total > 0.0)) return KS_ERR_INVALID_ARG;
    for (int i = 0; i < cols; ++i) ratio_out[i] = w[i] / total;
    return KS_OK;
}

"""CPU oracle of the prune-and-select pipeline (paper Sections II-A, III, III-A, IV).

TEST INFRASTRUCTURE ONLY; numpy, float64, written for reading rather than speed.
It shares no code with the library's own trainer (C++) and never imports it.

Notation: rows s are workloads (a set of matrix sizes and layout flags), columns c
are kernel configurations.
    P[s][c]      measured performance (flop/s) of configuration c on workload s
    Phat[s][c]   P normalised to the row's best:  Phat = P / max_c P   (Section II-A:
                 performance as a fraction of the optimal for that workload)
    S            the kept set of configurations after pruning (Section III)

Pruning by decision-tree regression (Section III, last method): a multi-output
regression tree maps the integer features of a workload to the vector Phat[s][.];
it is limited to a fixed number of leaves, each leaf's mean vector is one cluster
representative, and the configuration that is best for a representative is kept.
The deployed selector (Section IV) is a decision-tree classifier over the kept
set, whose label for a training row is the kept configuration that is fastest
there.  Scores (Section III-A and Table I) are geometric means over test rows.

Readings where the paper is silent:
  * trees are CART: axis-aligned splits "x[f] <= t" go left; candidate thresholds
    are floor(midpoint) of consecutive distinct integer feature values, so the
    deployed selector compares integers only;
  * regression impurity is the squared error summed over all outputs; the tree
    with a leaf limit is grown best-first (always split the leaf whose best split
    removes the most squared error);
  * the classifier uses Gini impurity, grown depth-first until pure, a depth cap,
    or no split helps;
  * ties: argmax takes the lowest index; a candidate split replaces the current
    best only if its gain exceeds it by more than a relative 1e-9 (so equal
    gains resolve to the lowest feature index, then the lowest threshold); equal
    best-first priorities resolve to the leaf created first;
  * a split must remove more than 1e-12 of impurity to be made at all.
"""
import numpy as np

GAIN_REL_EPS = 1e-9
GAIN_MIN = 1e-12


# ----------------------------------------------------------------- table and scores

def performance(flops, seconds):
    """P[s][c] = flops[s] / seconds[s][c]."""
    return np.asarray(flops, dtype=np.float64)[:, None] / np.asarray(seconds, dtype=np.float64)


def normalise(P):
    """Phat[s][c] = P[s][c] / max_c P[s][c]; every row's best is exactly 1."""
    P = np.asarray(P, dtype=np.float64)
    return P / P.max(axis=1, keepdims=True)


def geometric_mean(v):
    v = np.asarray(v, dtype=np.float64)
    return float(np.exp(np.mean(np.log(v))))


def achievable(Phat, kept):
    """Geometric mean over rows of the best normalised performance inside the kept set."""
    kept = sorted(set(int(c) for c in kept))
    return geometric_mean(np.asarray(Phat)[:, kept].max(axis=1))


def selector_score(Phat, chosen):
    """Geometric mean over rows of the normalised performance of the chosen configuration."""
    Phat = np.asarray(Phat)
    return geometric_mean(Phat[np.arange(Phat.shape[0]), np.asarray(chosen, dtype=np.int64)])


def labels_within(P, kept):
    """For each row the kept configuration with the highest performance (lowest id on ties)."""
    kept = sorted(set(int(c) for c in kept))
    sub = np.asarray(P)[:, kept]
    return np.asarray(kept, dtype=np.int64)[np.argmax(sub, axis=1)]


# ----------------------------------------------------------------- CART pieces

def _better(gain, best):
    return gain > best + GAIN_REL_EPS * abs(best)


def _candidate_thresholds(x):
    """floor(midpoint) between consecutive distinct values of an integer feature column."""
    u = np.unique(x)
    return [int((int(a) + int(b)) // 2) for a, b in zip(u[:-1], u[1:])]


def _sse(Y):
    """Squared error around the mean, summed over rows and outputs."""
    if Y.shape[0] == 0:
        return 0.0
    return float(np.sum((Y - Y.mean(axis=0)) ** 2))


def best_regression_split(X, Y, min_samples_leaf=1):
    """Best (gain, feature, threshold) of one node, or None.  gain = SSE(node) - SSE(L) - SSE(R)."""
    parent = _sse(Y)
    best = None
    for f in range(X.shape[1]):
        for t in _candidate_thresholds(X[:, f]):
            left = X[:, f] <= t
            nl = int(left.sum())
            if nl < min_samples_leaf or Y.shape[0] - nl < min_samples_leaf:
                continue
            gain = parent - _sse(Y[left]) - _sse(Y[~left])
            if gain <= GAIN_MIN:
                continue
            if best is None or _better(gain, best[0]):
                best = (gain, f, t)
    return best


def _gini_mass(y, classes):
    """n * Gini(node) = n - sum_k count_k^2 / n."""
    n = y.shape[0]
    if n == 0:
        return 0.0
    counts = np.array([(y == k).sum() for k in classes], dtype=np.float64)
    return float(n - np.sum(counts ** 2) / n)


def best_classification_split(X, y, classes, min_samples_leaf=1):
    parent = _gini_mass(y, classes)
    best = None
    for f in range(X.shape[1]):
        for t in _candidate_thresholds(X[:, f]):
            left = X[:, f] <= t
            nl = int(left.sum())
            if nl < min_samples_leaf or y.shape[0] - nl < min_samples_leaf:
                continue
            gain = parent - _gini_mass(y[left], classes) - _gini_mass(y[~left], classes)
            if gain <= GAIN_MIN:
                continue
            if best is None or _better(gain, best[0]):
                best = (gain, f, t)
    return best


def _leaf(rows, **kw):
    d = dict(feature=-1, threshold=0, left=-1, right=-1, rows=rows)
    d.update(kw)
    return d


# ----------------------------------------------------------------- pruning tree

def fit_regression_tree(X, Y, max_leaf_nodes, min_samples_leaf=1):
    """Best-first multi-output regression tree with at most max_leaf_nodes leaves.

    Returns a list of node dicts; node 0 is the root; children are appended in the order
    (left, right) at the moment their parent is split.  Leaves carry 'value' = mean vector.
    """
    X = np.asarray(X, dtype=np.int64)
    Y = np.asarray(Y, dtype=np.float64)
    nodes = [_leaf(np.arange(X.shape[0]))]
    nodes[0]["split"] = best_regression_split(X, Y, min_samples_leaf)
    n_leaves = 1
    while n_leaves < max_leaf_nodes:
        pick = None
        for i, nd in enumerate(nodes):
            if nd["feature"] == -1 and nd.get("split") is not None:
                if pick is None or _better(nd["split"][0], nodes[pick]["split"][0]):
                    pick = i
        if pick is None:
            break
        gain, f, t = nodes[pick]["split"]
        rows = nodes[pick]["rows"]
        go_left = X[rows, f] <= t
        for child_rows in (rows[go_left], rows[~go_left]):
            child = _leaf(child_rows)
            child["split"] = best_regression_split(X[child_rows], Y[child_rows], min_samples_leaf)
            nodes.append(child)
        nodes[pick].update(feature=f, threshold=t, left=len(nodes) - 2, right=len(nodes) - 1)
        n_leaves += 1
    for nd in nodes:
        nd["value"] = Y[nd["rows"]].mean(axis=0)
    return nodes


def kept_set(tree):
    """Configurations that are best for at least one leaf representative (sorted, unique)."""
    return sorted({int(np.argmax(nd["value"])) for nd in tree if nd["feature"] == -1})


# ----------------------------------------------------------------- selector tree

def fit_classification_tree(X, y, max_depth=12, min_samples_leaf=1):
    """Depth-first Gini classification tree.  Leaves carry 'label' (majority, lowest id on ties)."""
    X = np.asarray(X, dtype=np.int64)
    y = np.asarray(y, dtype=np.int64)
    classes = sorted(set(int(v) for v in y))
    nodes = []

    def grow(rows, depth):
        me = len(nodes)
        nodes.append(_leaf(rows))
        counts = [(int((y[rows] == k).sum()), -k) for k in classes]
        nodes[me]["label"] = -max(counts)[1]
        if depth < max_depth and len(set(y[rows].tolist())) > 1:
            split = best_classification_split(X[rows], y[rows], classes, min_samples_leaf)
            if split is not None:
                _, f, t = split
                go_left = X[rows, f] <= t
                l = grow(rows[go_left], depth + 1)
                r = grow(rows[~go_left], depth + 1)
                nodes[me].update(feature=f, threshold=t, left=l, right=r)
        return me

    grow(np.arange(X.shape[0]), 0)
    return nodes


def tree_leaf(tree, x):
    """Index of the leaf a feature vector falls into."""
    i = 0
    while tree[i]["feature"] != -1:
        i = tree[i]["left"] if int(x[tree[i]["feature"]]) <= tree[i]["threshold"] else tree[i]["right"]
    return i


def predict_labels(tree, X):
    return np.array([tree[tree_leaf(tree, x)]["label"] for x in np.asarray(X)], dtype=np.int64)


# ----------------------------------------------------------------- whole pipeline

def prune_and_train(X_train, P_train, n_kept, max_depth=12, min_samples_leaf=1):
    """Steps of Sections III and IV in order: normalise, regress with a leaf limit, keep each
    leaf's best configuration, label rows inside the kept set, fit the classifier."""
    Phat = normalise(P_train)
    reg = fit_regression_tree(X_train, Phat, n_kept)
    kept = kept_set(reg)
    y = labels_within(P_train, kept)
    clf = fit_classification_tree(X_train, y, max_depth, min_samples_leaf)
    return dict(regression_tree=reg, kept=kept, labels=y, selector=clf)


def prune_and_train_by_regime(X_train, P_train, n_single, n_batched, batch_feature=3, max_depth=12,
                              min_samples_leaf=1):
    """The pipeline applied per regime (reading: the paper has one kind of workload; here single
    GEMMs, batch count 1, and batched ones differ in what wins and in how many rows describe them,
    and a pooled pruning tree of Section III spends its leaves where the rows are).  Rows with
    feature[batch_feature] <= 1 are pruned to at most n_single leaves and classified on their own,
    the others with n_batched; the deployed selector is a root "batch <= 1" whose children are the
    two classifiers, i.e. still one tree of nested integer comparisons (Section IV).
    Returns dict(kept, selector, parts) where selector is a node list in the layout of
    fit_classification_tree (node 0 the root, left subtree first)."""
    X_train, P_train = np.asarray(X_train, dtype=np.int64), np.asarray(P_train, dtype=np.float64)
    single = X_train[:, batch_feature] <= 1
    if single.all() or not single.any():
        whole = prune_and_train(X_train, P_train, n_single, max_depth, min_samples_leaf)
        return dict(kept=whole["kept"], selector=whole["selector"], parts=[whole])
    one = prune_and_train(X_train[single], P_train[single], n_single, max_depth, min_samples_leaf)
    many = prune_and_train(X_train[~single], P_train[~single], n_batched, max_depth, min_samples_leaf)
    root = _leaf(np.arange(X_train.shape[0]), label=one["selector"][0]["label"])
    root.update(feature=batch_feature, threshold=1, left=1, right=1 + len(one["selector"]))
    joined = [root]
    for offset, part in ((1, one["selector"]), (1 + len(one["selector"]), many["selector"])):
        for nd in part:
            c = dict(nd)
            if c["feature"] != -1:
                c["left"], c["right"] = c["left"] + offset, c["right"] + offset
            joined.append(c)
    return dict(kept=sorted(set(one["kept"]) | set(many["kept"])), selector=joined, parts=[one, many])


def sampled_prune_and_train(X_train, P_train, stage1_rows, n_kept, max_depth=12, min_samples_leaf=1):
    """A two-stage form of the same pipeline for a configuration space too large to time in full
    (the paper's conclusion names this as the open problem; the reading is ours): only the rows
    in `stage1_rows` (boolean mask) are timed for every configuration and decide the kept set;
    every other training row is timed for the kept configurations only.  The classifier is then
    fitted on all training rows, labelled inside the kept set.  Entries of P_train that the
    procedure never measures (non-kept columns of rows outside stage 1) are not read.
    Returns the kept set, the selector and the number of timed cells."""
    X_train, P_train = np.asarray(X_train), np.asarray(P_train, dtype=np.float64)
    m = np.asarray(stage1_rows, dtype=bool)
    reg = fit_regression_tree(X_train[m], normalise(P_train[m]), n_kept)
    kept = kept_set(reg)
    measured = np.zeros_like(P_train)
    measured[:, kept] = P_train[:, kept]
    y = labels_within(measured, kept)
    clf = fit_classification_tree(X_train, y, max_depth, min_samples_leaf)
    cells = int(m.sum()) * P_train.shape[1] + int((~m).sum()) * len(kept)
    return dict(kept=kept, selector=clf, timed_cells=cells, regression_tree=reg)


# ----------------------------------------------------------------- the other pruning methods
# Section III compares the decision tree with: the N configurations that win most often, k-means
# on the normalised performance vectors, k-means in PCA coordinates with the centroids mapped back,
# and HDBSCAN (not implemented here).  Section II-B uses the PCA variance spectrum of the same
# vectors to choose the range of N.  Readings, where the paper gives no detail:
#   * k-means is Lloyd's algorithm with a deterministic "maximin" seeding instead of a random one:
#     the first centre is the row closest to the mean of all rows, every further centre is the row
#     farthest (squared Euclidean distance) from its nearest centre so far; lowest row on ties.
#     A row goes to its nearest centre (lowest centre index on ties); a centre that loses all its
#     rows stays where it is; iteration stops when no row changes cluster (or after max_iter).
#   * the representative of a cluster is its centroid and the kept configuration its argmax;
#   * PCA is the eigen-decomposition of the covariance of the centred rows; the number of
#     components used for clustering is a parameter (compare.py takes the smallest number that
#     explains 95 % of the variance).

def prune_top_n(Phat, n):
    """The n configurations that are optimal (normalised performance 1, first on ties) most often;
    equal counts resolve to the lowest id; configurations that never win are not kept."""
    Phat = np.asarray(Phat, dtype=np.float64)
    wins = np.bincount(np.argmax(Phat, axis=1), minlength=Phat.shape[1])
    order = sorted(range(Phat.shape[1]), key=lambda c: (-wins[c], c))
    return sorted(c for c in order[:n] if wins[c] > 0)


def _maximin_seeds(Z, k):
    mean = Z.mean(axis=0)
    first = int(np.argmin(((Z - mean) ** 2).sum(axis=1)))
    seeds = [first]
    d = ((Z - Z[first]) ** 2).sum(axis=1)
    while len(seeds) < k:
        nxt = int(np.argmax(d))
        seeds.append(nxt)
        d = np.minimum(d, ((Z - Z[nxt]) ** 2).sum(axis=1))
    return seeds


def kmeans(Z, k, max_iter=100):
    """Lloyd's algorithm with maximin seeding.  Returns (centres [k x d], assignment [rows])."""
    Z = np.asarray(Z, dtype=np.float64)
    k = min(k, Z.shape[0])
    centres = Z[_maximin_seeds(Z, k)].copy()
    assign = np.full(Z.shape[0], -1)
    for _ in range(max_iter):
        d = ((Z[:, None, :] - centres[None, :, :]) ** 2).sum(axis=2)
        new = np.argmin(d, axis=1)
        if np.array_equal(new, assign):
            break
        assign = new
        for c in range(k):
            if np.any(assign == c):
                centres[c] = Z[assign == c].mean(axis=0)
    return centres, assign


def prune_kmeans(Phat, n, max_iter=100):
    centres, _ = kmeans(Phat, n, max_iter)
    return sorted({int(np.argmax(c)) for c in centres})


def pca(Phat):
    """(mean, eigenvalues descending, eigenvectors as columns) of the covariance of the rows."""
    X = np.asarray(Phat, dtype=np.float64)
    mean = X.mean(axis=0)
    cov = (X - mean).T @ (X - mean) / max(X.shape[0] - 1, 1)
    w, V = np.linalg.eigh(cov)
    order = np.argsort(-w, kind="stable")
    return mean, np.maximum(w[order], 0.0), V[:, order]


def pca_variance_ratio(Phat):
    """Fraction of the total variance carried by each principal component, descending."""
    _, w, _ = pca(Phat)
    return w / w.sum()


def components_for(ratio, fraction):
    """Smallest number of leading components whose variance fractions add up to `fraction`."""
    return int(np.searchsorted(np.cumsum(ratio), fraction - 1e-12) + 1)


def prune_pca_kmeans(Phat, n, dims, max_iter=100):
    """k-means in the coordinates of the leading `dims` principal components; each centroid is
    mapped back to configuration space (mean + coordinates . components) and its argmax kept."""
    X = np.asarray(Phat, dtype=np.float64)
    mean, _, V = pca(X)
    Vd = V[:, :dims]
    centres, _ = kmeans((X - mean) @ Vd, n, max_iter)
    back = mean + centres @ Vd.T
    return sorted({int(np.argmax(c)) for c in back})

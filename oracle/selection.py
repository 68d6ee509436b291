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


# ----------------------------------------------------------------- HDBSCAN pruning (Section III)
# The last of the clustering methods the paper compares (its Fig. 4): density-based clustering of the
# normalised performance vectors in which the number of clusters is not a parameter.  The published
# algorithm (Campello, Moulavi, Sander 2013; McInnes, Healy, Astels 2017), by its steps:
#   1. core distance of a point = distance to its min_samples-th nearest point, itself included;
#   2. mutual reachability distance d(a, b) = max(core(a), core(b), |a - b|);
#   3. minimum spanning tree of the complete graph under d (Prim from point 0; the next vertex is
#      the one with the smallest key, lowest index on ties; a key changes only if strictly smaller);
#   4. single-linkage hierarchy: edges in ascending order of weight (order of insertion on ties)
#      merge components;
#   5. condensed tree: walking down from the root with lambda = 1 / distance, a split whose two sides
#      both hold at least min_cluster_size points creates two new clusters; otherwise the points of
#      a side that is too small fall out of the cluster at that lambda and the other side carries on
#      as the same cluster;
#   6. stability of a cluster = sum over the points that leave it (falling out, or in a child
#      cluster) of lambda_leave - lambda_birth; clusters are selected bottom-up by excess of mass:
#      a cluster replaces its selected descendants if its stability is at least their sum; the root
#      is never selected;
#   7. a point belongs to the nearest selected ancestor of the cluster it fell out of, else is noise.
# Readings: distances below 1e-12 count as 1e-12 (lambda stays finite); the kept configuration of a
# cluster is the best one of its centroid, as for k-means; rows labelled noise take no part; if no
# cluster is selected the centroid of all rows is used.
HDBSCAN_DMIN = 1e-12


def hdbscan_labels(Z, min_cluster_size, min_samples=None):
    """Cluster labels (0 .. n_clusters-1 in order of first member row; -1 = noise)."""
    Z = np.asarray(Z, dtype=np.float64)
    n = Z.shape[0]
    k = min(int(min_samples if min_samples is not None else min_cluster_size), n)
    D = np.sqrt(np.maximum(((Z[:, None, :] - Z[None, :, :]) ** 2).sum(axis=2), 0.0)) if n <= 1500 else None
    if D is None:
        sq = (Z * Z).sum(axis=1)
        D = np.sqrt(np.maximum(sq[:, None] + sq[None, :] - 2.0 * Z @ Z.T, 0.0))
        np.fill_diagonal(D, 0.0)
    core = np.sort(D, axis=1)[:, k - 1]
    # Prim
    in_tree = np.zeros(n, dtype=bool)
    key = np.full(n, np.inf)
    parent = np.full(n, -1)
    key[0] = 0.0
    edges = []
    for _ in range(n):
        cand = np.where(in_tree, np.inf, key)
        v = int(np.argmin(cand))
        in_tree[v] = True
        if parent[v] >= 0:
            edges.append((float(key[v]), int(parent[v]), v))
        w = np.maximum(np.maximum(core[v], core), D[v])
        better = (~in_tree) & (w < key)
        key[better] = w[better]
        parent[better] = v
    order = sorted(range(len(edges)), key=lambda e: (edges[e][0], e))
    # single linkage: node ids n.. for merges
    comp = list(range(n))                      # union-find over points -> current dendrogram node

    def find(x):
        while comp[x] != x:
            comp[x] = comp[comp[x]]
            x = comp[x]
        return x
    node_of = list(range(n))                   # dendrogram node of each union-find root
    left, right, dist, size = {}, {}, {}, {i: 1 for i in range(n)}
    nxt = n
    for e in order:
        w, a, b = edges[e]
        ra, rb = find(a), find(b)
        na, nb = node_of[ra], node_of[rb]
        left[nxt], right[nxt], dist[nxt], size[nxt] = na, nb, w, size[na] + size[nb]
        comp[rb] = ra
        node_of[ra] = nxt
        nxt += 1
    root = nxt - 1
    if n == 1:
        return np.full(1, -1)

    def leaves(x):
        out, stack = [], [x]
        while stack:
            y = stack.pop()
            if y < n:
                out.append(y)
            else:
                stack.extend((right[y], left[y]))
        return out
    # condensed tree
    birth = {0: 0.0}
    children = {0: []}
    parent_cluster = {0: -1}
    fell = {0: []}                              # (point, lambda) leaving cluster c
    child_mass = {0: []}                        # (size, lambda) of child clusters born from c
    stack = [(root, 0)]
    n_clusters = 1
    while stack:
        node, c = stack.pop(0)
        if node < n:
            fell[c].append((node, np.inf))      # cannot happen for min_cluster_size >= 2; kept for completeness
            continue
        lam = 1.0 / max(dist[node], HDBSCAN_DMIN)
        L, R = left[node], right[node]
        bigL, bigR = size[L] >= min_cluster_size, size[R] >= min_cluster_size
        if bigL and bigR:
            for side in (L, R):
                cid = n_clusters
                n_clusters += 1
                birth[cid], children[cid], parent_cluster[cid], fell[cid], child_mass[cid] = lam, [], c, [], []
                children[c].append(cid)
                child_mass[c].append((size[side], lam))
                stack.append((side, cid))
        else:
            for side, big in ((L, bigL), (R, bigR)):
                if big:
                    stack.append((side, c))
                else:
                    fell[c].extend((p, lam) for p in leaves(side))
    stability = {c: sum(l - birth[c] for _, l in fell[c]) + sum(s * (l - birth[c]) for s, l in child_mass[c])
                 for c in birth}
    selected = {c: False for c in birth}
    best = dict(stability)
    for c in sorted(birth, reverse=True):       # children have larger ids than their parents
        if not children[c]:
            selected[c] = c != 0
            continue
        below = sum(best[ch] for ch in children[c])
        if c == 0 or stability[c] < below:
            best[c] = below
        else:
            selected[c] = True
            todo = list(children[c])
            while todo:
                d = todo.pop()
                selected[d] = False
                todo.extend(children[d])
    labels = np.full(n, -1)
    for c in birth:
        a = c
        while a != -1 and not selected[a]:
            a = parent_cluster[a]
        if a == -1:
            continue
        for p, _ in fell[c]:
            labels[p] = a
    # renumber in order of first member row
    remap = {}
    for i in range(n):
        if labels[i] >= 0 and labels[i] not in remap:
            remap[int(labels[i])] = len(remap)
    return np.array([remap[int(v)] if v >= 0 else -1 for v in labels])


def prune_hdbscan(Phat, min_cluster_size, min_samples=None):
    """Kept configurations: the best configuration of every cluster's centroid."""
    Phat = np.asarray(Phat, dtype=np.float64)
    lab = hdbscan_labels(Phat, min_cluster_size, min_samples)
    if lab.max() < 0:
        return [int(np.argmax(Phat.mean(axis=0)))], lab
    return sorted({int(np.argmax(Phat[lab == c].mean(axis=0))) for c in range(lab.max() + 1)}), lab

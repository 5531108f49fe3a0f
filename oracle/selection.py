"""CPU oracle for the selection side of MTNN.  TEST INFRASTRUCTURE ONLY.

Plain, slow, step-by-step Python/numpy versions of
  * the performance figure and the label rule (Section IV-A),
  * the selection metrics GOW / LUB and the averages of Table VII (Section V-B),
  * the feature vector handed to the classifier (Section IV-A, restricted to one GPU),
  * gradient boosted CART trees with the paper's settings (Section IV-B:
    maximum depth 8, 8 estimators, eta = 1, gamma = 0), and their evaluation
    (Algorithm 2: label +1 runs NT, label -1 runs TNN).

The product's C++ trainer and evaluator share no code with this file; the tests
compare the two.  The paper delegates boosting to a library and prints neither
the objective nor a tree, so everything beyond the four settings above follows
that library's documented defaults (binary logistic objective, initial margin
0, L2 leaf penalty lambda = 1, minimum child hessian weight 1, exact greedy
splits, no subsampling).  Exact tree parity with the paper's tool: parity
unpinned (tool absent, no tree printed); what is pinned are the split gain and
leaf value formulas on hand-computed cases and behaviour on separable data.
"""
from __future__ import annotations

import math

import numpy as np

MAX_DEPTH = 8        # Section IV-B, parameter configuration
NUM_TREES = 8
ETA = 1.0
GAMMA = 0.0
LAMBDA = 1.0         # library default (paper silent)
MIN_CHILD_WEIGHT = 1.0

FEATURE_NAMES = ("m", "n", "k", "n*k", "m*n", "m*k", "m*n*k")


# ---------------------------------------------------------------- performance, labels, metrics

def gflops(m, n, k, seconds):
    """P = 2*m*n*k / t in GFLOP/s; the same 2mnk is charged to NT and to TNN (t = transpose + NN)."""
    return 2.0 * m * n * k / seconds / 1e9


def label_from_perf(p_nt, p_tnn):
    """Section IV-A: D = P_NT - P_TNN; D >= 0 -> +1 (NT, ties included), else -1 (TNN)."""
    return 1 if (p_nt - p_tnn) >= 0 else -1


def label_from_times(t_nt, t_tnn):
    """Same rule stated on times: P is inversely proportional to t for a fixed shape."""
    return 1 if t_nt <= t_tnn else -1


def gow(p_mtnn, p_nt, p_tnn):
    """Gain over worst (Section V-B): (P_MTNN - min(P_NT, P_TNN)) / min(P_NT, P_TNN)."""
    worst = min(p_nt, p_tnn)
    return (p_mtnn - worst) / worst


def lub(p_mtnn, p_nt, p_tnn):
    """Loss under best (Section V-B): (P_MTNN - max(P_NT, P_TNN)) / max(P_NT, P_TNN)."""
    best = max(p_nt, p_tnn)
    return (p_mtnn - best) / best


def tnn_pays(t_transpose, t_nt, t_nn):
    """Eq. 4 (Section III): TNN is the faster way exactly when the transpose costs less than what the
    NN product saves over the NT product, T_transpose < T_NT - T_NN (strict: a tie stays with NT)."""
    return t_transpose < t_nt - t_nn


def ratio_statistics(t_nt, t_nn, t_tnn):
    """The case counts the paper reads off its Fig. 1-3, for lists of per-shape times (P ~ 1 / t):
    share of shapes with P_NN > P_NT and with P_NN >= 2 P_NT (Section II), share with
    P_TNN / P_NT < 1 and the largest ratio either way (Section III)."""
    n = len(t_nt)
    nn_faster = sum(1 for a, b in zip(t_nt, t_nn) if b < a)
    nn_twice = sum(1 for a, b in zip(t_nt, t_nn) if a >= 2.0 * b)
    nt_ahead = sum(1 for a, c in zip(t_nt, t_tnn) if a < c)          # P_TNN / P_NT < 1
    return {"nn_faster_than_nt": nn_faster / n, "nn_twice_nt": nn_twice / n,
            "tnn_over_nt_below_1": nt_ahead / n,
            "max_tnn_over_nt": max(a / c for a, c in zip(t_nt, t_tnn)),
            "max_nt_over_tnn": max(c / a for a, c in zip(t_nt, t_tnn))}


def selection_metrics(p_nt, p_tnn, predicted):
    """Table VII for a list of shapes.  P_MTNN is the performance of whichever algorithm was predicted.

    Returns fractions (not percent): mean improvement over always-NT and over always-TNN,
    GOW average / maximum, LUB average / minimum, and the accuracy against the measured labels.
    """
    p_nt = [float(v) for v in p_nt]
    p_tnn = [float(v) for v in p_tnn]
    n = len(p_nt)
    p_mtnn = [p_nt[i] if predicted[i] == 1 else p_tnn[i] for i in range(n)]
    gows = [gow(p_mtnn[i], p_nt[i], p_tnn[i]) for i in range(n)]
    lubs = [lub(p_mtnn[i], p_nt[i], p_tnn[i]) for i in range(n)]
    truth = [label_from_perf(p_nt[i], p_tnn[i]) for i in range(n)]
    return {
        "mtnn_vs_nt": sum((p_mtnn[i] - p_nt[i]) / p_nt[i] for i in range(n)) / n,
        "mtnn_vs_tnn": sum((p_mtnn[i] - p_tnn[i]) / p_tnn[i] for i in range(n)) / n,
        "gow_avg": sum(gows) / n, "gow_max": max(gows),
        "lub_avg": sum(lubs) / n, "lub_min": min(lubs),
        "accuracy": sum(1 for i in range(n) if truth[i] == predicted[i]) / n,
    }


def features(m, n, k):
    """Feature vector of one NT operation: the sizes and the element counts built from them.

    The paper's vector is five GPU constants followed by m, n, k; on a single GPU the constants
    never split a tree, so they are dropped, and the sizes of B, C, A and of the iteration space
    are appended (all O(1), all exact in double).
    """
    m, n, k = float(m), float(n), float(k)
    return [m, n, k, n * k, m * n, m * k, m * n * k]


# ---------------------------------------------------------------- boosted trees

def _sigmoid(z):
    return 1.0 / (1.0 + math.exp(-z))


class Node:
    __slots__ = ("feature", "threshold", "left", "right", "value")

    def __init__(self):
        self.feature = -1      # -1 marks a leaf
        self.threshold = 0.0
        self.left = None
        self.right = None
        self.value = 0.0


def _score(G, H):
    return G * G / (H + LAMBDA)


def best_split(X, g, h, idx):
    """Exact greedy search over one node's samples `idx`.

    For every feature the samples are ordered by value (ties by sample index), the running
    sums G_L, H_L are taken in that order, and a threshold is tried halfway between each pair
    of distinct neighbouring values.  gain = 1/2 [G_L^2/(H_L+lambda) + G_R^2/(H_R+lambda)
    - G^2/(H+lambda)] - gamma.  Both children need hessian weight >= MIN_CHILD_WEIGHT.
    Strictly larger gain wins, so among equals the lowest feature, then the lowest
    threshold, is kept.  Returns (gain, feature, threshold) or None.
    """
    G = 0.0
    H = 0.0
    for i in idx:
        G += g[i]
        H += h[i]
    parent = _score(G, H)
    best = None
    for f in range(X.shape[1]):
        order = sorted(idx, key=lambda i: (X[i, f], i))
        GL = 0.0
        HL = 0.0
        for pos in range(len(order) - 1):
            i = order[pos]
            GL += g[i]
            HL += h[i]
            v, vnext = X[i, f], X[order[pos + 1], f]
            if v == vnext:
                continue
            GR = G - GL
            HR = H - HL
            if HL < MIN_CHILD_WEIGHT or HR < MIN_CHILD_WEIGHT:
                continue
            gain = 0.5 * (_score(GL, HL) + _score(GR, HR) - parent) - GAMMA
            if gain > 0.0 and (best is None or gain > best[0]):
                best = (gain, f, 0.5 * (v + vnext))
    return best


def _grow(X, g, h, idx, depth):
    node = Node()
    split = best_split(X, g, h, idx) if depth < MAX_DEPTH else None
    if split is None:
        G = 0.0
        H = 0.0
        for i in idx:
            G += g[i]
            H += h[i]
        node.value = -G / (H + LAMBDA) * ETA
        return node
    _, f, thr = split
    node.feature, node.threshold = f, thr
    node.left = _grow(X, g, h, [i for i in idx if X[i, f] < thr], depth + 1)
    node.right = _grow(X, g, h, [i for i in idx if not (X[i, f] < thr)], depth + 1)
    return node


def tree_value(node, x):
    while node.feature >= 0:
        node = node.left if x[node.feature] < node.threshold else node.right
    return node.value


def train_gbdt(X, labels, num_trees=NUM_TREES):
    """Fit the boosted trees.  X: rows of features; labels in {-1, +1}.  Returns a list of root nodes.

    Round by round: margin_i = sum of the trees so far (0 at the start), p_i = sigmoid(margin_i),
    g_i = p_i - y_i, h_i = p_i (1 - p_i) with y_i = 1 for label +1 and 0 for label -1;
    grow one tree on (g, h); add it with step eta.
    """
    X = np.asarray(X, dtype=np.float64)
    y = [1.0 if l == 1 else 0.0 for l in labels]
    n = X.shape[0]
    margin = [0.0] * n
    trees = []
    for _ in range(num_trees):
        p = [_sigmoid(z) for z in margin]
        g = [p[i] - y[i] for i in range(n)]
        h = [p[i] * (1.0 - p[i]) for i in range(n)]
        root = _grow(X, g, h, list(range(n)), 0)
        trees.append(root)
        for i in range(n):
            margin[i] += tree_value(root, X[i])
    return trees


def margin(trees, x):
    s = 0.0
    for t in trees:
        s += tree_value(t, x)
    return s


def predict_label(trees, x):
    """+1 (NT) if the summed margin is >= 0, else -1 (TNN); a zero margin keeps the memory-free choice."""
    return 1 if margin(trees, x) >= 0.0 else -1


def select(trees, m, n, k):
    return predict_label(trees, features(m, n, k))


def tree_depth(node):
    return 0 if node.feature < 0 else 1 + max(tree_depth(node.left), tree_depth(node.right))


def flatten(trees):
    """Trees as parallel arrays (pre-order), the form the model file uses: per node
    feature (-1 = leaf), threshold, left index, right index, value."""
    out = []
    for root in trees:
        rows = []

        def walk(nd):
            me = len(rows)
            rows.append(None)
            if nd.feature < 0:
                rows[me] = (-1, 0.0, -1, -1, nd.value)
            else:
                l = walk(nd.left)
                r = walk(nd.right)
                rows[me] = (nd.feature, nd.threshold, l, r, 0.0)
            return me

        walk(root)
        out.append(rows)
    return out


def stratified_split(labels, seed, test_fraction=0.2):
    """Seeded 80/20 split that keeps the class proportions (the paper stratifies its split by GPU;
    with one GPU the split is stratified by class instead).  Returns (train_idx, test_idx)."""
    rng = np.random.RandomState(seed)
    train, test = [], []
    for cls in (-1, 1):
        members = [i for i, l in enumerate(labels) if l == cls]
        perm = rng.permutation(len(members))
        n_test = int(round(test_fraction * len(members)))
        test += [members[j] for j in perm[:n_test]]
        train += [members[j] for j in perm[n_test:]]
    return sorted(train), sorted(test)

"""Pins for the selection oracle: label rule, GOW/LUB, features, boosted trees.

Expected values are the paper's formulas worked by hand (tests/golden/selection_cases.txt),
closed forms of the first boosting round, and behaviour on separable data.
"""
import math
import os

import numpy as np
import pytest

from oracle import selection as S


def _cases(golden_dir):
    rows = []
    for line in open(os.path.join(golden_dir, "selection_cases.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        left, right = line.split("|")
        p_nt, p_tnn, pred = left.split()
        lab, g, l = right.split()
        rows.append((float(p_nt), float(p_tnn), int(pred), int(lab), float(g), float(l)))
    return rows


def test_label_rule_and_metrics_golden(golden_dir):
    rows = _cases(golden_dir)
    assert len(rows) == 7
    for p_nt, p_tnn, pred, lab, g, l in rows:
        assert S.label_from_perf(p_nt, p_tnn) == lab
        p_mtnn = p_nt if pred == 1 else p_tnn
        assert S.gow(p_mtnn, p_nt, p_tnn) == pytest.approx(g, abs=1e-12)
        assert S.lub(p_mtnn, p_nt, p_tnn) == pytest.approx(l, abs=1e-12)


def test_label_from_times_agrees_with_perf_and_tie_goes_to_nt():
    m, n, k = 128, 256, 512
    for t_nt, t_tnn in [(1e-3, 2e-3), (2e-3, 1e-3), (1e-3, 1e-3), (3.3e-5, 3.31e-5)]:
        by_perf = S.label_from_perf(S.gflops(m, n, k, t_nt), S.gflops(m, n, k, t_tnn))
        assert S.label_from_times(t_nt, t_tnn) == by_perf
    assert S.label_from_times(5e-4, 5e-4) == 1
    assert S.gflops(1000, 1000, 1000, 1.0) == 2.0


def test_selection_metrics_table_by_hand():
    # three shapes; predictor right on the first two, wrong on the third
    p_nt = [100.0, 300.0, 100.0]
    p_tnn = [200.0, 150.0, 400.0]
    pred = [-1, 1, 1]
    r = S.selection_metrics(p_nt, p_tnn, pred)
    # P_MTNN = [200, 300, 100]
    assert r["mtnn_vs_nt"] == pytest.approx((1.0 + 0.0 + 0.0) / 3)
    assert r["mtnn_vs_tnn"] == pytest.approx((0.0 + 1.0 - 0.75) / 3)
    assert r["gow_avg"] == pytest.approx((1.0 + 1.0 + 0.0) / 3) and r["gow_max"] == 1.0
    assert r["lub_avg"] == pytest.approx((0.0 + 0.0 - 0.75) / 3) and r["lub_min"] == -0.75
    assert r["accuracy"] == pytest.approx(2 / 3)


def test_gow_lub_invariants_when_mtnn_runs_one_of_the_two():
    rng = np.random.RandomState(0)
    for _ in range(200):
        a, b = rng.uniform(1, 1000, size=2)
        for pick in (a, b):
            assert S.gow(pick, a, b) >= 0.0 and S.lub(pick, a, b) <= 0.0


def test_features_are_sizes_and_element_counts():
    assert S.features(2, 3, 5) == [2.0, 3.0, 5.0, 15.0, 6.0, 10.0, 30.0]
    assert len(S.FEATURE_NAMES) == len(S.features(1, 1, 1))
    big = S.features(65536, 65536, 65536)          # the paper's largest size stays exact in double
    assert big[-1] == float(2 ** 48)


# ---- boosted trees

def test_first_round_closed_form_single_split():
    # 8 points on a line, classes split at 4.5.  Round 1: margin 0 -> p = 1/2, g = +-1/2, h = 1/4.
    # Split there: G_L = 2, H_L = 1, G_R = -2, H_R = 1, G = 0:
    #   gain = 1/2 (4/2 + 4/2 - 0) = 2 ; leaves = -G/(H + 1) = -1 and +1.
    X = np.arange(1, 9, dtype=np.float64).reshape(-1, 1)
    y = [-1] * 4 + [1] * 4
    g = [0.5] * 4 + [-0.5] * 4
    h = [0.25] * 8
    gain, f, thr = S.best_split(X, g, h, list(range(8)))
    assert (gain, f, thr) == (2.0, 0, 4.5)
    trees = S.train_gbdt(X, y, num_trees=1)
    flat = S.flatten(trees)[0]
    assert flat == [(0, 4.5, 1, 2, 0.0), (-1, 0.0, -1, -1, -1.0), (-1, 0.0, -1, -1, 1.0)]
    assert [S.predict_label(trees, x) for x in X] == y
    # a second round on these 8 points cannot split (each side carries 4 p(1-p) < 1 hessian weight,
    # p = sigmoid(-1)) and its single leaf is -G/(H+1) with G = 4p - 4p = 0
    assert S.flatten(S.train_gbdt(X, y, num_trees=2))[1] == [(-1, 0.0, -1, -1, 0.0)]


def test_second_round_closed_form():
    # 16 points, 8 per class.  Round 1: G_L = 4, H_L = 2 -> leaves -4/3 and +4/3.
    # Round 2: p = sigmoid(-4/3) on the left (y = 0): g = p, h = p(1-p); the only profitable split is
    # the same one (splitting a group with equal g and h never gains), leaf = -8p / (8p(1-p) + 1).
    X = np.arange(1, 17, dtype=np.float64).reshape(-1, 1)
    y = [-1] * 8 + [1] * 8
    flat = S.flatten(S.train_gbdt(X, y, num_trees=2))
    assert flat[0][0][:2] == (0, 8.5)
    assert flat[0][1][4] == pytest.approx(-4.0 / 3.0, rel=1e-15) and flat[0][2][4] == pytest.approx(4.0 / 3.0, rel=1e-15)
    p = 1.0 / (1.0 + math.exp(4.0 / 3.0))
    want = -(8 * p) / (8 * p * (1 - p) + 1.0)
    assert len(flat[1]) == 3 and flat[1][0][:2] == (0, 8.5)
    assert flat[1][1][4] == pytest.approx(want, rel=1e-13) and flat[1][2][4] == pytest.approx(-want, rel=1e-13)


def test_min_child_weight_blocks_tiny_children():
    # 4 points: any split leaves a child with hessian weight <= 0.75 < 1 -> a single leaf, value -G/(H+1) = 0
    X = np.array([[1.0], [2.0], [3.0], [4.0]])
    trees = S.train_gbdt(X, [-1, -1, 1, 1], num_trees=1)
    assert S.flatten(trees)[0] == [(-1, 0.0, -1, -1, 0.0)]
    assert S.predict_label(trees, [1.0]) == 1          # zero margin -> NT


def test_lowest_feature_wins_ties_and_midpoint_threshold():
    base = np.array([1, 1, 1, 1, 9, 9, 9, 9], dtype=np.float64)
    X = np.stack([base * 3.0, base, base + 2.0], axis=1)        # three equally good features
    trees = S.train_gbdt(X, [-1] * 4 + [1] * 4, num_trees=1)
    root = trees[0]
    assert root.feature == 0 and root.threshold == 0.5 * (3.0 + 27.0)


def test_xor_needs_depth_two():
    pts = []
    lab = []
    # quadrants of unequal size: on a perfectly balanced XOR every first split has zero gain
    for qx, qy, l, side in [(0, 0, -1, 8), (1, 1, -1, 5), (0, 1, 1, 6), (1, 0, 1, 5)]:
        for i in range(side):
            for j in range(side):
                pts.append([qx * 10 + i * 0.5, qy * 10 + j * 0.5])
                lab.append(l)
    X = np.array(pts)
    trees = S.train_gbdt(X, lab, num_trees=8)
    assert all(S.predict_label(trees, x) == l for x, l in zip(X, lab))
    assert max(S.tree_depth(t) for t in trees) >= 2
    one = S.train_gbdt(X, lab, num_trees=1)
    assert S.tree_depth(one[0]) >= 2


def test_structure_limits_and_rule_recovery():
    # a rule in the spirit of the profitability condition of Section III: TNN (-1) wins when the
    # transposed matrix is amortised over many rows of A
    sizes = [2 ** i for i in range(6, 14)]
    X, lab = [], []
    for m in sizes:
        for n in sizes:
            for k in sizes:
                X.append(S.features(m, n, k))
                lab.append(-1 if (m >= 512 and k >= 256) else 1)
    trees = S.train_gbdt(np.array(X), lab)
    assert len(trees) == S.NUM_TREES == 8
    assert all(S.tree_depth(t) <= S.MAX_DEPTH == 8 for t in trees)
    assert all(S.predict_label(trees, x) == l for x, l in zip(X, lab))
    assert S.select(trees, 8192, 64, 8192) == -1 and S.select(trees, 64, 8192, 8192) == 1


def test_accuracy_is_in_line_with_an_independent_library():
    sk = pytest.importorskip("sklearn.ensemble")
    rng = np.random.RandomState(3)
    X = rng.uniform(0, 1, size=(400, 3))
    score = X[:, 0] * 2 - X[:, 1] + 0.3 * np.sin(6 * X[:, 2]) + rng.normal(0, 0.15, 400)
    lab = [1 if s > 0.5 else -1 for s in score]
    tr, te = S.stratified_split(lab, seed=1)
    ours = S.train_gbdt(X[tr], [lab[i] for i in tr])
    acc = np.mean([S.predict_label(ours, X[i]) == lab[i] for i in te])
    ref = sk.GradientBoostingClassifier(n_estimators=8, max_depth=8, learning_rate=1.0, random_state=0)
    ref.fit(X[tr], [lab[i] for i in tr])
    ref_acc = ref.score(X[te], [lab[i] for i in te])
    assert acc >= 0.75 and abs(acc - ref_acc) < 0.12


def test_stratified_split_keeps_proportions_and_is_seeded():
    lab = [1] * 100 + [-1] * 400
    tr, te = S.stratified_split(lab, seed=7)
    assert len(te) == 100 and len(tr) == 400 and not set(tr) & set(te)
    assert sum(1 for i in te if lab[i] == 1) == 20
    assert S.stratified_split(lab, seed=7) == (tr, te)
    assert S.stratified_split(lab, seed=8)[1] != te


def test_eq4_and_ratio_statistics_on_a_hand_table():
    # Eq. 4 (Section III): TNN pays exactly when the transpose costs less than NN saves over NT.
    assert S.tnn_pays(1.0, 10.0, 8.0) is True            # 1 < 10 - 8
    assert S.tnn_pays(2.0, 10.0, 8.0) is False           # a tie stays with NT
    assert S.tnn_pays(0.5, 8.0, 9.0) is False            # NT already faster than NN: never
    # four shapes, times chosen so that every count can be read off by eye:
    #   t_nt   t_nn   t_tnn    NN faster?  NN twice?  NT ahead of TNN?  P_TNN/P_NT  P_NT/P_TNN
    #   10      4      5        yes         yes        no                2.0         0.5
    #   10      8     12        yes         no         yes               0.833       1.2
    #    6      7      9        no          no         yes               0.667       1.5
    #    8      8      8        no          no         no (tie)          1.0         1.0
    st = S.ratio_statistics([10.0, 10.0, 6.0, 8.0], [4.0, 8.0, 7.0, 8.0], [5.0, 12.0, 9.0, 8.0])
    assert st == {"nn_faster_than_nt": 0.5, "nn_twice_nt": 0.25, "tnn_over_nt_below_1": 0.5,
                  "max_tnn_over_nt": 2.0, "max_nt_over_tnn": 1.5}
    # consistency with the label rule: "P_TNN / P_NT below 1" counts the strict NT wins, a subset of the +1 labels
    labels = [S.label_from_times(a, c) for a, c in zip([10.0, 10.0, 6.0, 8.0], [5.0, 12.0, 9.0, 8.0])]
    assert labels == [-1, 1, 1, 1]

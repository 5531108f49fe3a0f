"""Pins for the support-vector oracle (Section V-A, Table VI: C = 1000, gamma = 0.01, inputs in (0, 1)):
the closed form for two points, the optimality conditions of the dual at the returned multipliers, an
independent library routine on seeded data, and separable toy sets."""
import math

import numpy as np
import pytest

from oracle import svm


def toy(seed, n, nfeat=3, margin=0.0):
    rng = np.random.RandomState(seed)
    X = rng.uniform(0.0, 1.0, size=(n, nfeat))
    y = np.where(X[:, 0] + 0.5 * X[:, 1] > 0.75 + 0.0 * X[:, 2], 1, -1)
    if margin:
        keep = np.abs(X[:, 0] + 0.5 * X[:, 1] - 0.75) > margin
        X, y = X[keep], y[keep]
    return X.tolist(), y.tolist()


def test_paper_settings_and_scaling():
    assert svm.C_PAPER == 1000.0 and svm.GAMMA_PAPER == 0.01
    rows, lo, hi = svm.scale01([[64, 5.0], [8192, 5.0], [4128, 5.0]])
    assert rows == [[0.0, 0.0], [1.0, 0.0], [0.5, 0.0]] and lo == [64, 5.0] and hi == [8192, 5.0]
    other, _, _ = svm.scale01([[16320, 7.0]], lo, hi)
    assert other == [[2.0, 0.0]]                             # the training set's map, applied as is


def test_kernels_by_hand():
    assert svm.kernel("rbf", [0.0, 0.0], [3.0, 4.0], gamma=0.01) == math.exp(-0.25)
    assert svm.kernel("poly", [1.0, 2.0], [3.0, 4.0], gamma=0.5, degree=3, coef0=0.0) == (0.5 * 11.0) ** 3
    assert svm.kernel("poly", [1.0, 2.0], [3.0, 4.0], gamma=0.01) == pytest.approx(0.11 ** 3, rel=1e-15)


@pytest.mark.parametrize("kind", ["rbf", "poly"])
def test_two_points_closed_form(kind):
    """One point per class: both multipliers equal a = min(C, 2 / (K11 + K22 - 2 K12)) (the maximiser of
    2a - a^2 eta / 2), and b puts the two margins at +1 and -1 (or keeps them symmetric when a = C)."""
    x1, x2 = [0.9, 0.8], [0.1, 0.3]
    for C in (1000.0, 0.5):
        for gamma in (0.01, 2.0):
            m = svm.train([x1, x2], [1, -1], kind, C=C, gamma=gamma)
            k11, k22, k12 = (svm.kernel(kind, a, b, gamma) for a, b in ((x1, x1), (x2, x2), (x1, x2)))
            a = min(C, 2.0 / (k11 + k22 - 2.0 * k12))
            assert m["alpha"] == pytest.approx([a, a], rel=1e-9)
            f1, f2 = svm.decision(m, x1), svm.decision(m, x2)
            if a < C:
                assert f1 == pytest.approx(1.0, abs=1e-9) and f2 == pytest.approx(-1.0, abs=1e-9)
            else:
                assert f1 - f2 == pytest.approx(a * (k11 + k22 - 2.0 * k12), rel=1e-9) and f1 > 0 > f2


@pytest.mark.parametrize("kind,gamma,C", [("rbf", 0.01, 1000.0), ("rbf", 3.0, 10.0), ("poly", 0.01, 1000.0), ("poly", 1.0, 5.0)])
def test_optimality_conditions_hold_at_the_solution(kind, gamma, C):
    X, y = toy(3, 26)
    m = svm.train(X, y, kind, C=C, gamma=gamma)
    a = m["alpha"]
    assert all(-1e-12 <= v <= C + 1e-9 for v in a)
    assert abs(sum(v * t for v, t in zip(a, y))) <= 1e-9 * C
    # y f(x) >= 1 where a = 0, = 1 where 0 < a < C, <= 1 where a = C (to the solver's stopping tolerance)
    slack = 2e-3 if C >= 1000 else 2e-4
    for v, t, x in zip(a, y, X):
        yf = t * svm.decision(m, x)
        if v <= 1e-9 * C:
            assert yf >= 1.0 - slack
        elif v >= C * (1 - 1e-9):
            assert yf <= 1.0 + slack
        else:
            assert abs(yf - 1.0) <= slack
    # no feasible pair move lowers the dual any further, and the dual is below its value at a = 0
    K = [[svm.kernel(kind, p, q, gamma) for q in X] for p in X]
    assert svm.dual_objective(K, y, a) < 0.0


@pytest.mark.parametrize("kind,gamma,C", [("rbf", 0.5, 10.0), ("rbf", 0.01, 1000.0), ("poly", 1.0, 10.0), ("poly", 0.01, 1000.0)])
def test_against_an_independent_library_routine(kind, gamma, C):
    """scikit-learn's SVC solves the same dual with another algorithm: the decision values must agree."""
    sk = pytest.importorskip("sklearn.svm")
    X, y = toy(11, 30, nfeat=4)
    m = svm.train(X, y, kind, C=C, gamma=gamma, tol=1e-12)
    ref = sk.SVC(C=C, kernel=kind, gamma=gamma, degree=3, coef0=0.0, tol=1e-8).fit(np.array(X), np.array(y))
    probe = np.random.RandomState(5).uniform(0, 1, size=(40, 4))
    got = np.array([svm.decision(m, p.tolist()) for p in probe])
    want = ref.decision_function(probe)
    scale = max(1.0, float(np.abs(want).max()))
    assert np.abs(got - want).max() <= 2e-3 * scale
    far = np.abs(want) > 1e-2 * scale
    assert (np.where(got[far] >= 0, 1, -1) == ref.predict(probe)[far]).all()


def test_separable_sets_are_learnt_exactly():
    X, y = toy(21, 40, margin=0.08)
    assert 1 in y and -1 in y
    for kind, gamma in (("rbf", 1.0), ("poly", 1.0), ("rbf", 0.01)):
        m = svm.train(X, y, kind, C=1000.0, gamma=gamma)
        assert [svm.predict(m, x) for x in X] == y, (kind, gamma)
    # one class only: nothing to separate, every answer is that class's side of b = 0 ... i.e. +1 on f = 0
    m = svm.train(X[:5], [1] * 5, "rbf")
    assert all(v == 0.0 for v in m["alpha"]) and svm.predict(m, X[7]) == 1

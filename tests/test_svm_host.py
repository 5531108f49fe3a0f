"""The product's support-vector solver (classifier study, Section V-A / Table VI) against the CPU
oracle's exhaustive pair search on seeded toy data.  Host only."""
import numpy as np
import pytest

from oracle import svm as osvm
from paper_1702_03192_amd import svm


def toy(seed, n, nfeat=3, margin=0.0):
    rng = np.random.RandomState(seed)
    X = rng.uniform(0.0, 1.0, size=(n, nfeat))
    s = X[:, 0] + 0.5 * X[:, 1]
    keep = np.abs(s - 0.75) > margin
    return X[keep], np.where(s[keep] > 0.75, 1, -1)


def test_scaling_matches_the_oracle():
    raw = np.array([[64.0, 5.0, 4096.0], [8192.0, 5.0, 64.0], [4128.0, 5.0, 1024.0]])
    got, lo, hi = svm.scale01(raw)
    want, olo, ohi = osvm.scale01(raw.tolist())
    assert got.tolist() == want and lo.tolist() == olo and hi.tolist() == ohi
    more = np.array([[16320.0, 9.0, 0.0]])
    assert svm.scale01(more, lo, hi)[0].tolist() == osvm.scale01(more.tolist(), olo, ohi)[0]


def test_kernel_matrices_match_the_oracle():
    X, _ = toy(2, 9, nfeat=4)
    for kind, gamma in (("rbf", 0.01), ("rbf", 2.5), ("poly", 0.01), ("poly", 1.5)):
        K = svm.kernel_matrix(kind, X, X, gamma)
        for i in range(len(X)):
            for j in range(len(X)):
                assert K[i, j] == pytest.approx(osvm.kernel(kind, X[i].tolist(), X[j].tolist(), gamma), rel=1e-12, abs=1e-15)


@pytest.mark.parametrize("kind,gamma,C", [("rbf", 0.5, 10.0), ("rbf", 0.01, 1000.0), ("poly", 1.0, 10.0), ("poly", 0.01, 1000.0)])
def test_decision_values_match_the_oracle(kind, gamma, C):
    X, y = toy(11, 30, nfeat=4)
    ours = svm.train(X, y, kind, C=C, gamma=gamma, eps=1e-7)
    assert ours.converged
    ref = osvm.train(X.tolist(), y.tolist(), kind, C=C, gamma=gamma, tol=1e-12)
    probe = np.random.RandomState(5).uniform(0, 1, size=(40, 4))
    got = ours.decision(probe)
    want = np.array([osvm.decision(ref, p.tolist()) for p in probe])
    scale = max(1.0, float(np.abs(want).max()))
    assert np.abs(got - want).max() <= 2e-3 * scale
    far = np.abs(want) > 1e-2 * scale
    assert (ours.predict(probe)[far] == np.where(want[far] >= 0, 1, -1)).all()


def test_separable_toy_data_is_learnt_exactly_with_the_papers_settings():
    X, y = toy(21, 400, margin=0.05)
    assert (y == 1).any() and (y == -1).any()
    for kind in ("rbf", "poly"):
        m = svm.train(X, y, kind, C=svm.C_PAPER, gamma=1.0)
        assert m.converged and (m.predict(X) == y).all()
    # with the paper's gamma = 0.01 the radial kernel is nearly flat on (0, 1) inputs: C = 1000 still separates a wide margin
    Xw, yw = toy(22, 200, margin=0.2)
    m = svm.train(Xw, yw, "rbf")
    assert m.converged and (m.predict(Xw) == yw).all()
    one = svm.train(X[:5], np.ones(5), "rbf")
    assert one.predict(X[:3]).tolist() == [1, 1, 1]

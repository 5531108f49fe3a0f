"""Pins for the fully-connected training-step oracle (Section V-C sizes; the step itself is this
build's reading): a hand-worked tiny net, and central finite differences of the loss."""
import math

import numpy as np

from oracle import fc


def test_tiny_net_by_hand():
    # one layer, 1 sample, 2 inputs, 2 classes: logits = W x + b
    X = np.array([[1.0, 2.0]])
    W = [np.array([[0.5, -0.5], [0.25, 0.75]])]
    b = [np.array([0.0, -1.0])]
    out = fc.fc_step(X, np.array([1]), W, b, lr=0.1)
    z = np.array([0.5 - 1.0, 0.25 + 1.5 - 1.0])          # [-0.5, 0.75]
    p = np.exp(z) / np.exp(z).sum()
    assert math.isclose(out["loss"], -math.log(p[1]), rel_tol=1e-14)
    dz = p - np.array([0.0, 1.0])
    assert np.allclose(out["dW"][0], np.outer(dz, X[0]), rtol=1e-14)
    assert np.allclose(out["db"][0], dz, rtol=1e-14)
    assert np.allclose(out["W_new"][0], W[0] - 0.1 * np.outer(dz, X[0]), rtol=1e-14)


def test_gradients_match_finite_differences():
    rng = np.random.RandomState(0)
    dims = [5, 7, 6, 4]
    batch = 9
    X = rng.normal(size=(batch, dims[0]))
    labels = rng.randint(0, dims[-1], size=batch)
    W = [rng.normal(scale=0.5, size=(dims[i + 1], dims[i])) for i in range(3)]
    b = [rng.normal(scale=0.1, size=dims[i + 1]) for i in range(3)]
    out = fc.fc_step(X, labels, W, b, lr=0.0)
    eps = 1e-6
    for l in range(3):
        for (r, c) in [(0, 0), (dims[l + 1] - 1, dims[l] - 1), (1, 2)]:
            Wp = [w.copy() for w in W]
            Wm = [w.copy() for w in W]
            Wp[l][r, c] += eps
            Wm[l][r, c] -= eps
            num = (fc.fc_step(X, labels, Wp, b, 0.0)["loss"] - fc.fc_step(X, labels, Wm, b, 0.0)["loss"]) / (2 * eps)
            assert math.isclose(out["dW"][l][r, c], num, rel_tol=1e-5, abs_tol=1e-8)
        bp = [v.copy() for v in b]
        bm = [v.copy() for v in b]
        bp[l][1] += eps
        bm[l][1] -= eps
        num = (fc.fc_step(X, labels, W, bp, 0.0)["loss"] - fc.fc_step(X, labels, W, bm, 0.0)["loss"]) / (2 * eps)
        assert math.isclose(out["db"][l][1], num, rel_tol=1e-5, abs_tol=1e-8)


def test_uniform_logits_give_log_classes():
    X = np.zeros((4, 3))
    W = [np.zeros((6, 3)), np.zeros((10, 6))]
    b = [np.zeros(6), np.zeros(10)]
    out = fc.fc_step(X, np.array([0, 3, 9, 5]), W, b, lr=0.01)
    assert math.isclose(out["loss"], math.log(10.0), rel_tol=1e-14)

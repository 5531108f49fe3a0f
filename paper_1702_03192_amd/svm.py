"""Support-vector baselines for the classifier comparison (Section V-A, Table VI of the MTNN paper).

The paper sets its boosted trees against two support vector machines -- radial basis function and
polynomial kernels, C = 1000, gamma = 0.01, inputs scaled to (0, 1) -- trained with an external
library.  This module is our own solver for the same soft-margin dual, so that the comparison can be
run on this machine's timing tables: sequential minimal optimisation, at each step the pair of
multipliers that violates the optimality conditions most (the largest gap between -y_i G_i over the
multipliers that may still rise and over those that may still fall, G the dual's gradient), solved
jointly in closed form and clipped to the box.  The kernel matrix is formed once (a timing table has
a few thousand rows at most); everything else is numpy vector arithmetic.  Host only.
"""
from __future__ import annotations

import numpy as np

C_PAPER = 1000.0
GAMMA_PAPER = 0.01


def scale01(X, lo=None, hi=None):
    """Each feature mapped linearly so that the training rows span [0, 1]; returns (scaled, lo, hi)."""
    X = np.asarray(X, dtype=np.float64)
    if lo is None:
        lo, hi = X.min(axis=0), X.max(axis=0)
    span = np.where(hi > lo, hi - lo, 1.0)
    return np.where(hi > lo, (X - lo) / span, 0.0), lo, hi


def kernel_matrix(kind, A, B, gamma=GAMMA_PAPER, degree=3, coef0=0.0):
    A = np.asarray(A, dtype=np.float64)
    B = np.asarray(B, dtype=np.float64)
    if kind == "rbf":
        d2 = (A * A).sum(1)[:, None] + (B * B).sum(1)[None, :] - 2.0 * (A @ B.T)
        return np.exp(-gamma * np.maximum(d2, 0.0))
    if kind == "poly":
        return (gamma * (A @ B.T) + coef0) ** degree
    raise ValueError(kind)


class Model:
    def __init__(self, kind, gamma, sv, coef, b, steps, converged):
        self.kind, self.gamma, self.sv, self.coef, self.b = kind, gamma, sv, coef, b
        self.steps, self.converged = steps, converged

    def decision(self, X):
        if self.sv.shape[0] == 0:
            return np.full(len(X), self.b)
        return kernel_matrix(self.kind, X, self.sv, self.gamma) @ self.coef + self.b

    def predict(self, X):
        return np.where(self.decision(X) >= 0.0, 1, -1)


def train(X, y, kind="rbf", C=C_PAPER, gamma=GAMMA_PAPER, eps=1e-3, max_steps=2000000):
    """X: rows already scaled; y: +1 / -1.  eps: stopping gap of the optimality conditions."""
    X = np.asarray(X, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    n = len(y)
    K = kernel_matrix(kind, X, X, gamma)
    diag = K.diagonal().copy()
    a = np.zeros(n)
    G = -np.ones(n)                       # gradient of the dual at a = 0
    pos = y > 0
    steps, converged = 0, False
    m_up = m_low = 0.0
    while steps < max_steps:
        score = -y * G
        up = np.where(pos, a < C, a > 0)          # multipliers that may move in the +y direction
        low = np.where(pos, a > 0, a < C)         # ... in the -y direction
        if not up.any() or not low.any():
            converged = True
            break
        su = np.where(up, score, -np.inf)
        sl = np.where(low, score, np.inf)
        i, j = int(su.argmax()), int(sl.argmin())
        m_up, m_low = su[i], sl[j]
        if m_up - m_low < eps:
            converged = True
            break
        eta = max(diag[i] + diag[j] - 2.0 * K[i, j], 1e-12)
        t = (m_up - m_low) / eta
        t = min(t, C - a[i] if pos[i] else a[i], a[j] if pos[j] else C - a[j])
        a[i] += y[i] * t
        a[j] -= y[j] * t
        G += y * (t * (K[:, i] - K[:, j]))
        steps += 1
    score = -y * G
    free = (a > 1e-9 * C) & (a < C * (1.0 - 1e-9))
    if free.any():
        b = float(score[free].mean())
    elif n and (pos.any() and (~pos).any()):
        b = 0.5 * float(m_up + m_low)
    else:
        b = 0.0
    keep = a > 0
    return Model(kind, gamma, X[keep], (a * y)[keep], b, steps, converged)

"""CPU oracle for the support-vector baselines of the paper's classifier comparison.  TEST
INFRASTRUCTURE ONLY.

Section V-A / Table VI compare the boosted trees with two support vector machines -- a radial basis
function kernel and a polynomial kernel, C = 1000, gamma = 0.01, inputs scaled to (0, 1) -- trained
with an external library.  What such a machine computes has a plain definition, the soft-margin dual

    minimise   W(a) = 1/2 sum_ij a_i a_j y_i y_j K(x_i, x_j) - sum_i a_i
    subject to 0 <= a_i <= C,  sum_i a_i y_i = 0,

with decision function f(x) = sum_i a_i y_i K(x_i, x) + b and label sign(f(x)) (+1 on f = 0), and this
file solves exactly that in the slowest obvious way: plain Python loops, no caching, and at every
step the pair of multipliers whose joint optimum lowers W the most, found by trying all pairs.
Kernels: rbf K = exp(-gamma |x - z|^2); poly K = (gamma x.z + coef0)^degree with the documented
defaults of the library the paper names (degree 3, coef0 0).
"""
from __future__ import annotations

import math

C_PAPER = 1000.0        # Section V-A
GAMMA_PAPER = 0.01      # Section V-A


def scale01(rows, lo=None, hi=None):
    """Each feature mapped linearly so that the training set spans [0, 1] (a constant feature maps to 0).
    Returns (scaled rows, lo, hi); pass lo / hi of the training set to scale other rows the same way."""
    nfeat = len(rows[0])
    if lo is None:
        lo = [min(r[f] for r in rows) for f in range(nfeat)]
        hi = [max(r[f] for r in rows) for f in range(nfeat)]
    out = []
    for r in rows:
        out.append([(r[f] - lo[f]) / (hi[f] - lo[f]) if hi[f] > lo[f] else 0.0 for f in range(nfeat)])
    return out, lo, hi


def kernel(kind, x, z, gamma=GAMMA_PAPER, degree=3, coef0=0.0):
    if kind == "rbf":
        d2 = 0.0
        for a, b in zip(x, z):
            d2 += (a - b) * (a - b)
        return math.exp(-gamma * d2)
    if kind == "poly":
        dot = 0.0
        for a, b in zip(x, z):
            dot += a * b
        return (gamma * dot + coef0) ** degree
    raise ValueError(kind)


def dual_objective(K, y, a):
    n = len(y)
    w = 0.0
    for i in range(n):
        for j in range(n):
            w += 0.5 * a[i] * a[j] * y[i] * y[j] * K[i][j]
        w -= a[i]
    return w


def train(X, y, kind="rbf", C=C_PAPER, gamma=GAMMA_PAPER, tol=1e-10, max_steps=200000):
    """Solve the dual.  y in {+1, -1}.  Returns dict(alpha, b, X, y, kind, gamma)."""
    n = len(y)
    K = [[kernel(kind, X[i], X[j], gamma) for j in range(n)] for i in range(n)]
    a = [0.0] * n
    # f0[i] = sum_j a_j y_j K_ij, kept up to date
    f0 = [0.0] * n
    for _ in range(max_steps):
        best_gain, best = 0.0, None
        for i in range(n):
            for j in range(i + 1, n):
                # move a_i by y_i t and a_j by -y_j t: sum_i a_i y_i is unchanged.  Along that line
                # W(t) = W(0) + t g + 1/2 t^2 eta with
                g = (y[i] * (y[i] * f0[i] - 1.0)) - (y[j] * (y[j] * f0[j] - 1.0))
                eta = K[i][i] + K[j][j] - 2.0 * K[i][j]
                lo_t = max(-a[i] if y[i] > 0 else a[i] - C, a[j] - C if y[j] > 0 else -a[j])
                hi_t = min(C - a[i] if y[i] > 0 else a[i], a[j] if y[j] > 0 else C - a[j])
                if eta > 1e-300:
                    t = min(max(-g / eta, lo_t), hi_t)
                else:
                    t = lo_t if g > 0 else hi_t
                gain = -(t * g + 0.5 * t * t * eta)
                if gain > best_gain:
                    best_gain, best = gain, (i, j, t)
        if best is None or best_gain <= tol:
            break
        i, j, t = best
        a[i] += y[i] * t
        a[j] -= y[j] * t
        a[i] = min(max(a[i], 0.0), C)
        a[j] = min(max(a[j], 0.0), C)
        for k in range(n):
            f0[k] += t * (K[k][i] - K[k][j])
    # threshold: y_t (f0_t + b) = 1 on the free multipliers; with none free, the middle of the allowed interval
    free = [y[t] - f0[t] for t in range(n) if 1e-9 * C < a[t] < C * (1.0 - 1e-9)]
    if free:
        b = sum(free) / len(free)
    else:
        ups = [y[t] - f0[t] for t in range(n) if (y[t] > 0 and a[t] < C) or (y[t] < 0 and a[t] > 0)]
        lows = [y[t] - f0[t] for t in range(n) if (y[t] < 0 and a[t] < C) or (y[t] > 0 and a[t] > 0)]
        b = 0.5 * (max(ups) + min(lows)) if ups and lows else 0.0
    return {"alpha": a, "b": b, "X": [list(r) for r in X], "y": list(y), "kind": kind, "gamma": gamma}


def decision(model, x):
    s = model["b"]
    for a, yi, xi in zip(model["alpha"], model["y"], model["X"]):
        if a != 0.0:
            s += a * yi * kernel(model["kind"], xi, x, model["gamma"])
    return s


def predict(model, x):
    return 1 if decision(model, x) >= 0.0 else -1

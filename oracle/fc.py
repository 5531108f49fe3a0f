"""CPU oracle for one training step of a fully connected net.  TEST INFRASTRUCTURE ONLY.

The paper evaluates MTNN inside fully connected networks described only by their layer
sizes (Section V-C, Table IX): the forward pass of a layer multiplies the mini-batch of
activations (mb x l1) by the transpose of the weights (l2 x l1) -- an NT operation whose
shape is fixed by l1, l2 and mb -- and the backward pass uses products without that
transpose.  Everything else about the step is this build's reading, since the paper is
silent: ReLU after every hidden layer, a bias on every layer, softmax cross-entropy averaged
over the mini-batch, plain SGD.

All arithmetic is float64.  The three matrix products of a layer are the definitions written
out as sums in increasing order of the summation index (``mtnn_oracle.c``: Eq. 2 for the forward
product, Eq. 1 for the two backward products); the elementwise steps are numpy's.  Inputs are
the float32 values the GPU path receives, widened.
"""
from __future__ import annotations

import numpy as np

from .gemm import nn_f64, nt_f64, tn_f64


def fc_step(X, labels, weights, biases, lr):
    """One forward/backward/update.

    X: batch x d0.  labels: batch ints.  weights[l]: d_{l+1} x d_l.  biases[l]: d_{l+1}.
    Returns dict(loss, logits, dW[], db[], W_new[], b_new[]), all float64, and the intermediates
    H[] (H[0] = X, H[l] = output of layer l) and dZ[] (gradient w.r.t. layer l's pre-activation).
    """
    H = [np.asarray(X, dtype=np.float64)]
    W = [np.asarray(w, dtype=np.float64) for w in weights]
    b = [np.asarray(v, dtype=np.float64) for v in biases]
    L = len(W)
    Z = []
    for l in range(L):
        z = nt_f64(H[l], W[l]) + b[l]             # forward: an NT operation per layer (Eq. 2)
        Z.append(z)
        H.append(np.maximum(z, 0.0) if l < L - 1 else z)
    logits = Z[-1]
    batch = logits.shape[0]
    shifted = logits - logits.max(axis=1, keepdims=True)
    logsum = np.log(np.exp(shifted).sum(axis=1, keepdims=True))
    logp = shifted - logsum
    loss = -logp[np.arange(batch), labels].mean()
    dZ = np.exp(logp)
    dZ[np.arange(batch), labels] -= 1.0
    dZ /= batch
    dW = [None] * L
    db = [None] * L
    dZs = [None] * L
    for l in range(L - 1, -1, -1):
        dZs[l] = dZ
        dW[l] = tn_f64(dZ, H[l])                   # d_{l+1} x d_l: sum over the mini-batch of dZ^T x H
        db[l] = dZ.sum(axis=0)
        if l > 0:
            dH = nn_f64(dZ, W[l])                  # batch x d_l  (an NN operation, Eq. 1)
            dZ = dH * (Z[l - 1] > 0.0)
    W_new = [W[l] - lr * dW[l] for l in range(L)]
    b_new = [b[l] - lr * db[l] for l in range(L)]
    return {"loss": float(loss), "logits": logits, "dW": dW, "db": db, "W_new": W_new, "b_new": b_new,
            "H": H, "dZ": dZs}

"""CPU oracle for one training step of a fully connected net.  TEST INFRASTRUCTURE ONLY.

The paper evaluates MTNN inside fully connected networks described only by their layer
sizes (Section V-C, Table IX): the forward pass of a layer multiplies the mini-batch of
activations (mb x l1) by the transpose of the weights (l2 x l1) -- an NT operation whose
shape is fixed by l1, l2 and mb -- and the backward pass uses products without that
transpose.  Everything else about the step is this build's reading, since the paper is
silent: ReLU after every hidden layer, a bias on every layer, softmax cross-entropy averaged
over the mini-batch, plain SGD.

All arithmetic is float64 numpy; matrix products are numpy's (a library primitive used as
one step).  Inputs are the float32 values the GPU path receives, widened.
"""
from __future__ import annotations

import numpy as np


def fc_step(X, labels, weights, biases, lr):
    """One forward/backward/update.

    X: batch x d0.  labels: batch ints.  weights[l]: d_{l+1} x d_l.  biases[l]: d_{l+1}.
    Returns dict(loss, logits, dW[], db[], W_new[], b_new[]), all float64.
    """
    H = [np.asarray(X, dtype=np.float64)]
    W = [np.asarray(w, dtype=np.float64) for w in weights]
    b = [np.asarray(v, dtype=np.float64) for v in biases]
    L = len(W)
    Z = []
    for l in range(L):
        z = H[l] @ W[l].T + b[l]                  # forward: an NT operation per layer
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
    for l in range(L - 1, -1, -1):
        dW[l] = dZ.T @ H[l]                        # d_{l+1} x d_l
        db[l] = dZ.sum(axis=0)
        if l > 0:
            dH = dZ @ W[l]                         # batch x d_l  (an NN operation)
            dZ = dH * (Z[l - 1] > 0.0)
    W_new = [W[l] - lr * dW[l] for l in range(L)]
    b_new = [b[l] - lr * db[l] for l in range(L)]
    return {"loss": float(loss), "logits": logits, "dW": dW, "db": db, "W_new": W_new, "b_new": b_new}

"""CPU oracle of the feed-forward classifier training step (TEST INFRASTRUCTURE ONLY).

The paper's neural-network training benchmark (its section on the Torch7 comparison) trains
10-class classifiers of a 784-dimensional input -- logistic regression, one hidden layer of 500
units, three hidden layers of 1000 units -- by stochastic gradient descent on single examples
or mini-batches of 10 or 60.  It prints no equations; the textbook ones are used:

    a_0 = x;   a_l = act(W_l a_{l-1} + b_l)  for the hidden layers;   z = W_L a_{L-1} + b_L
    loss = mean over the batch of ( logsumexp(z) - z[y] )          (natural log)
    after every batch:  W_l <- W_l - lr dloss/dW_l,  b_l <- b_l - lr dloss/db_l

Everything in float64 with numpy; one matrix product per layer and direction (a library
primitive used as a step), no blocking or fusion.  Only tests, the smoke check and the bench's
cpu_baseline leg may import this module; it shares no code with the GPU path.
"""
from __future__ import annotations

import numpy as np


def _act(a, kind):
    return 1.0 / (1.0 + np.exp(-a)) if kind == 0 else np.tanh(a)


def _act_grad(h, kind):
    return h * (1.0 - h) if kind == 0 else 1.0 - h * h


def forward(W, b, X, act):
    """Activations of every layer: [a_0 = X, a_1, ..., a_{L-1}] and the logits z [B, out]."""
    acts = [np.asarray(X, dtype=np.float64)]
    for l in range(len(W) - 1):
        acts.append(_act(acts[-1] @ np.asarray(W[l], np.float64).T + np.asarray(b[l], np.float64), act))
    z = acts[-1] @ np.asarray(W[-1], np.float64).T + np.asarray(b[-1], np.float64)
    return acts, z


def loss_and_grads(W, b, X, y, act):
    """Mean cross-entropy of one batch and its gradient w.r.t. every W_l, b_l."""
    acts, z = forward(W, b, X, act)
    B = z.shape[0]
    m = z.max(axis=1, keepdims=True)
    lse = m[:, 0] + np.log(np.exp(z - m).sum(axis=1))
    loss = float(np.mean(lse - z[np.arange(B), y]))
    dz = np.exp(z - lse[:, None])
    dz[np.arange(B), y] -= 1.0
    dz /= B
    dW, db = [None] * len(W), [None] * len(W)
    for l in range(len(W) - 1, -1, -1):
        dW[l] = dz.T @ acts[l]                  # [fan_out, fan_in]
        db[l] = dz.sum(axis=0)
        if l > 0:
            dz = (dz @ np.asarray(W[l], np.float64)) * _act_grad(acts[l], act)
    return loss, dW, db


def train(case, lr, n_batches=None):
    """Plain SGD over consecutive batches of case['X'], case['y'].  Returns dict W, b (float64 lists,
    updated copies) and losses [n_batches] (each computed with the parameters before its update)."""
    B = case["batch"]
    n = case["n_batches"] if n_batches is None else n_batches
    W = [np.array(w, dtype=np.float64) for w in case["W"]]
    b = [np.array(v, dtype=np.float64) for v in case["b"]]
    X = np.asarray(case["X"], dtype=np.float64)
    y = np.asarray(case["y"])
    losses = np.empty(n)
    for i in range(n):
        loss, dW, db = loss_and_grads(W, b, X[i * B:(i + 1) * B], y[i * B:(i + 1) * B], case["act"])
        losses[i] = loss
        for l in range(len(W)):
            W[l] -= lr * dW[l]
            b[l] -= lr * db[l]
    return dict(W=W, b=b, losses=losses)

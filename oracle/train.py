"""Loss, parameter update and one training iteration of Algorithm 1 (oracle side; test infrastructure).

Section II: empirical risk with the cross-entropy as the loss, minimised by gradient descent (SGD); Section
III / Algorithm 1: every worker computes the gradient of its partition's share of the risk, the shares are
summed (R11 of the design notes: equal replicas taking the same step and being averaged is the same update).

  loss      L = scale * sum over labelled rows i of ( logsumexp(logits_i) - logits_i[y_i] ),  scale = 1/m
  gradient  dlogits_i = scale * (softmax(logits_i) - onehot(y_i)),  zero for unlabelled rows (y_i < 0)
  update    H <- H - lr * dH

Everything in fp64.
"""
from __future__ import annotations

import numpy as np

from . import layer as _layer


def softmax_xent(logits: np.ndarray, labels: np.ndarray, scale: float):
    """(loss, dlogits, n_correct) of the rows of `logits` [n, C] with integer labels [n] (< 0: row ignored).
    A row counts as correct when its largest logit (lowest index on ties) is its label."""
    z = np.asarray(logits, dtype=np.float64)
    y = np.asarray(labels, dtype=np.int64)
    on = y >= 0
    zmax = z.max(axis=1, keepdims=True)
    e = np.exp(z - zmax)
    se = e.sum(axis=1, keepdims=True)
    lse = (zmax + np.log(se))[:, 0]
    idx = np.where(on, y, 0)
    row_loss = np.where(on, lse - z[np.arange(z.shape[0]), idx], 0.0)
    d = e / se
    d[np.arange(z.shape[0]), idx] -= 1.0
    d *= scale
    d[~on] = 0.0
    correct = int(np.sum(on & (z.argmax(axis=1) == y)))
    return float(scale * row_loss.sum()), d, correct


def sgd(weight: np.ndarray, grad: np.ndarray, lr: float) -> np.ndarray:
    return np.asarray(weight, dtype=np.float64) - lr * np.asarray(grad, dtype=np.float64)


def train_step(parts, x0, weights, acts, keep, key, step, labels, scale, lr, round_store=None):
    """One iteration of Algorithm 1 without the rate update: forward with compressed exchange, loss on every
    partition's labelled rows, backward, summed weight gradients, gradient step.
    labels[q]: integer labels of partition q's rows (< 0 = not a training node).
    Returns (new weights, loss, n_correct, forward state, backward state, dlogits per partition)."""
    rnd = (lambda a: a) if round_store is None else round_store
    fwd = _layer.network_forward(parts, x0, weights, acts, keep, key, step, round_store)
    loss, correct, dlast = 0.0, 0, []
    for p in parts:
        l_q, d_q, c_q = softmax_xent(fwd["x"][-1][p.q], labels[p.q], scale)
        loss += l_q
        correct += c_q
        dlast.append(rnd(d_q))
    bwd = _layer.network_backward(parts, fwd, weights, acts, keep, key, step, dlast, round_store)
    new_weights = []
    for (h1, h0), (g1, g0) in zip(weights, bwd["dh"]):
        new_weights.append((sgd(h1, g1, lr), sgd(h0, g0, lr) if h0 is not None else None))
    return new_weights, loss, correct, fwd, bwd, dlast

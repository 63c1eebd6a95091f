"""Oracle for model averaging across replicas (test infrastructure).

Sec. 3: each replica trains on its own data partition; every n minibatch updates the
parameters of all replicas are replaced by their mean (eqs. 1-2; the all-reduce of
Fig. 1 leaves every node with the same averaged model).
"""
from __future__ import annotations

import numpy as np

from . import dnn


def average_replicas(thetas: np.ndarray) -> np.ndarray:
    """thetas: K x P.  Returns K x P with every row = (1/K) * sum_k thetas[k]  (float64)."""
    thetas = np.asarray(thetas, dtype=np.float64)
    mean = thetas.sum(axis=0) / thetas.shape[0]
    return np.broadcast_to(mean, thetas.shape).copy()


def train_with_averaging(theta0, dims, shards, lr, n_avg, mean_grad=True, precondition=None,
                         trace=None):
    """Local SGD with periodic averaging.

    shards[k][t] = (X, y) is replica k's t-th minibatch.  All replicas start from theta0.
    After every n_avg-th minibatch the replicas are averaged.  Returns (K x P thetas, K x T losses).
    `trace`, if a list, receives a copy of the K x P parameters after every minibatch
    (after averaging when one happens).
    """
    K = len(shards)
    T = len(shards[0])
    thetas = np.tile(np.asarray(theta0, dtype=np.float64), (K, 1))
    losses = np.zeros((K, T))
    for t in range(T):
        for k in range(K):
            X, y = shards[k][t]
            pre = None if precondition is None else precondition[k]
            thetas[k], losses[k, t], _ = dnn.sgd_step(thetas[k], dims, X, y, lr, mean_grad, pre)
        if (t + 1) % n_avg == 0:
            thetas = average_replicas(thetas)
        if trace is not None:
            trace.append(thetas.copy())
    return thetas, losses

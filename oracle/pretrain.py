"""Oracle for greedy layer-wise RBM pretraining and the DNN initialisation from the stack (test infrastructure).

The paper (Sec. 5.1, Sec. 5.3) says only that the networks are initialised from a stack of restricted Boltzmann
machines trained layer by layer, the first one on the real-valued features; Table 2 compares that start with a
random one.  The procedure written out here is the usual one, with this build's readings:

  * RBM 1 is Gaussian-Bernoulli on the features, RBM l > 1 Bernoulli-Bernoulli on the hidden *probabilities*
    (not samples) of RBM l-1, computed with RBM l-1's final parameters;
  * every RBM takes `steps` CD-1 updates (oracle.rbm.cd1_step), minibatch t of the list at step t (cycled),
    Philox keys (seed, step t, layer l, phase), momentum buffers starting at zero, no sampling of the
    reconstruction;
  * DNN hidden layer l takes W_l <- W of RBM l, b_l <- its hidden bias c; visible biases are dropped; the
    softmax layer keeps whatever the caller put there (random).

All float64.
"""
from __future__ import annotations

import numpy as np

from . import rbm as orbm


def propagate(stack, X):
    """Hidden probabilities of the last RBM of `stack` for input rows X (X itself for an empty stack)."""
    A = np.asarray(X, np.float64)
    for (W, a, c) in stack:
        A = orbm.hidden_prob(A, W, c)
    return A


def pretrain_stack(widths, minibatches, init, steps, lr_gauss, lr_bern, momentum, seed):
    """widths = [d_0, d_1, ..., d_H]; minibatches: list of (n x d_0) arrays; init: list of (W, a, c) per RBM.

    Returns the trained stack [(W, a, c)] and, per RBM, the list of reconstruction errors."""
    stack, errs = [], []
    for l in range(1, len(widths)):
        W, a, c = (np.asarray(t, np.float64).copy() for t in init[l - 1])
        assert W.shape == (widths[l], widths[l - 1])
        MW, Ma, Mc = np.zeros_like(W), np.zeros_like(a), np.zeros_like(c)
        vis = orbm.GAUSSIAN if l == 1 else orbm.BERNOULLI
        lr = lr_gauss if l == 1 else lr_bern
        e = []
        for t in range(steps):
            V0 = propagate(stack, minibatches[t % len(minibatches)])
            W, a, c, MW, Ma, Mc, info = orbm.cd1_step(W, a, c, MW, Ma, Mc, V0, vis, lr, momentum, seed, t, l)
            e.append(info["recon_err"])
        stack.append((W, a, c))
        errs.append(e)
    return stack, errs


def init_dnn_from_stack(theta, dims, stack):
    """Copy of theta with hidden layer l = 1..len(stack) replaced by RBM l's (W, c)."""
    theta = np.asarray(theta, np.float64).copy()
    off = 0
    for l in range(1, len(dims)):
        nw = dims[l] * dims[l - 1]
        if l <= len(stack):
            W, _, c = stack[l - 1]
            assert W.shape == (dims[l], dims[l - 1])
            theta[off:off + nw] = np.asarray(W, np.float64).reshape(-1)
            theta[off + nw:off + nw + dims[l]] = np.asarray(c, np.float64)
        off += nw + dims[l]
    return theta

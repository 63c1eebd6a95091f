"""Greedy layer-wise RBM pretraining and DNN initialisation from the stack (paper Sec. 5.1, Sec. 5.3).

A host-side driver only: every CD-1 update, every propagation through the lower RBMs and the copy into the
network's parameter vector is a call of the HIP library (rbm_cd1_step, rbm_hidden_prob,
dnn_init_layer_from_rbm).  RBM 1 is Gaussian-Bernoulli on the features, RBM l > 1 Bernoulli-Bernoulli on the
hidden probabilities of RBM l-1; momentum buffers start at zero; Philox keys are (seed, step, layer, phase).
"""
from __future__ import annotations

import torch

from . import binding as B


def pretrain_stack(widths, minibatches, init, steps, lr_gauss, lr_bern, momentum, seed, stream=None):
    """widths = [d_0, ..., d_H]; minibatches: list of device tensors n x d_0; init: per RBM (W, a, c) device tensors
    (trained in place).  Returns the list of per-RBM device tensors of reconstruction errors (one float per step)."""
    n = minibatches[0].shape[0]
    dev = minibatches[0].device
    ws = torch.empty(max(B.rbm_workspace_bytes(widths[l - 1], widths[l], n) for l in range(1, len(widths))) + 256,
                     dtype=torch.uint8, device=dev)
    hidden = [None] + [torch.empty(n, widths[j], device=dev) for j in range(1, len(widths) - 1)]
    errs = []
    for l in range(1, len(widths)):
        W, a, c = init[l - 1]
        mw, ma, mc = torch.zeros_like(W), torch.zeros_like(a), torch.zeros_like(c)
        vis = B.VIS_GAUSSIAN if l == 1 else B.VIS_BERNOULLI
        lr = lr_gauss if l == 1 else lr_bern
        err = torch.zeros(steps, device=dev)
        for t in range(steps):
            v = minibatches[t % len(minibatches)]
            for j in range(1, l):                      # through the trained RBMs below
                B.rbm_hidden_prob(widths[j - 1], widths[j], init[j - 1][0], init[j - 1][2], v, n, hidden[j], ws, stream=stream)
                v = hidden[j]
            B.rbm_cd1_step(widths[l - 1], widths[l], vis, W, a, c, mw, ma, mc, v, n, lr, momentum, seed, t, l, 0,
                           err[t:t + 1], ws, stream=stream)
        errs.append(err)
    return errs


def init_dnn_from_stack(shape, k, theta, theta_stride, stack, stream=None):
    """Hidden layer l of all k replicas <- (W, c) of RBM l, for l = 1..len(stack)."""
    for l, (W, _, c) in enumerate(stack, start=1):
        B.dnn_init_layer_from_rbm(shape, k, theta, theta_stride, l, W, c, stream=stream)

"""Greedy layer-wise RBM pretraining and DNN initialisation from the stack (paper Sec. 5.1, Sec. 5.3).

A host-side driver only: every CD-1 update, every propagation through the lower RBMs and the copy into the
network's parameter vector is a call of the HIP library (rbm_cd1_step, rbm_hidden_prob,
dnn_init_layer_from_rbm).  RBM 1 is Gaussian-Bernoulli on the features, RBM l > 1 Bernoulli-Bernoulli on the
hidden probabilities of RBM l-1; momentum buffers start at zero; Philox keys are (seed, step, layer, phase).
"""
from __future__ import annotations

import time

import torch

from . import binding as B


def pretrain_stack(widths, minibatches, init, steps, lr_gauss, lr_bern, momentum, seed, stream=None, timings=False):
    """widths = [d_0, ..., d_H]; minibatches: list of device tensors n x d_0; init: per RBM (W, a, c) device tensors
    (trained in place).  Returns the list of per-RBM device tensors of reconstruction errors (one float per step);
    with timings=True, (that list, seconds spent on each RBM, measured between device synchronisations).

    The inputs of RBM l are the hidden probabilities of the trained RBM l-1 on the same minibatches.  Once an RBM is
    trained they do not change, so when the minibatch list is cycled (fewer distinct minibatches than steps) each
    level is propagated once per distinct minibatch and kept, instead of once per step."""
    n = minibatches[0].shape[0]
    dev = minibatches[0].device
    ws = torch.empty(max(B.rbm_workspace_bytes(widths[l - 1], widths[l], n) for l in range(1, len(widths))) + 256,
                     dtype=torch.uint8, device=dev)
    level = list(minibatches)                          # inputs of the RBM being trained, one per distinct minibatch
    errs, secs = [], []
    for l in range(1, len(widths)):
        if timings:
            torch.cuda.synchronize()
            t0 = time.perf_counter()
        W, a, c = init[l - 1]
        mw, ma, mc = torch.zeros_like(W), torch.zeros_like(a), torch.zeros_like(c)
        vis = B.VIS_GAUSSIAN if l == 1 else B.VIS_BERNOULLI
        lr = lr_gauss if l == 1 else lr_bern
        err = torch.zeros(steps, device=dev)
        for t in range(steps):
            B.rbm_cd1_step(widths[l - 1], widths[l], vis, W, a, c, mw, ma, mc, level[t % len(level)], n, lr, momentum, seed, t, l, 0,
                           err[t:t + 1], ws, stream=stream)
        errs.append(err)
        if l + 1 < len(widths):                        # through the RBM just trained: the next one's inputs
            nxt = [torch.empty(n, widths[l], device=dev) for _ in level]
            for v, h in zip(level, nxt):
                B.rbm_hidden_prob(widths[l - 1], widths[l], W, c, v, n, h, ws, stream=stream)
            level = nxt
        if timings:
            torch.cuda.synchronize()
            secs.append(time.perf_counter() - t0)
    return (errs, secs) if timings else errs


def init_dnn_from_stack(shape, k, theta, theta_stride, stack, stream=None):
    """Hidden layer l of all k replicas <- (W, c) of RBM l, for l = 1..len(stack)."""
    for l, (W, _, c) in enumerate(stack, start=1):
        B.dnn_init_layer_from_rbm(shape, k, theta, theta_stride, l, W, c, stream=stream)

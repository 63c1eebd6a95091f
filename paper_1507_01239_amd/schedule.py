"""Learning-rate schedules of the paper's Sec. 5.6 (host logic) and the held-out frame accuracy that drives
the first one (computed on the GPU by dnn_forward + dnn_count_correct).

Newbob: run at the initial rate until the gain in held-out frame accuracy (percent points) between two
successive epochs drops below 0.5; from then on halve the rate before every epoch, and stop once the gain
drops below 0.1.  Exponential: lr_e = lr_0 * 0.01^(e / (E - 1)), e = 0..E-1 (E = 15 in the paper).  With m
replicas under averaging the initial rate is m times the single-replica rate.
"""
from __future__ import annotations

import torch

from . import binding as B


class Newbob:
    def __init__(self, lr0, halve_below=0.5, stop_below=0.1):
        self.lr = float(lr0)
        self.halve_below, self.stop_below = halve_below, stop_below
        self.prev = None
        self.halving = False
        self.stopped = False

    def after_epoch(self, accuracy_percent):
        """Feed the held-out accuracy measured after the epoch just run; returns the rate of the next epoch
        (None when training is to stop)."""
        if self.stopped:
            return None
        gain = None if self.prev is None else accuracy_percent - self.prev
        self.prev = accuracy_percent
        if gain is not None:
            if self.halving and gain < self.stop_below:
                self.stopped = True
                return None
            if gain < self.halve_below:
                self.halving = True
            if self.halving:
                self.lr *= 0.5
        return self.lr


def exponential_rates(lr0, epochs=15, final_ratio=0.01):
    if epochs == 1:
        return [float(lr0)]
    step = final_ratio ** (1.0 / (epochs - 1))
    out, lr = [], float(lr0)
    for _ in range(epochs):
        out.append(lr)
        lr *= step
    return out


def scaled_initial_rate(lr_single, replicas):
    return lr_single * replicas


def frame_accuracy(shape, k, theta, theta_stride, x, x_stride, labels, label_stride, n, acts, act_stride, workspace,
                   stream=None):
    """Held-out frame accuracy of each of the k replicas on one batch: fractions as a host list."""
    correct = torch.zeros(k, dtype=torch.int32, device=acts.device)
    B.dnn_forward(shape, k, theta, theta_stride, x, x_stride, n, acts, act_stride, workspace, stream=stream)
    B.dnn_count_correct(shape, k, acts, act_stride, labels, label_stride, n, correct, stream=stream)
    return [c / n for c in correct.cpu().tolist()]

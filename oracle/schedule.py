"""Oracle for the two learning-rate schedules and the frame accuracy that drives one of them (test infrastructure).

Sec. 5.6 of the paper: (i) "Newbob": start from an initial rate; after each epoch measure the frame accuracy on
held-out data; once the gain over the previous epoch falls below 0.5 % (absolute, in percent) the rate is
halved for every following epoch, and training stops when the gain falls below 0.1 %; (ii) exponential decay
from the initial rate to 0.01 x initial over 15 epochs.  The initial rate is multiplied by the number of
replicas m when training with averaging.

Readings: gains are differences of accuracies in percent points; the halving is sticky (every epoch after the
first small gain halves again); the stop test applies only once halving has begun; the exponential schedule is
lr_e = lr_0 * 0.01^(e/(E-1)) for e = 0..E-1, so that epoch 0 runs at lr_0 and the last one at 0.01 lr_0.
"""
from __future__ import annotations

import numpy as np


def frame_accuracy(posteriors, labels):
    """Fraction of rows whose largest posterior (lowest index among equals) is the label's."""
    p = np.asarray(posteriors, np.float64)
    return float((np.argmax(p, axis=1) == np.asarray(labels)).mean())


def newbob(lr0, accuracies_percent, halve_below=0.5, stop_below=0.1):
    """Rates used for epochs 0, 1, ... given the held-out accuracy (percent) measured AFTER each epoch.

    Returns (rates, stopped_after): rates[e] is the rate epoch e ran at; training stops after epoch
    stopped_after (None if the list of accuracies ran out first)."""
    rates, lr, halving, prev = [], float(lr0), False, None
    for e, acc in enumerate(accuracies_percent):
        rates.append(lr)
        gain = None if prev is None else acc - prev
        prev = acc
        if gain is None:
            continue
        if halving and gain < stop_below:
            return rates, e
        if gain < halve_below:
            halving = True
        if halving:
            lr *= 0.5
    return rates, None


def exponential(lr0, epochs=15, final_ratio=0.01):
    return [float(lr0) * final_ratio ** (e / (epochs - 1)) for e in range(epochs)]


def scaled_initial_rate(lr_single, replicas):
    """Sec. 5.6: the single-replica rate times the number of replicas."""
    return lr_single * replicas

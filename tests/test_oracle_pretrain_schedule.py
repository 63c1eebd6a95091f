"""Pins of the pretraining-stack and schedule oracles (no GPU): brute force, closed forms, invariants and a
worked example of the schedule rule of the paper's Sec. 5.6."""
import math

import numpy as np

import gen
from oracle import dnn as odnn
from oracle import pretrain as opre
from oracle import rbm as orbm
from oracle import schedule as osch


def _tiny_stack(seed=3, widths=(6, 5, 4, 3), n=7, nmb=2):
    rng = np.random.default_rng(seed)
    mbs = [rng.standard_normal((n, widths[0])) for _ in range(nmb)]
    init = [(rng.standard_normal((widths[l], widths[l - 1])) * 0.3, rng.standard_normal(widths[l - 1]) * 0.1,
             rng.standard_normal(widths[l]) * 0.1) for l in range(1, len(widths))]
    return list(widths), mbs, init


def test_initialised_network_reproduces_the_stack_layer_by_layer():
    # brute force, element by element: hidden layer l of the initialised DNN must output what RBM l outputs on
    # the output of RBM l-1 (pins offsets, orientation of W and the use of the HIDDEN bias)
    widths, mbs, init = _tiny_stack()
    dims = widths + [5]
    theta0 = np.random.default_rng(0).standard_normal(sum(dims[l] * dims[l - 1] + dims[l] for l in range(1, len(dims))))
    theta = opre.init_dnn_from_stack(theta0, dims, init)
    X = mbs[0]
    A = X
    acts = odnn.forward(theta, dims, X)
    for l, (W, a, c) in enumerate(init, start=1):
        H = np.empty((X.shape[0], widths[l]))
        for n in range(X.shape[0]):
            for j in range(widths[l]):
                z = c[j]
                for i in range(widths[l - 1]):
                    z += W[j, i] * A[n, i]
                H[n, j] = 1.0 / (1.0 + math.exp(-z))
        assert np.allclose(acts[l - 1], H, rtol=1e-12, atol=1e-14)
        assert np.allclose(opre.propagate(init[:l], X), H, rtol=1e-12, atol=1e-14)
        A = H
    # the softmax layer is left as the caller had it
    last = dims[-1] * dims[-2] + dims[-1]
    assert np.array_equal(theta[-last:], theta0[-last:])


def test_training_is_greedy_and_degenerate_settings_change_nothing():
    widths, mbs, init = _tiny_stack()
    full, _ = opre.pretrain_stack(widths, mbs, init, 4, 0.01, 0.2, 0.9, seed=11)
    first_only, _ = opre.pretrain_stack(widths[:2], mbs, init[:1], 4, 0.01, 0.2, 0.9, seed=11)
    for u, v in zip(full[0], first_only[0]):          # upper RBMs never touch the lower ones
        assert np.array_equal(u, v)
    none, _ = opre.pretrain_stack(widths, mbs, init, 0, 0.01, 0.2, 0.9, seed=11)
    frozen, _ = opre.pretrain_stack(widths, mbs, init, 3, 0.0, 0.0, 0.9, seed=11)
    for l in range(3):
        for u, v, w in zip(init[l], none[l], frozen[l]):
            assert np.array_equal(u, v) and np.array_equal(u, w)


def test_second_rbm_sees_probabilities_of_the_trained_first_one_with_its_own_keys():
    widths, mbs, init = _tiny_stack()
    stack, _ = opre.pretrain_stack(widths, mbs, init, 2, 0.05, 0.3, 0.5, seed=5)
    # replay RBM 2 by hand: inputs are sigmoid(V W1^T + c1) with the FINAL W1, c1; Philox layer key 2, steps 0, 1
    W1, _, c1 = stack[0]
    W, a, c = (t.copy() for t in init[1])
    MW, Ma, Mc = np.zeros_like(W), np.zeros_like(a), np.zeros_like(c)
    for t in range(2):
        V0 = 1.0 / (1.0 + np.exp(-(mbs[t % 2] @ W1.T + c1[None, :])))
        W, a, c, MW, Ma, Mc, _ = orbm.cd1_step(W, a, c, MW, Ma, Mc, V0, orbm.BERNOULLI, 0.3, 0.5, 5, t, 2)
    assert np.allclose(stack[1][0], W, rtol=1e-13) and np.allclose(stack[1][2], c, rtol=1e-13)


def test_cd1_lowers_the_reconstruction_error_of_a_learnable_pattern():
    # two well separated binary prototypes: a few hundred CD-1 updates must reconstruct them far better than at the start
    rng = np.random.default_rng(2)
    protos = np.array([[1, 1, 1, 0, 0, 0, 1, 0], [0, 0, 0, 1, 1, 1, 0, 1]], float)
    mbs = [protos[rng.integers(0, 2, 16)] for _ in range(4)]
    init = [(rng.standard_normal((4, 8)) * 0.01, np.zeros(8), np.zeros(4))]
    _, errs = opre.pretrain_stack([8, 4], mbs, init, 200, 0.1, 0.1, 0.5, seed=1)
    assert np.mean(errs[0][-8:]) < 0.3 * np.mean(errs[0][:8])


def test_newbob_worked_example():
    # gains: +5, +3, +0.3 (< 0.5: halving starts), +0.3 (>= 0.1: go on, halve again), +0.05 (< 0.1: stop)
    rates, stopped = osch.newbob(0.32, [40.0, 45.0, 48.0, 48.3, 48.6, 48.65, 60.0])
    assert rates == [0.32, 0.32, 0.32, 0.32, 0.16, 0.08]
    assert stopped == 5
    # a small gain before any halving halves but does not stop, however small
    rates, stopped = osch.newbob(1.0, [10.0, 10.01, 20.0, 20.05])
    assert rates == [1.0, 1.0, 0.5, 0.25] and stopped == 3
    # never below the thresholds: constant rate, no stop
    rates, stopped = osch.newbob(0.32, [10, 20, 30, 40])
    assert rates == [0.32] * 4 and stopped is None


def test_exponential_schedule_closed_form():
    r = osch.exponential(0.32, 15, 0.01)
    assert len(r) == 15 and r[0] == 0.32 and math.isclose(r[-1], 0.0032, rel_tol=1e-12)
    ratios = [r[i + 1] / r[i] for i in range(14)]
    assert np.allclose(ratios, 0.01 ** (1 / 14), rtol=1e-12)
    assert osch.scaled_initial_rate(0.008, 16) == 0.128


def test_frame_accuracy_brute_force_with_ties():
    p = np.array([[0.2, 0.5, 0.3], [0.4, 0.4, 0.2], [0.1, 0.1, 0.8], [0.3, 0.3, 0.4]])
    y = np.array([1, 1, 2, 0])           # row 1: tie between 0 and 1 -> lowest index 0 wins -> wrong
    hits = 0
    for n in range(4):
        best = 0
        for j in range(1, 3):
            if p[n, j] > p[n, best]:
                best = j
        hits += best == y[n]
    assert hits == 2 and osch.frame_accuracy(p, y) == 0.5

"""Pins for the DNN and averaging oracle (no GPU): each checks oracle/ against something that is not
the oracle itself -- finite differences, an autograd library, closed forms, and the identities of
Sec. 3 of the paper."""
import math
import os

import numpy as np
import pytest
import torch

import gen
from oracle import averaging, dnn

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _tiny(seed=0, dims=(5, 4, 3, 3), n=3, w_std=0.7):
    rng = np.random.default_rng(seed)
    theta = rng.standard_normal(dnn.param_count(dims)) * w_std
    X = rng.standard_normal((n, dims[0]))
    y = rng.integers(0, dims[-1], n)
    return theta, X, y


def test_param_count_matches_hand_arithmetic():
    # Sec. 5.1 topology; totals worked by hand in the fixture
    for line in open(os.path.join(GOLDEN, "topology_param_count.txt")):
        if line.startswith("#") or not line.strip():
            continue
        lhs, rhs = line.split("->")
        dims = tuple(int(t) for t in lhs.split())
        assert dnn.param_count(dims) == int(rhs)
        assert gen.param_count(dims) == int(rhs)


@pytest.mark.parametrize("mean", [True, False])
@pytest.mark.parametrize("dims", [(5, 4, 3, 3), (4, 6), (3, 5, 4, 2, 6)])
def test_gradient_matches_central_differences(dims, mean):
    theta, X, y = _tiny(1, dims, n=4)
    g, _ = dnn.gradient(theta, dims, X, y, mean_grad=mean)
    h = 1e-5
    fd = np.zeros_like(theta)
    for i in range(theta.size):
        tp, tm = theta.copy(), theta.copy()
        tp[i] += h
        tm[i] -= h
        fd[i] = (dnn.loss_only(tp, dims, X, y, mean) - dnn.loss_only(tm, dims, X, y, mean)) / (2 * h)
    assert np.max(np.abs(fd - g)) <= 1e-7 * max(1.0, np.max(np.abs(g)))
    assert np.linalg.norm(fd - g) <= 1e-7 * np.linalg.norm(g)


@pytest.mark.parametrize("dims", [(5, 4, 3, 3), (3, 5, 4, 2, 6)])
def test_tanh_variant_gradient_matches_central_differences_and_a_rescaled_sigmoid_network(dims):
    theta, X, y = _tiny(7, dims, n=4)
    g, _ = dnn.gradient(theta, dims, X, y, mean_grad=True, hidden="tanh")
    h = 1e-5
    fd = np.zeros_like(theta)
    for i in range(theta.size):
        tp, tm = theta.copy(), theta.copy()
        tp[i] += h
        tm[i] -= h
        fd[i] = (dnn.loss_only(tp, dims, X, y, True, hidden="tanh") - dnn.loss_only(tm, dims, X, y, True, hidden="tanh")) / (2 * h)
    assert np.linalg.norm(fd - g) <= 1e-7 * np.linalg.norm(g)
    # closed form: tanh(z) = 2 sigmoid(2z) - 1, so the tanh network equals a sigmoid network whose hidden
    # layers have their weights and biases doubled and whose next layer sees 2 a - 1:
    # W'_1 = 2 W_1, b'_1 = 2 b_1; for l > 1: W'_l = s_l * 2 W_l, b'_l = s_l (b_l - W_l 1), s_l = 2 (hidden) or 1 (softmax)
    layers = dnn.unpack(theta, dims)
    t2 = theta.copy()
    l2 = dnn.unpack(t2, dims)
    L = len(layers)
    for l, ((W, b), (W2, b2)) in enumerate(zip(layers, l2), start=1):
        s_out = 2.0 if l < L else 1.0
        if l == 1:
            W2[:, :] = s_out * W
            b2[:] = s_out * b
        else:
            W2[:, :] = s_out * 2.0 * W
            b2[:] = s_out * (b - W.sum(axis=1))
    np.testing.assert_allclose(dnn.forward(theta, dims, X, hidden="tanh")[-1], dnn.forward(t2, dims, X)[-1], rtol=1e-11, atol=1e-14)


def test_gradient_and_loss_match_autograd_library():
    dims = (7, 6, 5, 9)
    theta, X, y = _tiny(2, dims, n=11)
    t = torch.tensor(theta, dtype=torch.float64, requires_grad=True)
    a = torch.tensor(X, dtype=torch.float64)
    off = 0
    for l in range(1, len(dims)):
        nw = dims[l] * dims[l - 1]
        W = t[off:off + nw].reshape(dims[l], dims[l - 1])
        b = t[off + nw:off + nw + dims[l]]
        off += nw + dims[l]
        z = torch.nn.functional.linear(a, W, b)
        a = torch.sigmoid(z) if l < len(dims) - 1 else z
    loss = torch.nn.functional.cross_entropy(a, torch.tensor(y, dtype=torch.long), reduction="sum")
    loss.backward()
    g, loss_sum = dnn.gradient(theta, dims, X, y, mean_grad=False)
    assert abs(loss_sum - loss.item()) <= 1e-12 * abs(loss.item())
    np.testing.assert_allclose(g, t.grad.numpy(), rtol=1e-10, atol=1e-13)
    gm, _ = dnn.gradient(theta, dims, X, y, mean_grad=True)
    np.testing.assert_allclose(gm * X.shape[0], t.grad.numpy(), rtol=1e-10, atol=1e-13)
    p_ref = torch.softmax(a, dim=1).detach().numpy()
    np.testing.assert_allclose(dnn.forward(theta, dims, X)[-1], p_ref, rtol=1e-12, atol=1e-15)


def test_softmax_identities():
    dims = (6, 5, 8)
    theta, X, y = _tiny(3, dims, n=9)
    acts = dnn.forward(theta, dims, X)
    p = acts[-1]
    np.testing.assert_allclose(p.sum(axis=1), 1.0, rtol=0, atol=1e-14)
    assert np.all(p > 0)
    for mean in (True, False):
        d = dnn.output_delta(p, y, mean)
        np.testing.assert_allclose(d.sum(axis=1), 0.0, atol=1e-15)
    # shift invariance: adding a constant to every output bias leaves the posteriors unchanged
    th2 = theta.copy()
    th2[-dims[-1]:] += 3.25
    np.testing.assert_allclose(dnn.forward(th2, dims, X)[-1], p, rtol=1e-12)
    # large logits do not overflow
    th3 = theta.copy()
    th3[-dims[-1]:] += 5000.0
    assert np.all(np.isfinite(dnn.forward(th3, dims, X)[-1]))


@pytest.mark.parametrize("classes", [32, 8000])
def test_uniform_logits_give_log_classes(classes):
    dims = (4, 3, classes)
    n = 5
    theta = np.zeros(dnn.param_count(dims))
    X = np.random.default_rng(0).standard_normal((n, 4))
    y = np.arange(n) % classes
    loss = dnn.cross_entropy_sum(dnn.forward(theta, dims, X)[-1], y)
    assert abs(loss - n * math.log(classes)) < 1e-10
    # printed values of ln 32 and ln 8000
    assert abs(loss / n - {32: 3.4657359, 8000: 8.9871968}[classes]) < 1e-6


def test_bias_gradient_equals_weight_gradient_of_a_ones_column():
    dims = (5, 4, 3)
    theta, X, y = _tiny(4, dims, n=6)
    g, _ = dnn.gradient(theta, dims, X, y)
    # same first layer written with the bias folded into an extra all-ones input column
    dims2 = (6, 4, 3)
    (W1, b1), (W2, b2) = dnn.unpack(theta, dims)
    th2 = np.concatenate([np.concatenate([W1, b1[:, None]], axis=1).ravel(), np.zeros(4), W2.ravel(), b2])
    X2 = np.concatenate([X, np.ones((6, 1))], axis=1)
    g2, _ = dnn.gradient(th2, dims2, X2, y)
    G1aug = dnn.unpack(g2, dims2)[0][0]
    np.testing.assert_allclose(G1aug[:, -1], dnn.unpack(g, dims)[0][1], rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(G1aug[:, :-1], dnn.unpack(g, dims)[0][0], rtol=1e-12, atol=1e-15)


def test_zero_learning_rate_is_identity_and_step_descends():
    dims = (5, 4, 3, 3)
    theta, X, y = _tiny(5, dims, n=8)
    th, _, _ = dnn.sgd_step(theta, dims, X, y, 0.0)
    assert np.array_equal(th, theta)
    before = dnn.loss_only(theta, dims, X, y)
    th, loss_sum, _ = dnn.sgd_step(theta, dims, X, y, 1e-3)
    assert abs(loss_sum / 8 - before) < 1e-12
    assert dnn.loss_only(th, dims, X, y) < before    # eq. 3 moves along the ascent direction of -loss


def test_single_layer_step_is_multinomial_logistic_regression():
    # one affine + softmax layer with two classes: p(class 1) = logistic(w.x + b) with w = W[1]-W[0];
    # the step on W[1]-W[0] must equal 2x the textbook binary logistic-regression step lr * mean((t - q) x)
    dims = (3, 2)
    rng = np.random.default_rng(6)
    theta = rng.standard_normal(dnn.param_count(dims))
    X = rng.standard_normal((10, 3))
    y = rng.integers(0, 2, 10)
    lr = 0.3
    th, _, _ = dnn.sgd_step(theta, dims, X, y, lr)
    (W, b), (Wn, bn) = dnn.unpack(theta, dims)[0], dnn.unpack(th, dims)[0]
    w, wn = W[1] - W[0], Wn[1] - Wn[0]
    q = 1.0 / (1.0 + np.exp(-(X @ w + (b[1] - b[0]))))
    expect = w + 2 * lr * ((y - q)[:, None] * X).mean(axis=0)
    np.testing.assert_allclose(wn, expect, rtol=1e-12)


# ---- Sec. 3: averaging ---------------------------------------------------------------------------

def _shards(dims, K, T, n, seed):
    return [[(gen.features_iid(n, dims[0], seed, k, t), gen.labels_uniform(n, dims[-1], seed, k, t))
             for t in range(T)] for k in range(K)]


def test_averaging_every_update_equals_gradient_averaging():
    # Sec. 3: with averaging after each update, model averaging is gradient averaging, i.e. one
    # mean-gradient step on the concatenation of the K shards' minibatches
    dims, K, n = gen.CONFIG_TINY_DIMS, 4, 32
    theta0 = gen.init_theta(dims, 11, 0.1)
    shards = _shards(dims, K, 3, n, 11)
    thetas, _ = averaging.train_with_averaging(theta0, dims, shards, 0.1, 1)
    ref = theta0.astype(np.float64)
    for t in range(3):
        Xc = np.concatenate([shards[k][t][0] for k in range(K)])
        yc = np.concatenate([shards[k][t][1] for k in range(K)])
        ref, _, _ = dnn.sgd_step(ref, dims, Xc, yc, 0.1, mean_grad=True)
    for k in range(K):
        np.testing.assert_allclose(thetas[k], ref, rtol=0, atol=1e-13)


def test_average_is_mean_of_accumulated_updates():
    # eqs. 1-2: theta_bar(t+n) - theta_bar(t) = mean over replicas of the sum of their n updates
    dims, K, n_avg = (6, 5, 4), 3, 4
    theta0 = gen.init_theta(dims, 5, 0.3)
    shards = _shards(dims, K, n_avg, 7, 5)
    thetas, _ = averaging.train_with_averaging(theta0, dims, shards, 0.2, n_avg)
    acc = np.zeros((K, theta0.size))
    for k in range(K):
        th = theta0.astype(np.float64)
        for t in range(n_avg):
            g, _ = dnn.gradient(th, dims, *shards[k][t])
            acc[k] += -0.2 * g
            th = th - 0.2 * g
    np.testing.assert_allclose(thetas[0], theta0 + acc.mean(axis=0), rtol=0, atol=1e-14)
    assert all(np.array_equal(thetas[0], thetas[k]) for k in range(K))


def test_averaging_identities():
    rng = np.random.default_rng(7)
    v = rng.standard_normal(1000).astype(np.float32)
    for K in (1, 2, 3, 4, 8):
        out = averaging.average_replicas(np.tile(v, (K, 1)))
        np.testing.assert_allclose(out, np.tile(v.astype(np.float64), (K, 1)), rtol=1e-15)
    th = rng.standard_normal((5, 257))
    once = averaging.average_replicas(th)
    np.testing.assert_allclose(averaging.average_replicas(once), once, rtol=1e-15)
    np.testing.assert_allclose(averaging.average_replicas(th[::-1]), once, rtol=1e-14)
    exact = np.array([math.fsum(th[:, j]) / 5 for j in range(257)])
    np.testing.assert_allclose(once[2], exact, rtol=1e-14, atol=1e-16)


def test_generators_are_deterministic_and_shaped():
    a = gen.features_speech_like(16, 440, 3, 1, 2)
    b = gen.features_speech_like(16, 440, 3, 1, 2)
    assert a.dtype == np.float32 and a.shape == (16, 440) and np.array_equal(a, b)
    assert not np.array_equal(a, gen.features_speech_like(16, 440, 3, 1, 3))
    lab = gen.labels_zipf(200000, 8000, 3, 0, 0)
    assert lab.dtype == np.int32 and lab.min() >= 0 and lab.max() < 8000
    cdf = gen.zipf_cdf(8000)
    assert abs(cdf[0] - 0.1535) < 2e-3                     # top-class mass of Zipf(1.1) on 8000 ranks
    assert abs((lab == 0).mean() - cdf[0]) < 5e-3
    th = gen.init_theta(gen.CONFIG_TINY_DIMS, 1, 0.1)
    assert th.dtype == np.float32 and th.size == 8864
    assert np.all(dnn.unpack(th, gen.CONFIG_TINY_DIMS)[0][1] == 0)

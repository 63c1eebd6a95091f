"""Oracle for one minibatch-SGD step of the fully connected DNN (test infrastructure).

Network (Sec. 5.1): input -> sigmoid hidden layers -> softmax output, trained by
minibatch SGD on the cross-entropy against the target class.  Update rule: eq. 3,
theta <- theta + alpha * g with g the ascent direction of the objective, i.e.
theta <- theta - lr * d(loss)/d(theta) for loss = cross-entropy.

Parameter vector layout: [W_1 | b_1 | W_2 | b_2 | ...], W_l is d_l x d_{l-1}
row-major (row = output unit).  Everything is float64.
"""
from __future__ import annotations

import numpy as np


def param_count(dims) -> int:
    return int(sum(dims[l] * dims[l - 1] + dims[l] for l in range(1, len(dims))))


def unpack(theta: np.ndarray, dims):
    """Views (W_l, b_l) for l = 1..L into the flat vector."""
    out, off = [], 0
    for l in range(1, len(dims)):
        nw = dims[l] * dims[l - 1]
        W = theta[off:off + nw].reshape(dims[l], dims[l - 1])
        b = theta[off + nw:off + nw + dims[l]]
        out.append((W, b))
        off += nw + dims[l]
    assert off == theta.shape[0]
    return out


def sigmoid(z: np.ndarray) -> np.ndarray:
    return 1.0 / (1.0 + np.exp(-z))


def softmax_rows(z: np.ndarray) -> np.ndarray:
    e = np.exp(z - z.max(axis=1, keepdims=True))
    return e / e.sum(axis=1, keepdims=True)


def hidden_activation(z, hidden):
    """Sec. 5.1 names both: tanh hidden units in one sentence, sigmoids in the next.  Sigmoid is this build's
    reading for every benchmarked configuration; tanh is kept as the variant."""
    if hidden == "tanh":
        return np.tanh(z)
    assert hidden == "sigmoid"
    return sigmoid(z)


def hidden_derivative(a, hidden):
    """d activation / d pre-activation, written in terms of the activation a."""
    return (1.0 - a * a) if hidden == "tanh" else a * (1.0 - a)


def forward(theta, dims, X, hidden="sigmoid"):
    """Activations [A_1, ..., A_L]; A_l = act(A_{l-1} W_l^T + b_l), A_L = softmax posteriors."""
    theta = np.asarray(theta, dtype=np.float64)
    A = np.asarray(X, dtype=np.float64)
    acts = []
    layers = unpack(theta, dims)
    for l, (W, b) in enumerate(layers, start=1):
        Z = A @ W.T + b[None, :]
        A = softmax_rows(Z) if l == len(layers) else hidden_activation(Z, hidden)
        acts.append(A)
    return acts


def cross_entropy_sum(p: np.ndarray, y: np.ndarray) -> float:
    """Summed (not averaged) cross-entropy  -sum_n log p[n, y_n]."""
    return float(-np.log(p[np.arange(p.shape[0]), y]).sum())


def output_delta(p: np.ndarray, y: np.ndarray, mean_grad: bool) -> np.ndarray:
    """d(loss*s)/dZ_L = s * (p - onehot(y)); s = 1/N for the mean-gradient convention, else 1."""
    d = p.copy()
    d[np.arange(p.shape[0]), y] -= 1.0
    return d / p.shape[0] if mean_grad else d


def gradient(theta, dims, X, y, acts=None, mean_grad=True, precondition=None, hidden="sigmoid"):
    """Flat gradient of the (mean or summed) cross-entropy w.r.t. theta, and the summed loss.

    precondition, if given, is a callable (layer l, A_in_aug [N x (d_{l-1}+1)], delta_l [N x d_l])
    -> (A_in_aug_hat, delta_hat) applied to the two factors of each layer's gradient before they
    are multiplied (NG-SGD, eq. 4); the delta that is propagated downwards stays untouched.
    """
    theta = np.asarray(theta, dtype=np.float64)
    X = np.asarray(X, dtype=np.float64)
    y = np.asarray(y)
    if acts is None:
        acts = forward(theta, dims, X, hidden)
    layers = unpack(theta, dims)
    L = len(layers)
    grad = np.zeros_like(theta)
    glayers = unpack(grad, dims)
    delta = output_delta(acts[-1], y, mean_grad)
    for l in range(L, 0, -1):
        A_in = X if l == 1 else acts[l - 2]
        W, _ = layers[l - 1]
        GW, Gb = glayers[l - 1]
        if precondition is None:
            GW[:, :] = delta.T @ A_in
            Gb[:] = delta.sum(axis=0)
        else:
            aug = np.concatenate([A_in, np.ones((A_in.shape[0], 1))], axis=1)
            aug_h, delta_h = precondition(l, aug, delta)
            G = delta_h.T @ aug_h
            GW[:, :] = G[:, :-1]
            Gb[:] = G[:, -1]
        if l > 1:
            delta = (delta @ W) * hidden_derivative(A_in, hidden)
    return grad, cross_entropy_sum(acts[-1], y)


def sgd_step(theta, dims, X, y, lr, mean_grad=True, precondition=None, hidden="sigmoid"):
    """One update theta - lr * gradient (eq. 3).  Returns (new theta, summed loss, activations)."""
    theta = np.asarray(theta, dtype=np.float64)
    acts = forward(theta, dims, X, hidden)
    g, loss = gradient(theta, dims, X, y, acts, mean_grad, precondition, hidden)
    return theta - lr * g, loss, acts


def loss_only(theta, dims, X, y, mean=True, hidden="sigmoid") -> float:
    """Scalar objective whose gradient `gradient` returns (used by finite-difference pins)."""
    p = forward(theta, dims, X, hidden)[-1]
    s = cross_entropy_sum(p, np.asarray(y))
    return s / X.shape[0] if mean else s

"""Seeded synthetic stand-ins for the paper's training data (Sec. 5.1).

The paper trains on 440-dimensional spliced speech features (11 frames x 40)
with several thousand tied-state targets; that data is not available here.
These generators produce arrays with the same shapes and a comparable value
distribution: Gaussian features with per-dimension mean and spread, and class
labels with a heavy-tailed (Zipf) prior.

Everything is a pure function of (seed, stream ids): the same arguments give
the same bytes.  All arrays are returned in the dtypes the C ABI takes
(float32 / int32); the oracle widens them to float64 itself.
"""
from __future__ import annotations

import numpy as np

# Layer widths d_0..d_L.
CONFIG_TINY_DIMS = (40, 64, 64, 32)
CONFIG_FULL_DIMS = (440, 2048, 2048, 2048, 2048, 2048, 2048, 8000)
# Topology as stated in Sec. 5.1 of the paper (8806 outputs).
CONFIG_PAPER_DIMS = (440, 2048, 2048, 2048, 2048, 2048, 2048, 8806)

# Stream ids (first sub-stream key) so different purposes never share draws.
_S_THETA, _S_FEAT_STATS, _S_FEAT, _S_LABEL, _S_RBM, _S_MISC = 1, 2, 3, 4, 5, 6


def stream(seed: int, *ids: int) -> np.random.Generator:
    """A reproducible generator for (seed, ids...)."""
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(seed), *map(int, ids)])))


def param_count(dims) -> int:
    """Length of the flat parameter vector [W1|b1|W2|b2|...], W_l is d_l x d_{l-1}."""
    return int(sum(dims[l] * dims[l - 1] + dims[l] for l in range(1, len(dims))))


def init_theta(dims, seed: int, w_std: float) -> np.ndarray:
    """Flat float32 parameter vector: weights N(0, w_std^2), biases 0."""
    g = stream(seed, _S_THETA)
    out = np.zeros(param_count(dims), dtype=np.float32)
    off = 0
    for l in range(1, len(dims)):
        nw = dims[l] * dims[l - 1]
        out[off:off + nw] = (g.standard_normal(nw) * w_std).astype(np.float32)
        off += nw + dims[l]
    return out


def features_iid(n: int, dim: int, seed: int, replica: int, minibatch: int) -> np.ndarray:
    """n x dim features, iid N(0,1)."""
    g = stream(seed, _S_FEAT, replica, minibatch)
    return g.standard_normal((n, dim)).astype(np.float32)


def feature_stats(dim: int, seed: int):
    """Per-dimension mean ~ U(-1,1) and standard deviation ~ U(0.5,2)."""
    g = stream(seed, _S_FEAT_STATS)
    mu = g.uniform(-1.0, 1.0, dim)
    sd = g.uniform(0.5, 2.0, dim)
    return mu, sd


def features_speech_like(n: int, dim: int, seed: int, replica: int, minibatch: int) -> np.ndarray:
    """n x dim Gaussian features x = mu_j + sd_j * N(0,1) with the per-dimension stats of `seed`."""
    mu, sd = feature_stats(dim, seed)
    g = stream(seed, _S_FEAT, replica, minibatch)
    return (mu[None, :] + sd[None, :] * g.standard_normal((n, dim))).astype(np.float32)


def labels_uniform(n: int, classes: int, seed: int, replica: int, minibatch: int) -> np.ndarray:
    g = stream(seed, _S_LABEL, replica, minibatch)
    return g.integers(0, classes, n).astype(np.int32)


def zipf_cdf(classes: int, s: float = 1.1) -> np.ndarray:
    """CDF of P(rank r) ~ r^-s on ranks 1..classes (class id = rank - 1)."""
    w = np.arange(1, classes + 1, dtype=np.float64) ** (-s)
    c = np.cumsum(w)
    return c / c[-1]


def labels_zipf(n: int, classes: int, seed: int, replica: int, minibatch: int, s: float = 1.1) -> np.ndarray:
    """n labels with a Zipf(s) prior over `classes` classes, by inverse CDF."""
    g = stream(seed, _S_LABEL, replica, minibatch)
    u = g.random(n)
    idx = np.searchsorted(zipf_cdf(classes, s), u, side="right")
    return np.minimum(idx, classes - 1).astype(np.int32)


def rbm_params(n_vis: int, n_hid: int, seed: int, layer: int, w_std: float = 0.05):
    """(W [n_hid x n_vis], a [n_vis], c [n_hid]) float32: W ~ N(0, w_std^2), biases 0."""
    g = stream(seed, _S_RBM, layer)
    w = (g.standard_normal((n_hid, n_vis)) * w_std).astype(np.float32)
    return w, np.zeros(n_vis, np.float32), np.zeros(n_hid, np.float32)


def rbm_binary_input(n: int, dim: int, seed: int, minibatch: int) -> np.ndarray:
    """n x dim values in (0,1), shaped like the hidden probabilities a stacked RBM is fed with."""
    g = stream(seed, _S_MISC, minibatch)
    return g.beta(0.5, 0.5, (n, dim)).astype(np.float32)

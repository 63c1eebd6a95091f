"""Pins for the Philox and CD-1 oracle (no GPU)."""
import itertools
import os

import numpy as np
import pytest

from oracle import philox, rbm

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_philox_known_answers():
    for line in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(t, 16) for t in line.split()]
        out = philox.philox4x32_10(w[0], w[1], w[2], w[3], w[4], w[5])
        assert [int(x) for x in out] == w[6:]


def test_philox_vectorised_equals_scalar_calls():
    rng = np.random.default_rng(0)
    c = rng.integers(0, 2**32, (4, 50), dtype=np.uint64)
    out = philox.philox4x32_10(c[0], c[1], c[2], c[3], 123, 456)
    for i in (0, 17, 49):
        one = philox.philox4x32_10(int(c[0, i]), int(c[1, i]), int(c[2, i]), int(c[3, i]), 123, 456)
        assert [int(o[i]) for o in out] == [int(o) for o in one]


def test_uniforms_layout_range_and_streams():
    seed = 0x1234567887654321
    u = philox.uniforms(1 << 16, seed, 3, 1, 0)
    assert u.min() >= 0.0 and u.max() < 1.0
    assert np.array_equal(u.astype(np.float32).astype(np.float64), u)       # exact in float32
    # element e uses word e&3 of the block with counter word0 = e>>2
    blk = philox.philox4x32_10(5, 3, 1, 0, seed & 0xFFFFFFFF, seed >> 32)
    for j in range(4):
        assert u[20 + j] == (int(blk[j]) >> 8) / 2.0**24
    # statistics of a uniform
    assert abs(u.mean() - 0.5) < 4 * np.sqrt(1 / 12 / u.size)
    assert abs(u.var() - 1 / 12) < 2e-3
    hist = np.bincount((u * 256).astype(int), minlength=256)
    chi2 = ((hist - u.size / 256) ** 2 / (u.size / 256)).sum()
    assert chi2 < 255 + 5 * np.sqrt(2 * 255)
    # distinct (step, layer, phase, seed) give distinct streams
    for other in (philox.uniforms(4096, seed, 4, 1, 0), philox.uniforms(4096, seed, 3, 2, 0),
                  philox.uniforms(4096, seed, 3, 1, 1), philox.uniforms(4096, seed + 1, 3, 1, 0),
                  philox.uniforms(4096, seed + (1 << 32), 3, 1, 0)):
        assert (other == u[:4096]).mean() < 0.01


def _brute_force_expectation(W, a, c, v0, vis_type, sample_v1):
    """Exact E[dW], E[da], E[dc] and their per-sample variances for a single training vector v0 by
    enumerating every hidden configuration (and every visible one when V1 is sampled)."""
    H, V = W.shape
    sig = lambda z: 1.0 / (1.0 + np.exp(-z))
    ph0 = sig(W @ v0 + c)
    m1 = {k: 0.0 for k in ("dW", "da", "dc")}
    m2 = {k: 0.0 for k in ("dW", "da", "dc")}
    total = 0.0
    for h in itertools.product((0.0, 1.0), repeat=H):
        h = np.array(h)
        pr_h = np.prod(np.where(h == 1.0, ph0, 1.0 - ph0))
        pre = W.T @ h + a
        if vis_type == rbm.GAUSSIAN:
            outcomes = [(pre, 1.0)]
        elif not sample_v1:
            outcomes = [(sig(pre), 1.0)]
        else:
            pv = sig(pre)
            outcomes = []
            for v in itertools.product((0.0, 1.0), repeat=V):
                v = np.array(v)
                outcomes.append((v, np.prod(np.where(v == 1.0, pv, 1.0 - pv))))
        for v1, pr_v in outcomes:
            pr = pr_h * pr_v
            ph1 = sig(W @ v1 + c)
            st = dict(dW=np.outer(ph0, v0) - np.outer(ph1, v1), da=v0 - v1, dc=ph0 - ph1)
            for k in st:
                m1[k] = m1[k] + pr * st[k]
                m2[k] = m2[k] + pr * st[k] ** 2
            total += pr
    assert abs(total - 1.0) < 1e-12
    return m1, {k: np.maximum(m2[k] - m1[k] ** 2, 0.0) for k in m1}


@pytest.mark.parametrize("vis_type,sample_v1", [(rbm.BERNOULLI, False), (rbm.BERNOULLI, True), (rbm.GAUSSIAN, False)])
def test_cd1_statistics_converge_to_brute_force_expectation(vis_type, sample_v1):
    rng = np.random.default_rng(5)
    V, H, M = 4, 3, 200000
    W = rng.standard_normal((H, V)) * 0.8
    a = rng.standard_normal(V) * 0.3
    c = rng.standard_normal(H) * 0.3
    v0 = rng.standard_normal(V) if vis_type == rbm.GAUSSIAN else rng.integers(0, 2, V).astype(float)
    mean, var = _brute_force_expectation(W, a, c, v0, vis_type, sample_v1)
    # M independent draws = M identical rows of one minibatch: the minibatch mean IS the Monte-Carlo mean
    V0 = np.tile(v0, (M, 1))
    u_h = philox.uniforms(M * H, 99, 7, 2, 0).reshape(M, H)
    u_v = philox.uniforms(M * V, 99, 7, 2, 1).reshape(M, V) if sample_v1 else None
    s = rbm.cd1_statistics(W, a, c, V0, vis_type, u_h, u_v)
    for k in ("dW", "da", "dc"):
        tol = 4.5 * np.sqrt(var[k] / M) + 1e-12
        assert np.all(np.abs(s[k] - mean[k]) <= tol), k
        # and it is a genuine Monte-Carlo estimate, not the expectation itself
    assert np.any(np.abs(s["dW"] - mean["dW"]) > 1e-9)


def test_bernoulli_sampler_frequencies_and_extremes():
    H, N = 6, 100000
    W = np.zeros((H, 2))
    c = np.array([-800.0, -2.0, -0.3, 0.0, 1.5, 40.0])       # sigmoid(-800) == 0.0, sigmoid(40) == 1.0 in float64
    V0 = np.zeros((N, 2))
    u = philox.uniforms(N * H, 4, 0, 0, 0).reshape(N, H)
    with np.errstate(over="ignore"):
        s = rbm.cd1_statistics(W, np.zeros(2), c, V0, rbm.BERNOULLI, u)
        p = 1.0 / (1.0 + np.exp(-c))
    assert p[0] == 0.0 and p[-1] == 1.0
    f = s["H0"].mean(axis=0)
    assert f[0] == 0.0 and f[-1] == 1.0                         # u < 0 never, u < 1 always
    assert np.all(np.abs(f - p) <= 4.5 * np.sqrt(p * (1 - p) / N) + 1e-15)
    assert set(np.unique(s["H0"])) <= {0.0, 1.0}


@pytest.mark.parametrize("vis_type", [rbm.GAUSSIAN, rbm.BERNOULLI])
def test_zero_weights_closed_form(vis_type):
    # W = 0: hidden probabilities are sigmoid(c) whatever the data, the reconstruction is a (or sigmoid(a)),
    # so dc = 0, da = mean(V0) - V1, dW = sigmoid(c) (x) da  -- independent of the uniforms
    rng = np.random.default_rng(8)
    N, V, H = 13, 5, 4
    a, c = rng.standard_normal(V), rng.standard_normal(H)
    V0 = rng.standard_normal((N, V))
    for seed in (1, 2):
        W2, a2, c2, MW, Ma, Mc, s = rbm.cd1_step(np.zeros((H, V)), a, c, np.zeros((H, V)), np.zeros(V), np.zeros(H),
                                                 V0, vis_type, 0.5, 0.0, seed, 0, 0)
        v1 = a if vis_type == rbm.GAUSSIAN else 1 / (1 + np.exp(-a))
        da = V0.mean(axis=0) - v1
        np.testing.assert_allclose(s["dc"], 0.0, atol=1e-15)
        np.testing.assert_allclose(s["da"], da, rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(s["dW"], np.outer(1 / (1 + np.exp(-c)), da), rtol=1e-12, atol=1e-15)
        # momentum 0: plain step on the CD statistic
        np.testing.assert_allclose(W2, 0.5 * s["dW"], rtol=1e-14)
        np.testing.assert_allclose(a2, a + 0.5 * da, rtol=1e-12)
        assert abs(s["recon_err"] - ((V0 - v1[None, :]) ** 2).sum()) < 1e-10


def test_momentum_recursion_and_zero_lr():
    rng = np.random.default_rng(9)
    N, V, H = 6, 4, 3
    W, a, c = rng.standard_normal((H, V)), rng.standard_normal(V), rng.standard_normal(H)
    MW, Ma, Mc = rng.standard_normal((H, V)), rng.standard_normal(V), rng.standard_normal(H)
    V0 = rng.random((N, V))
    W2, a2, c2, MW2, Ma2, Mc2, s = rbm.cd1_step(W, a, c, MW, Ma, Mc, V0, rbm.BERNOULLI, 0.0, 0.0, 3, 1, 1, True)
    assert np.array_equal(W2, W) and np.array_equal(a2, a) and np.array_equal(c2, c)
    W3, _, _, MW3, _, _, s3 = rbm.cd1_step(W, a, c, MW, Ma, Mc, V0, rbm.BERNOULLI, 0.1, 0.9, 3, 1, 1, True)
    np.testing.assert_allclose(MW3, 0.9 * MW + 0.1 * s3["dW"], rtol=1e-14)
    np.testing.assert_allclose(W3, W + MW3, rtol=1e-14)
    assert set(np.unique(s3["V1"])) <= {0.0, 1.0}               # sampled visibles are binary
    # the two phases use different uniforms
    assert not np.array_equal(s3["u_h"].ravel()[:12], s3["u_v"].ravel()[:12])

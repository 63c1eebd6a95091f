"""Oracle for one CD-1 minibatch update of a restricted Boltzmann machine (test infrastructure).

The paper (Sec. 5.1) only names the method: the DNN is initialised from a stack of RBMs
pretrained greedily layer by layer with contrastive divergence; the first RBM sees real-valued
features.  The steps below are the standard one-step contrastive divergence (CD-1) with the
choices this build fixes (listed as readings in the design notes):

  1. P_h0 = sigmoid(V0 W^T + c)
  2. H0   = 1[u < P_h0]                 u: Philox uniform, phase 0, strict '<'
  3. V1   = H0 W + a                    Gaussian visible units (unit variance, mean, no noise)
     V1   = sigmoid(H0 W + a)           Bernoulli visible units (mean field), or
     V1   = 1[u' < sigmoid(H0 W + a)]   with sample_v1 (phase 1)
  4. P_h1 = sigmoid(V1 W^T + c)         probabilities, never sampled
  5. dW = (P_h0^T V0 - P_h1^T V1)/N,  da = mean_n(V0 - V1),  dc = mean_n(P_h0 - P_h1)
  6. M <- mu*M + lr*d ;  param <- param + M      (momentum form; no weight decay)
  recon_err = sum (V0 - V1)^2

W is n_hid x n_vis; a visible bias; c hidden bias.  All float64.
"""
from __future__ import annotations

import numpy as np

from . import philox

GAUSSIAN, BERNOULLI = 1, 0


def sigmoid(z):
    return 1.0 / (1.0 + np.exp(-z))


def hidden_prob(V, W, c):
    return sigmoid(np.asarray(V, np.float64) @ np.asarray(W, np.float64).T + np.asarray(c, np.float64)[None, :])


def cd1_statistics(W, a, c, V0, vis_type, u_h, u_v=None):
    """Steps 1-5 for given uniforms.  u_h: N x H uniforms (phase 0); u_v: N x V uniforms or None.

    Returns dict with P_h0, H0, V1pre (visible pre-sample mean / probability), V1, P_h1, dW, da, dc."""
    W = np.asarray(W, np.float64)
    a = np.asarray(a, np.float64)
    c = np.asarray(c, np.float64)
    V0 = np.asarray(V0, np.float64)
    N = V0.shape[0]
    P_h0 = sigmoid(V0 @ W.T + c[None, :])
    H0 = (u_h < P_h0).astype(np.float64)
    pre = H0 @ W + a[None, :]
    if vis_type == GAUSSIAN:
        V1mean = pre
        V1 = pre
    else:
        V1mean = sigmoid(pre)
        V1 = V1mean if u_v is None else (u_v < V1mean).astype(np.float64)
    P_h1 = sigmoid(V1 @ W.T + c[None, :])
    dW = (P_h0.T @ V0 - P_h1.T @ V1) / N
    da = (V0 - V1).sum(axis=0) / N
    dc = (P_h0 - P_h1).sum(axis=0) / N
    return dict(P_h0=P_h0, H0=H0, V1mean=V1mean, V1=V1, P_h1=P_h1, dW=dW, da=da, dc=dc,
                recon_err=float(((V0 - V1) ** 2).sum()))


def cd1_step(W, a, c, MW, Ma, Mc, V0, vis_type, lr, momentum, seed, step, layer, sample_v1=False):
    """One CD-1 update with Philox-driven sampling.  Returns (W, a, c, MW, Ma, Mc, info)."""
    W = np.asarray(W, np.float64)
    N, V = np.asarray(V0).shape
    H = W.shape[0]
    u_h = philox.uniforms(N * H, seed, step, layer, 0).reshape(N, H)
    u_v = philox.uniforms(N * V, seed, step, layer, 1).reshape(N, V) if (sample_v1 and vis_type == BERNOULLI) else None
    s = cd1_statistics(W, a, c, V0, vis_type, u_h, u_v)
    MW = momentum * np.asarray(MW, np.float64) + lr * s["dW"]
    Ma = momentum * np.asarray(Ma, np.float64) + lr * s["da"]
    Mc = momentum * np.asarray(Mc, np.float64) + lr * s["dc"]
    s["u_h"], s["u_v"] = u_h, u_v
    return W + MW, np.asarray(a, np.float64) + Ma, np.asarray(c, np.float64) + Mc, MW, Ma, Mc, s

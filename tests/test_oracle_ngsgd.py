"""Pins for the NG-SGD oracle (no GPU): dense-matrix checks of every algebraic step, the invariants
the paper fixes (E symmetric positive definite, Sec. 4 eq. 4; Fisher = second moment of the
score, eq. 5), and the reduction to plain SGD."""
import numpy as np
import pytest

import gen
from oracle import dnn, ngsgd


def _random_state(rng, D, R):
    Q, _ = np.linalg.qr(rng.standard_normal((D, R)))
    d = np.sort(rng.random(R) * 3 + 0.1)[::-1]
    return ngsgd.NGState(Q.T.copy(), d, 0.37, 5)


def test_apply_is_dense_inverse_of_smoothed_fisher():
    # (F + (alpha/D) tr(F) I)^-1 x, renormalised, computed with a dense inverse
    rng = np.random.default_rng(0)
    D, R, N, alpha = 12, 3, 7, 4.0
    st = _random_state(rng, D, R)
    X = rng.standard_normal((N, D))
    out, st2 = ngsgd.precondition(st, X, alpha, update=False)
    F = st.fisher()
    Fs = F + alpha / D * np.trace(F) * np.eye(D)
    Xd = X @ np.linalg.inv(Fs)                   # symmetric, so row-wise application
    Xd *= np.linalg.norm(X) / np.linalg.norm(Xd)
    np.testing.assert_allclose(out, Xd, rtol=1e-11, atol=1e-13)
    assert abs(np.linalg.norm(out) - np.linalg.norm(X)) < 1e-12 * np.linalg.norm(X)     # norm preserved
    assert st2.t == st.t and np.array_equal(st2.R, st.R)                                # update=False
    # E symmetric positive definite: spectrum of I - R^T E R is {1 (D-R times), 1 - e_i in (0,1]}
    beta, e = ngsgd.apply_coefficients(st, alpha)
    M = np.eye(D) - st.R.T @ np.diag(e) @ st.R
    ev = np.linalg.eigvalsh(M)
    assert np.all(ev > 0) and np.allclose(M, M.T)
    np.testing.assert_allclose(np.sort(ev), np.sort(np.concatenate([np.ones(D - R), 1 - e])), rtol=1e-12)
    assert float((out * X).sum()) > 0            # positive inner product with the raw quantity


def test_fold_matches_dense_subspace_iteration():
    rng = np.random.default_rng(1)
    D, R, N, eta = 10, 3, 20, 0.2
    st = _random_state(rng, D, R)
    X = rng.standard_normal((N, D)) * np.linspace(0.2, 3, D)[None, :]
    new = ngsgd.fold(st, X, eta)
    T = eta * X.T @ X / N + (1 - eta) * st.fisher()
    Y = st.R @ T
    Z = st.R @ T @ T @ st.R.T
    c = np.sort(np.linalg.eigvalsh(Z))[::-1]
    # rows orthonormal, spanning the row space of R_t T
    np.testing.assert_allclose(new.R @ new.R.T, np.eye(R), atol=1e-12)
    P_new = new.R.T @ new.R
    Qy, _ = np.linalg.qr(Y.T)
    np.testing.assert_allclose(P_new, Qy @ Qy.T, atol=1e-11)
    # d + rho = sqrt(eigenvalues of Z), trace of the new Fisher estimate = trace of T (no floor active here)
    np.testing.assert_allclose(new.d + new.rho, np.sqrt(c), rtol=1e-11)
    assert abs(new.d.sum() + D * new.rho - np.trace(T)) < 1e-11 * np.trace(T)
    assert new.t == st.t + 1


def test_iteration_converges_to_low_rank_second_moment():
    # data confined to an R-dimensional subspace with second moment S: the estimate converges to S's
    # top-R eigenpairs (eq. 5: Fisher = E[score score^T] -- here the 'scores' are the rows of X)
    rng = np.random.default_rng(2)
    D, R, N = 9, 3, 4000
    B, _ = np.linalg.qr(rng.standard_normal((D, R)))
    scales = np.array([3.0, 1.5, 0.7])
    st = ngsgd.init_state(D, R)
    for it in range(60):
        X = (rng.standard_normal((N, R)) * scales[None, :]) @ B.T
        _, st = ngsgd.precondition(st, X, eta=0.3)
    S = B @ np.diag(scales ** 2) @ B.T
    w, V = np.linalg.eigh(S)
    np.testing.assert_allclose(st.d + st.rho, w[::-1][:R], rtol=0.08)
    np.testing.assert_allclose(st.R.T @ st.R, B @ B.T, atol=2e-2)
    assert st.rho < 1e-3
    assert st.t == 60


def test_first_call_folds_three_times_and_counts_steps():
    rng = np.random.default_rng(3)
    D, R, N = 8, 2, 16
    X = rng.standard_normal((N, D))
    st0 = ngsgd.init_state(D, R)
    assert np.array_equal(st0.R, np.eye(R, D)) and st0.t == 0
    out, st1 = ngsgd.precondition(st0, X, eta=0.25)
    ref = st0
    for _ in range(3):
        ref = ngsgd.fold(ref, X, 0.25)
    ref.t = 0
    out_ref, _ = ngsgd.precondition(ref.copy(), X, eta=0.25, update=False)
    np.testing.assert_allclose(out, out_ref, rtol=1e-13)
    st1_ref = ngsgd.fold(ref, X, 0.25)
    np.testing.assert_allclose(st1.R.T @ st1.R, st1_ref.R.T @ st1_ref.R, atol=1e-12)
    assert st1.t == 1


def test_floors():
    rng = np.random.default_rng(4)
    D, R = 6, 3
    st = ngsgd.fold(ngsgd.init_state(D, R), np.zeros((4, D)), 0.1)       # all-zero data
    assert st.rho >= ngsgd.EPS and np.all(st.d >= ngsgd.EPS) and np.all(np.isfinite(st.R))
    X = np.outer(rng.standard_normal(50), rng.standard_normal(D))        # rank-1 data
    s = ngsgd.init_state(D, R)
    for _ in range(5):
        _, s = ngsgd.precondition(s, X, eta=0.5)
    assert np.all(s.d >= ngsgd.DELTA * s.d.max() * (1 - 1e-12))
    assert np.all(np.isfinite(s.R)) and s.rho >= ngsgd.EPS


def test_preconditioning_factors_equals_two_sided_preconditioning_of_gradient():
    # X_out_hat^T X_in_hat = g_out g_in M_out (delta^T A) M_in   (Kronecker structure of eq. 4's E)
    rng = np.random.default_rng(5)
    N, Di, Do = 9, 7, 6
    si, so = _random_state(rng, Di, 2), _random_state(rng, Do, 3)
    A, dlt = rng.standard_normal((N, Di)), rng.standard_normal((N, Do))
    Ah, _ = ngsgd.precondition(si, A, update=False)
    Dh, _ = ngsgd.precondition(so, dlt, update=False)
    def M_gamma(st, X):
        _, e = ngsgd.apply_coefficients(st, 4.0)
        M = np.eye(X.shape[1]) - st.R.T @ np.diag(e) @ st.R
        return M, np.linalg.norm(X) / np.linalg.norm(X @ M)
    Mi, gi = M_gamma(si, A)
    Mo, go = M_gamma(so, dlt)
    np.testing.assert_allclose(Dh.T @ Ah, go * gi * Mo @ (dlt.T @ A) @ Mi, rtol=1e-11, atol=1e-13)


def test_negligible_fisher_reduces_to_plain_sgd():
    # d = 0 -> e = 0 -> X_hat = X, gamma = 1: the NG-SGD step is the plain SGD step of eq. 3
    dims = (6, 5, 4)
    rng = np.random.default_rng(6)
    theta = rng.standard_normal(dnn.param_count(dims)) * 0.5
    X, y = rng.standard_normal((8, 6)), rng.integers(0, 4, 8)
    s_in = [ngsgd.NGState(np.eye(2, dims[l - 1] + 1), np.zeros(2), 1.0, 1) for l in range(1, len(dims))]
    s_out = [ngsgd.NGState(np.eye(2, dims[l]), np.zeros(2), 1.0, 1) for l in range(1, len(dims))]
    pre = ngsgd.make_layer_preconditioner(s_in, s_out, update=False)
    a, _, _ = dnn.sgd_step(theta, dims, X, y, 0.1, precondition=pre)
    b, _, _ = dnn.sgd_step(theta, dims, X, y, 0.1)
    np.testing.assert_allclose(a, b, rtol=1e-13, atol=1e-15)


def test_ng_step_is_a_descent_direction_on_tiny_config():
    dims = gen.CONFIG_TINY_DIMS
    theta = gen.init_theta(dims, 2, 0.1).astype(np.float64)
    R = 4
    s_in = [ngsgd.init_state(dims[l - 1] + 1, R) for l in range(1, len(dims))]
    s_out = [ngsgd.init_state(dims[l], R) for l in range(1, len(dims))]
    pre = ngsgd.make_layer_preconditioner(s_in, s_out)
    for t in range(4):
        X, y = gen.features_iid(32, 40, 2, 0, t), gen.labels_uniform(32, 32, 2, 0, t)
        g_raw, _ = dnn.gradient(theta, dims, X, y)
        new, _, _ = dnn.sgd_step(theta, dims, X, y, 0.1, precondition=pre)
        assert float(((theta - new) * g_raw).sum()) > 0          # E g has positive inner product with g
        theta = new
    assert all(s.t == 4 for s in s_in + s_out)
    for s in s_in + s_out:
        np.testing.assert_allclose(s.R @ s.R.T, np.eye(R), atol=1e-10)

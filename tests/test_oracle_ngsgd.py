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


def test_floors_hand_worked_rank_one():
    # D = 3, rank 1, R = e_0, one data row: every quantity of the fold is a one-line hand calculation.
    # (a) data along the tracked direction only: X = (2, 0, 0), d = 1, rho = 0, eta = 1/2.
    #     J = H^T X = (4, 0, 0);  Y = 0.5*4 e_0 + 0.5*(1 + 0) e_0 = 2.5 e_0;  sqrt(c) = 2.5
    #     tr T = 0.5*4 + 0.5*(3*0 + 1) = 2.5;  rho' = (2.5 - 2.5)/(3 - 1) = 0 -> raised to 1e-10;  d' = 2.5 - 0 = 2.5
    st = ngsgd.fold(ngsgd.NGState(np.array([[1.0, 0.0, 0.0]]), np.array([1.0]), 0.0, 7), np.array([[2.0, 0.0, 0.0]]), 0.5)
    assert st.rho == 1e-10 and st.t == 8
    np.testing.assert_allclose(st.d, [2.5], rtol=1e-15)
    np.testing.assert_allclose(np.abs(st.R), [[1.0, 0.0, 0.0]], atol=1e-15)
    # (b) data orthogonal to the tracked direction: X = (0, 2, 2), d = 0.5, rho = 0.1, eta = 1/2.
    #     H = 0, J = 0;  Y = 0.5*(0.5 + 0.1) e_0 = 0.3 e_0;  sqrt(c) = 0.3
    #     tr T = 0.5*8 + 0.5*(3*0.1 + 0.5) = 4.4;  rho' = (4.4 - 0.3)/2 = 2.05;  d' = 0.3 - 2.05 < 0 -> raised to 1e-10
    #     (DELTA * max d is negative here, so the absolute floor is the one that binds)
    st = ngsgd.fold(ngsgd.NGState(np.array([[1.0, 0.0, 0.0]]), np.array([0.5]), 0.1, 0), np.array([[0.0, 2.0, 2.0]]), 0.5)
    np.testing.assert_allclose(st.rho, 2.05, rtol=1e-15)
    assert st.d[0] == 1e-10
    np.testing.assert_allclose(np.abs(st.R), [[1.0, 0.0, 0.0]], atol=1e-15)


def test_floors_hand_worked_rank_two_diagonal():
    # D = 4, rank 2, R = [e_0; e_1], data rows along coordinate axes so that X^T X / N = diag(s) and every matrix of
    # the fold stays diagonal:  y_i = eta s_i + (1 - eta)(d_i + rho),  sqrt(c) = (y_0, y_1),
    # rho' = eta (s_2 + s_3)/2 + (1 - eta) rho,  d'_i = y_i - rho'.
    R0 = np.eye(2, 4)
    # (a) the relative floor on d: N = 2 rows, 4 sqrt(2) e_0 and 0.2 e_2, so s = (32/2, 0, 0.04/2, 0) = (16, 0, 0.02, 0);
    #     d = (8, 0.001), rho = 0.01, eta = 1/2.
    X = np.array([[4.0 * np.sqrt(2.0), 0.0, 0.0, 0.0], [0.0, 0.0, 0.2, 0.0]])
    st = ngsgd.fold(ngsgd.NGState(R0.copy(), np.array([8.0, 0.001]), 0.01, 0), X, 0.5)
    #     y_0 = 8 + 0.5*8.01 = 12.005;  y_1 = 0.5*0.011 = 0.0055;  rho' = 0.5*0.02/2 + 0.5*0.01 = 0.01
    #     d' = (11.995, -0.0045) -> second raised to DELTA * 11.995 = 5e-4 * 11.995 = 0.0059975
    np.testing.assert_allclose(st.rho, 0.01, rtol=1e-12)
    np.testing.assert_allclose(st.d, [11.995, 0.0059975], rtol=1e-12)
    np.testing.assert_allclose(np.abs(st.R), R0, atol=1e-12)
    # (b) the floor on the eigenvalues of Z: fresh state d = rho = 1e-10, one row 20 e_0 (s_0 = 400), eta = 1/2.
    #     y_0 = 200 + 1e-10, y_1 = 0.5*2e-10 = 1e-10, so c_1 = 1e-20 < 1e-24 * c_0 = 4e-20 and is raised to it:
    #     sqrt(c_1) = 1e-12 * y_0 = 2e-10.  Row 1 of the new R is Y_1 / sqrt(c_1) = e_1 * 1e-10 / 2e-10 = 0.5 e_1.
    #     tr T = 200 + 3e-10 = sum sqrt(c) to rounding, so rho' is at most rounding noise of 200 (2.8e-14) and is
    #     raised to 1e-10;  d' = (200, 2e-10) -> second raised to DELTA * 200 = 0.1.
    st = ngsgd.fold(ngsgd.init_state(4, 2), np.array([[20.0, 0.0, 0.0, 0.0]]), 0.5)
    assert st.rho == 1e-10
    np.testing.assert_allclose(st.d, [200.0, 0.1], rtol=1e-12)
    np.testing.assert_allclose(np.abs(st.R), [[1.0, 0, 0, 0], [0, 0.5, 0, 0]], atol=1e-9)


def test_first_call_equals_three_dense_subspace_iterations():
    # The first call on a fresh state, written out with dense D x D matrices and library routines that the oracle's
    # fold does not use (SVD of Y instead of the eigen-decomposition of Y Y^T, an explicit inverse instead of the
    # Woodbury form), and without calling ngsgd.fold: start from R = [I 0], d = rho = 1e-10; three times
    #   T = eta X^T X / N + (1 - eta) F,  Y = R T = U S V^T,  R <- V^T (rows),  rho <- (tr T - sum S)/(D - rank),  d <- S - rho
    # then precondition X with (F + (alpha/D) tr F I)^-1 and rescale to the norm of X.
    rng = np.random.default_rng(8)
    D, rank, N, eta, alpha = 9, 3, 40, 0.3, 4.0
    X = rng.standard_normal((N, D)) * np.linspace(2.0, 0.2, D)[None, :] + rng.standard_normal((N, 2)) @ rng.standard_normal((2, D))
    S = X.T @ X / N

    def dense_first_output(folds):
        R, d, rho = np.eye(rank, D), np.full(rank, 1e-10), 1e-10
        for _ in range(folds):
            F = R.T @ np.diag(d) @ R + rho * np.eye(D)
            T = eta * S + (1 - eta) * F
            _, sv, Vt = np.linalg.svd(R @ T, full_matrices=False)
            R = Vt
            rho = (np.trace(T) - sv.sum()) / (D - rank)
            d = sv - rho
            assert rho > 1e-10 and d.min() > 5e-4 * d.max()      # no floor is active in this example
        F = R.T @ np.diag(d) @ R + rho * np.eye(D)
        out = X @ np.linalg.inv(F + alpha / D * np.trace(F) * np.eye(D))
        return out * np.linalg.norm(X) / np.linalg.norm(out), F

    out, st = ngsgd.precondition(ngsgd.init_state(D, rank), X, alpha, eta, update=True)
    want, _ = dense_first_output(3)
    np.testing.assert_allclose(out, want, rtol=1e-9, atol=1e-12)
    # two or four folds give a visibly different first preconditioner: the count is pinned, not incidental
    for other in (2, 4):
        alt, _ = dense_first_output(other)
        assert np.linalg.norm(alt - want) > 1e-4 * np.linalg.norm(want)
    # the state returned has folded the minibatch once more (a fourth dense iteration) and counts one step
    R, d, rho = np.eye(rank, D), np.full(rank, 1e-10), 1e-10
    for _ in range(4):
        F = R.T @ np.diag(d) @ R + rho * np.eye(D)
        T = eta * S + (1 - eta) * F
        _, sv, Vt = np.linalg.svd(R @ T, full_matrices=False)
        R, rho = Vt, (np.trace(T) - sv.sum()) / (D - rank)
        d = sv - rho
    np.testing.assert_allclose(st.fisher(), R.T @ np.diag(d) @ R + rho * np.eye(D), rtol=1e-9, atol=1e-12)
    assert st.t == 1


def test_default_forgetting_factor_closed_form():
    # eta = 1 - exp(-N/2000): the weight of a minibatch of N frames when the estimate forgets with a time constant
    # of 2000 frames; N frames folded one at a time with per-frame weight 1 - exp(-1/2000) leave the same weight
    for n in (128, 256, 512, 1024):
        per_frame = 1.0 - np.exp(-1.0 / 2000.0)
        assert abs(ngsgd.default_eta(n) - (1.0 - (1.0 - per_frame) ** n)) < 1e-13
    assert abs(ngsgd.default_eta(512) - 0.2258580312) < 1e-10


def test_floors_keep_degenerate_inputs_finite():
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

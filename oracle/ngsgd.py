"""Oracle for the online low-rank natural-gradient preconditioner (test infrastructure).

The paper (Sec. 4, eq. 4) replaces the scalar learning rate by alpha_t * E_t with E_t symmetric
positive definite, standing for the inverse Fisher matrix (eq. 5), which is "approximated
directly"; every detail is left to the cited NG-SGD work.  This module fixes one concrete
reading of that online scheme, in this build's own notation; the HIP path implements the same
steps and parity is defined against THIS list.  That the constants (alpha = 4, the 2000-frame
forgetting constant, EPS, DELTA, C_FLOOR), the initial state and the three initial folds are those
of the cited algorithm: parity unpinned (the paper does not print them).  What this module does
with them is pinned: the algebra by dense checks, the floors by hand-worked examples, the first
call by three dense subspace iterations written without this module's fold.

Per preconditioned matrix X (N rows of dimension D: a layer's input activations with a 1
appended, or its output derivatives), rank R < D, the state is
    R_t  (R x D, orthonormal rows),  d_t (R, >= 0),  rho_t > 0,  t (minibatches seen)
and stands for the Fisher estimate  F_t = R_t^T diag(d_t) R_t + rho_t I.

Apply (uses F_t, which excludes the current minibatch except on the very first call):
  beta = rho (1 + alpha) + alpha * sum(d) / D      i.e. F_t + (alpha/D) tr(F_t) I = R^T D R + beta I
  e_i  = d_i / (d_i + beta)                        (R^T D R + beta I)^-1 = (I - R^T E R) / beta
  H    = X R^T ;  Xh = X - H diag(e) R
  out  = gamma * Xh,  gamma = ||X||_F / ||Xh||_F   (1 if either norm is 0)

Fold the minibatch in (T = eta * X^T X / N + (1 - eta) F_t, one step of subspace iteration):
  J = H^T X ;  Y = (eta/N) J + (1 - eta) (diag(d) + rho I) R   (= R_t T)
  Z = Y Y^T = U diag(c) U^T, c descending, floored at C_FLOOR * max(c)
  R' = diag(c)^-1/2 U^T Y
  rho' = [eta ||X||_F^2 / N + (1 - eta)(D rho + sum d) - sum sqrt(c)] / (D - R)    (tr F' = tr T)
  d'   = sqrt(c) - rho'
  floors: rho' >= EPS ;  d'_i >= max(EPS, DELTA * max_j d'_j)

First call on a fresh state (R = [I 0], d = rho = EPS): fold the minibatch in three times before
applying, so that the very first preconditioner already reflects data.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

EPS = 1e-10
DELTA = 5e-4
C_FLOOR = 1e-24
INIT_FOLDS = 3


@dataclass
class NGState:
    R: np.ndarray      # rank x dim
    d: np.ndarray      # rank
    rho: float
    t: int

    def copy(self):
        return NGState(self.R.copy(), self.d.copy(), float(self.rho), int(self.t))

    def fisher(self) -> np.ndarray:
        """Dense F_t (only sensible for tiny dim)."""
        D = self.R.shape[1]
        return self.R.T @ np.diag(self.d) @ self.R + self.rho * np.eye(D)


def init_state(dim: int, rank: int) -> NGState:
    assert 0 < rank < dim
    R = np.zeros((rank, dim))
    R[np.arange(rank), np.arange(rank)] = 1.0
    return NGState(R, np.full(rank, EPS), EPS, 0)


def default_eta(n: int) -> float:
    return 1.0 - float(np.exp(-n / 2000.0))


def apply_coefficients(state: NGState, alpha: float):
    """(beta, e) of the apply step."""
    D = state.R.shape[1]
    beta = state.rho * (1.0 + alpha) + alpha * state.d.sum() / D
    return beta, state.d / (state.d + beta)


def fold(state: NGState, X: np.ndarray, eta: float, H: np.ndarray | None = None) -> NGState:
    """Return the state after folding minibatch X in."""
    X = np.asarray(X, np.float64)
    N, D = X.shape
    Rk = state.R.shape[0]
    if H is None:
        H = X @ state.R.T
    J = H.T @ X
    Drho = state.d + state.rho
    Y = (eta / N) * J + (1.0 - eta) * Drho[:, None] * state.R
    Z = Y @ Y.T
    c, U = np.linalg.eigh(0.5 * (Z + Z.T))
    order = np.argsort(-c, kind="stable")
    c, U = c[order], U[:, order]
    c = np.maximum(c, C_FLOOR * c[0])
    sq = np.sqrt(c)
    Rn = (U.T @ Y) / sq[:, None]
    trT = eta * float((X * X).sum()) / N + (1.0 - eta) * (D * state.rho + state.d.sum())
    rho = (trT - sq.sum()) / (D - Rk)
    d = sq - rho
    rho = max(rho, EPS)
    d = np.maximum(d, max(EPS, DELTA * d.max()))
    return NGState(Rn, d, float(rho), state.t + 1)


def precondition(state: NGState, X: np.ndarray, alpha: float = 4.0, eta: float | None = None,
                 update: bool = True):
    """Returns (gamma * Xh, new state).  `state` itself is not modified."""
    X = np.asarray(X, np.float64)
    N = X.shape[0]
    if eta is None:
        eta = default_eta(N)
    st = state
    if update and st.t == 0:
        for _ in range(INIT_FOLDS):
            st = fold(st, X, eta)
        st = NGState(st.R, st.d, st.rho, 0)
    beta, e = apply_coefficients(st, alpha)
    H = X @ st.R.T
    Xh = X - (H * e[None, :]) @ st.R
    nx, nh = float((X * X).sum()), float((Xh * Xh).sum())
    gamma = np.sqrt(nx / nh) if (nx > 0.0 and nh > 0.0) else 1.0
    out = gamma * Xh
    if update:
        st = fold(st, X, eta, H)
    return out, st


def make_layer_preconditioner(states_in, states_out, alpha=4.0, eta=None, update=True):
    """Callable for dnn.gradient(precondition=...).  states_in[l-1] has dim d_{l-1}+1, states_out[l-1] has dim d_l.

    The lists are updated in place with the new states."""
    def pre(l, aug, delta):
        a_h, states_in[l - 1] = precondition(states_in[l - 1], aug, alpha, eta, update)
        d_h, states_out[l - 1] = precondition(states_out[l - 1], delta, alpha, eta, update)
        return a_h, d_h
    return pre

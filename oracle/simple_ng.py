"""Simple natural-gradient preconditioner (float64, NumPy).

TEST INFRASTRUCTURE ONLY - see oracle/__init__.py.

App. A of the paper: the Fisher factor that multiplies row i of a minibatch
matrix X (N x D) is estimated from the other N - 1 rows of the same minibatch,
smoothed with a multiple of the identity, and the result is rescaled to the
Frobenius norm of the input:

    beta   = alpha * max(tr(X^T X), epsilon) / (N D)
    F_i    = 1/(N-1) * sum_{j != i} x_j x_j^T
    xhat_i = (beta I + F_i)^{-1} x_i
    Xbar   = gamma * Xhat,   gamma = sqrt(tr(X^T X) / tr(Xhat^T Xhat))   (1 if the denominator is 0)

Two routines compute this:

  * `simple_ng_definitional` is the definition written out (App. A.2): one
    D x D solve per row with that row held out.  It is the reference; its cost
    (N solves of size D) restricts it to small matrices.
  * `simple_ng` follows App. A.3: one solve with nothing held out, Q = X G^{-1}
    in column space (N > D) or the equal row-space form (N <= D), then the
    per-row factor b_i = 1 + a_i / (N - 1 - a_i) with a_i = x_i . q_i.  The
    tests pin it to the definitional routine; the GPU path is compared with it
    at sizes the definitional routine cannot reach.

Reading: the paper's printed "xhat_i = G_i^{-1} x_i" has G_i already defined as
the inverse; the product meant is with the inverse smoothed Fisher matrix, as
the overview (xbar_i = F_i^{-1} x_i) states.

Both return (Xbar, gamma, gamma^2 * ||xhat_i||^2 per row), the same triple as the
online method, so that the max-change rule (App. C.3) can use the row norms.
"""
from __future__ import annotations

import numpy as np


def smoothing(X: np.ndarray, alpha: float, epsilon: float) -> float:
    """beta of App. A.2."""
    N, D = X.shape
    return alpha * max(float(np.sum(X * X)), epsilon) / (N * D)


def _rescale(X: np.ndarray, Xhat: np.ndarray):
    num = float(np.sum(X * X))
    den = float(np.sum(Xhat * Xhat))
    gamma = float(np.sqrt(num / den)) if den > 0.0 else 1.0
    return gamma * Xhat, gamma, gamma * gamma * np.sum(Xhat * Xhat, axis=1)


def simple_ng_definitional(X: np.ndarray, alpha: float = 4.0, epsilon: float = 1.0e-20):
    """App. A.2, row by row."""
    X = np.asarray(X, dtype=np.float64)
    N, D = X.shape
    assert N >= 2
    beta = smoothing(X, alpha, epsilon)
    Xhat = np.empty_like(X)
    for i in range(N):
        others = np.delete(X, i, axis=0)
        Gi = beta * np.eye(D) + (others.T @ others) / (N - 1)
        Xhat[i] = np.linalg.solve(Gi, X[i])
    return _rescale(X, Xhat)


def simple_ng(X: np.ndarray, alpha: float = 4.0, epsilon: float = 1.0e-20):
    """App. A.3: one solve for the whole minibatch and a per-row correction."""
    X = np.asarray(X, dtype=np.float64)
    N, D = X.shape
    assert N >= 2
    beta = smoothing(X, alpha, epsilon)
    if N > D:   # column space
        G = beta * np.eye(D) + (X.T @ X) / (N - 1)
        Q = np.linalg.solve(G, X.T).T          # X G^{-1}, G symmetric
    else:       # row space
        Grow = beta * np.eye(N) + (X @ X.T) / (N - 1)
        Q = np.linalg.solve(Grow, X)
    a = np.sum(X * Q, axis=1)
    b = 1.0 + a / (N - 1.0 - a)
    Xhat = b[:, None] * Q
    return _rescale(X, Xhat)

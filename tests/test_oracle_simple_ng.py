"""Pins for the float64 oracle of the simple natural-gradient method (App. A).

The efficient routine (App. A.3) is checked against the definition (App. A.2),
and the definition against closed forms that follow from it by hand, chosen so
that a dropped hold-out, a wrong normaliser (N instead of N - 1), a missing
smoothing term or a wrong sign in the per-row factor fails at least one.
"""
import os

import numpy as np
import pytest

from oracle.simple_ng import simple_ng, simple_ng_definitional, smoothing

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "constants.txt")


def golden():
    out = {}
    for line in open(GOLDEN):
        line = line.strip()
        if line and not line.startswith("#"):
            k, v = line.split()[:2]
            out[k] = float(v)
    return out


def data(rng, N, D, decay=0.8, mean=0.3):
    scales = decay ** np.arange(D) + 0.05
    Q, _ = np.linalg.qr(rng.standard_normal((D, D)))
    return (rng.standard_normal((N, D)) * scales[None, :]) @ Q.T + mean


def test_defaults_are_the_papers_settings():
    g = golden()
    import inspect
    for f in (simple_ng, simple_ng_definitional):
        p = inspect.signature(f).parameters
        assert p["alpha"].default == g["simple_alpha"]
        assert p["epsilon"].default == g["simple_epsilon"]


@pytest.mark.parametrize("N,D", [(40, 7), (12, 12), (9, 30), (2, 5), (33, 32), (32, 33)])
def test_efficient_form_equals_definition(N, D):
    """Column space (N > D) and row space (N <= D) both reproduce the row-by-row hold-out solve."""
    rng = np.random.default_rng(100 + N * 31 + D)
    X = data(rng, N, D)
    want, g_w, rn_w = simple_ng_definitional(X)
    got, g_g, rn_g = simple_ng(X)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-10 * np.abs(want).max())
    assert g_g == pytest.approx(g_w, rel=1e-10)
    np.testing.assert_allclose(rn_g, rn_w, rtol=1e-9)


def test_definition_against_explicit_inverse_of_the_held_out_fisher():
    """Row 3 of a small matrix, with F_3 accumulated by explicit outer products and inverted densely."""
    rng = np.random.default_rng(5)
    N, D, alpha = 6, 4, 4.0
    X = data(rng, N, D)
    beta = alpha * np.sum(X * X) / (N * D)
    F3 = np.zeros((D, D))
    for j in range(N):
        if j != 3:
            F3 += np.outer(X[j], X[j]) / (N - 1)
    xhat3 = np.linalg.inv(beta * np.eye(D) + F3) @ X[3]
    Xbar, gamma, _ = simple_ng_definitional(X, alpha=alpha)
    np.testing.assert_allclose(Xbar[3] / gamma, xhat3, rtol=1e-11)
    assert smoothing(X, alpha, 1e-20) == pytest.approx(beta, rel=1e-14)


def test_rows_on_distinct_axes_are_left_unchanged():
    """x_i = s_i e_i: F_i has no component along e_i, so xhat_i = x_i / beta, gamma = beta, Xbar = X.
    Without the hold-out the rows would be shrunk by different amounts."""
    s = np.array([3.0, 0.5, 2.0, 1.0, 7.0])
    N, D, alpha = 5, 8, 4.0
    X = np.zeros((N, D))
    X[np.arange(N), np.arange(N)] = s
    beta = alpha * np.sum(s * s) / (N * D)
    for f in (simple_ng_definitional, simple_ng):
        Xbar, gamma, rn = f(X, alpha=alpha)
        np.testing.assert_allclose(Xbar, X, atol=1e-13)
        assert gamma == pytest.approx(beta, rel=1e-13)
        np.testing.assert_allclose(rn, s * s, rtol=1e-12)


def test_two_rows_closed_form():
    """N = 2: F_0 = x_1 x_1^T, so xhat_0 = (x_0 - x_1 (x_1.x_0) / (beta + |x_1|^2)) / beta (Sherman-Morrison by hand)."""
    rng = np.random.default_rng(7)
    D, alpha = 5, 2.5
    X = rng.standard_normal((2, D))
    beta = alpha * np.sum(X * X) / (2 * D)
    xh0 = (X[0] - X[1] * (X[1] @ X[0]) / (beta + X[1] @ X[1])) / beta
    xh1 = (X[1] - X[0] * (X[0] @ X[1]) / (beta + X[0] @ X[0])) / beta
    Xhat = np.stack([xh0, xh1])
    gamma = np.sqrt(np.sum(X * X) / np.sum(Xhat * Xhat))
    for f in (simple_ng_definitional, simple_ng):
        Xbar, g, _ = f(X, alpha=alpha)
        np.testing.assert_allclose(Xbar, gamma * Xhat, rtol=1e-11, atol=1e-13)
        assert g == pytest.approx(gamma, rel=1e-12)


def test_identical_rows_closed_form():
    """All rows equal to x: F_i = x x^T, xhat_i = x / (beta + |x|^2), beta = alpha |x|^2 / D, Xbar = X."""
    x = np.array([1.0, -2.0, 0.5, 3.0])
    N, alpha = 7, 4.0
    X = np.tile(x, (N, 1))
    n2 = x @ x
    for f in (simple_ng_definitional, simple_ng):
        Xbar, gamma, rn = f(X, alpha=alpha)
        np.testing.assert_allclose(Xbar, X, rtol=1e-12)
        assert gamma == pytest.approx(alpha * n2 / len(x) + n2, rel=1e-12)
        np.testing.assert_allclose(rn, np.full(N, n2), rtol=1e-12)


@pytest.mark.parametrize("N,D", [(30, 9), (10, 25)])
def test_invariants(N, D):
    rng = np.random.default_rng(N + D)
    X = data(rng, N, D)
    Xbar, gamma, rn = simple_ng(X)
    # same Frobenius norm as the input (Sec. 4.7), row norms consistent with the output
    assert np.linalg.norm(Xbar) == pytest.approx(np.linalg.norm(X), rel=1e-12)
    np.testing.assert_allclose(rn, np.sum(Xbar * Xbar, axis=1), rtol=1e-12)
    # homogeneity: scaling the data by s scales the output by s and gamma by s^2
    s = 37.5
    Xs, gs, rns = simple_ng(s * X)
    np.testing.assert_allclose(Xs, s * Xbar, rtol=1e-10, atol=1e-12)
    assert gs == pytest.approx(s * s * gamma, rel=1e-10)
    # rotating the coordinates rotates the output; permuting the rows permutes it
    U, _ = np.linalg.qr(rng.standard_normal((D, D)))
    np.testing.assert_allclose(simple_ng(X @ U)[0], Xbar @ U, rtol=0, atol=1e-10 * np.abs(Xbar).max())
    perm = rng.permutation(N)
    np.testing.assert_allclose(simple_ng(X[perm])[0], Xbar[perm], rtol=0, atol=1e-11 * np.abs(Xbar).max())


def test_heavy_smoothing_tends_to_the_identity():
    """alpha -> infinity: G_i -> beta I, every row is scaled alike and the rescaling restores X."""
    rng = np.random.default_rng(11)
    X = data(rng, 20, 6)
    Xbar, _, _ = simple_ng(X, alpha=1e9)
    np.testing.assert_allclose(Xbar, X, rtol=0, atol=1e-7 * np.abs(X).max())
    # and with the usual alpha the result is not a multiple of X (the Fisher factor acts)
    Xbar4, _, _ = simple_ng(X, alpha=4.0)
    c = np.sum(Xbar4 * X) / np.sum(X * X)
    assert np.linalg.norm(Xbar4 - c * X) > 0.05 * np.linalg.norm(X)


def test_zero_matrix():
    """tr(X^T X) = 0: beta = alpha epsilon / (N D), Xhat = 0, gamma = 1."""
    X = np.zeros((5, 3))
    assert smoothing(X, 4.0, 1e-20) == pytest.approx(4.0e-20 / 15.0)
    for f in (simple_ng_definitional, simple_ng):
        Xbar, gamma, rn = f(X)
        assert not Xbar.any() and gamma == 1.0 and not rn.any()

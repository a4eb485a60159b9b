"""Pins for the float64 oracle of the online natural-gradient preconditioner.

Every check here compares the oracle with something fixed by the paper or by
linear algebra, computed by an independent route (dense solves, SVD, closed
forms), never with the oracle's own formula retyped.
"""
import math
import os

import numpy as np
import pytest
import scipy.linalg

from oracle.online_ng import (OnlineNaturalGradient, forgetting_factor, initial_state,
                              reorthogonalise_if_needed)
from oracle.online_ng_efficient import OnlineNaturalGradientEfficient

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "constants.txt")


def golden():
    out = {}
    for line in open(GOLDEN):
        line = line.strip()
        if line and not line.startswith("#"):
            k, v = line.split()[:2]
            out[k] = float(v)
    return out


def data(rng, N, D, decay=0.7, mean=0.5):
    """Rows with an anisotropic covariance and a non-zero mean."""
    scales = decay ** np.arange(D) + 0.05
    Q, _ = np.linalg.qr(rng.standard_normal((D, D)))
    return (rng.standard_normal((N, D)) * scales[None, :]) @ Q.T + mean


def dense_fisher(R, d, rho):
    return R.T @ np.diag(d) @ R + rho * np.eye(R.shape[1])


# ---------------------------------------------------------------------------------------------
def test_forgetting_factor_closed_form():
    g = golden()
    for n in (64, 128, 512, 1024):
        assert forgetting_factor(n, g["num_samples_history"]) == pytest.approx(g[f"eta_N{n}"], abs=1e-14)


def test_defaults_match_paper_configuration():
    g = golden()
    ng = OnlineNaturalGradient(dim=100, rank=int(g["rank_input_side"]))
    assert ng.alpha == g["alpha"] and ng.num_samples_history == g["num_samples_history"]
    assert ng.epsilon == g["epsilon"] and ng.update_period == g["update_period"]
    assert ng.always_update_first == g["always_update_first"]
    # update schedule: t < 10 always, afterwards only when 4 divides t (App. B.4)
    sched = []
    for t in range(20):
        ng.t = t
        sched.append(ng.will_update())
    assert sched == [True] * 10 + [False, False, True, False, False, False, True, False, False, False]


@pytest.mark.parametrize("N,D,R", [(30, 12, 3), (8, 11, 2), (40, 9, 1), (16, 16, 5)])
def test_apply_equals_dense_inverse_fisher(N, D, R):
    """P1: gamma X G^{-1} with G = F + alpha tr(F)/D I by a dense solve (eq. low:rank and following)."""
    rng = np.random.default_rng(100 + D)
    ng = OnlineNaturalGradient(D, R, alpha=4.0, num_samples_history=50.0, update_period=1)
    for t in range(6):
        M = data(rng, N, D)
        if t > 0:
            F = dense_fisher(ng.R, ng.d, ng.rho)
        Mbar, gamma, rn2 = ng.precondition(M)
        if t == 0:
            continue          # state was built inside the call; covered by the init tests
        G = F + (4.0 * np.trace(F) / D) * np.eye(D)
        XG = np.linalg.solve(G, M.T).T                      # X G^{-1}, G symmetric
        expect = XG * (np.linalg.norm(M) / np.linalg.norm(XG))
        np.testing.assert_allclose(Mbar, expect, rtol=0, atol=1e-12 * np.linalg.norm(M))
        np.testing.assert_allclose(rn2, np.sum(expect ** 2, axis=1), rtol=1e-10)
        assert np.linalg.norm(Mbar) == pytest.approx(np.linalg.norm(M), rel=1e-13)


@pytest.mark.parametrize("N,D,R", [(30, 12, 3), (8, 11, 2), (25, 10, 4)])
def test_update_equals_dense_power_step_via_svd(N, D, R):
    """P2: F_{t+1} from Y = R_t T_t by an SVD of Y (the paper notes the SVD is the direct route)."""
    rng = np.random.default_rng(7 + N)
    S_hist = 60.0
    ng = OnlineNaturalGradient(D, R, num_samples_history=S_hist, update_period=1)
    ng.precondition(data(rng, N, D))
    checked_trace = []
    for t in range(5):
        M = data(rng, N, D)
        R0, d0, rho0 = ng.R.copy(), ng.d.copy(), ng.rho
        F = dense_fisher(R0, d0, rho0)
        eta = 1.0 - math.exp(-N / S_hist)
        T = eta * (M.T @ M) / N + (1.0 - eta) * F
        Y = R0 @ T
        _, s, Vt = np.linalg.svd(Y, full_matrices=False)
        rho_new = (np.trace(T) - s.sum()) / (D - R)
        d_floor_fired = bool(np.any(s - rho_new < 1e-10)) or rho_new < 1e-10
        F_expect = Vt.T @ np.diag(np.maximum(s - rho_new, 1e-10)) @ Vt + max(rho_new, 1e-10) * np.eye(D)  # eq. dt1, rhot1
        ng.precondition(M)
        assert not ng.last["floored"]
        F_new = dense_fisher(ng.R, ng.d, ng.rho)
        np.testing.assert_allclose(F_new, F_expect, atol=1e-11 * np.trace(T))
        np.testing.assert_allclose(ng.R @ ng.R.T, np.eye(R), atol=1e-12)          # orthonormal rows
        if not d_floor_fired:
            assert np.trace(F_new) == pytest.approx(np.trace(T), rel=1e-12)       # trace matching
            checked_trace.append(t)
        # eigenvalues of Z are bounded below by ((1-eta) rho)^2 (App. B.3)
        assert np.all(ng.last["c"] >= ((1 - eta) * rho0) ** 2 * (1 - 1e-9))
        # decreasing order, 0 < e < 1
        assert np.all(np.diff(ng.last["c"]) <= 0)
        assert np.all((ng.last["e"] > 0) & (ng.last["e"] < 1))
    if (N, D, R) != (25, 10, 4):
        assert len(checked_trace) == 5


@pytest.mark.parametrize("N,D,R", [(40, 14, 3), (10, 23, 4), (64, 33, 6)])
@pytest.mark.parametrize("trace_identity", [False, True])
def test_efficient_form_reproduces_definitional_form(N, D, R, trace_identity):
    """P3 / P10: App. B.3's W, H, J, K, L, Z, A_t B_t route equals App. B.1-B.2."""
    rng = np.random.default_rng(5 * D + R)
    a = OnlineNaturalGradient(D, R, num_samples_history=120.0, update_period=2, always_update_first=3)
    b = OnlineNaturalGradientEfficient(D, R, num_samples_history=120.0, update_period=2,
                                       always_update_first=3, trace_identity=trace_identity)
    for t in range(12):
        n = N if t != 5 else N - 3          # the minibatch size may vary (App. B.5)
        M = data(rng, n, D)
        Ma, ga, ra = a.precondition(M)
        Mb, gb, rb = b.precondition(M)
        np.testing.assert_allclose(Mb, Ma, atol=1e-10 * np.linalg.norm(M))
        assert gb == pytest.approx(ga, rel=1e-9)
        np.testing.assert_allclose(rb, ra, rtol=1e-8)
        np.testing.assert_allclose(b.fisher(), a.fisher(), atol=1e-10 * np.trace(a.fisher()))
        assert b.rho == pytest.approx(a.rho, rel=1e-8)


def test_rank_zero_is_scaled_identity():
    """P4: with R = 0 the factor is rho I, the output equals the input and rho follows the trace."""
    rng = np.random.default_rng(3)
    N, D = 20, 7
    ng = OnlineNaturalGradient(D, 0, num_samples_history=40.0, update_period=1)
    M = data(rng, N, D)
    Mbar, gamma, rn2 = ng.precondition(M)
    np.testing.assert_array_equal(Mbar, M)
    assert gamma == 1.0
    np.testing.assert_allclose(rn2, np.sum(M * M, axis=1), rtol=1e-15)
    eta = 1 - math.exp(-N / 40.0)
    rho0 = np.sum(M * M) / N / D
    assert ng.rho == pytest.approx(eta * np.sum(M * M) / N / D + (1 - eta) * rho0, rel=1e-14)
    M2 = data(rng, N, D)
    rho1 = ng.rho
    Mbar2, _, _ = ng.precondition(M2)
    np.testing.assert_array_equal(Mbar2, M2)
    assert ng.rho == pytest.approx(eta * np.sum(M2 * M2) / N / D + (1 - eta) * rho1, rel=1e-14)


def test_scale_invariants():
    """P6: ||Xbar||_F = ||X||_F; scaling all inputs by s scales Xbar by s and d, rho by s^2."""
    rng = np.random.default_rng(11)
    N, D, R, s = 32, 15, 4, 37.5
    a = OnlineNaturalGradient(D, R, num_samples_history=100.0, update_period=1)
    b = OnlineNaturalGradient(D, R, num_samples_history=100.0, update_period=1)
    for _ in range(8):
        M = data(rng, N, D)
        Ma, ga, _ = a.precondition(M)
        Mb, gb, _ = b.precondition(s * M)
        assert np.linalg.norm(Ma) == pytest.approx(np.linalg.norm(M), rel=1e-13)
        np.testing.assert_allclose(Mb, s * Ma, rtol=0, atol=1e-11 * np.linalg.norm(s * M))
        live = a.d > 10 * a.epsilon                           # the epsilon floors do not scale
        assert live.sum() >= 3
        np.testing.assert_allclose(b.d[live], s * s * a.d[live], rtol=1e-9)
        assert b.rho == pytest.approx(s * s * a.rho, rel=1e-9)


def test_rotation_equivariance():
    """P7: X -> X Q with Q orthogonal gives Xbar -> Xbar Q."""
    rng = np.random.default_rng(12)
    N, D, R = 30, 13, 3
    Q, _ = np.linalg.qr(rng.standard_normal((D, D)))
    a = OnlineNaturalGradient(D, R, num_samples_history=80.0, update_period=1)
    b = OnlineNaturalGradient(D, R, num_samples_history=80.0, update_period=1)
    for _ in range(7):
        M = data(rng, N, D)
        Ma, _, _ = a.precondition(M)
        Mb, _, _ = b.precondition(M @ Q)
        np.testing.assert_allclose(Mb, Ma @ Q, atol=1e-10 * np.linalg.norm(M))


def test_directional_scaling():
    """P8: along row r_i of R the input is scaled by (1 - e_i); orthogonal directions pass unchanged."""
    rng = np.random.default_rng(13)
    N, D, R = 25, 12, 3
    ng = OnlineNaturalGradient(D, R, num_samples_history=50.0, update_period=1)
    for _ in range(4):
        ng.precondition(data(rng, N, D))
    Rm, d, rho = ng.R.copy(), ng.d.copy(), ng.rho
    M = data(rng, N, D)
    Mbar, gamma, _ = ng.precondition(M)
    Mhat = Mbar / gamma
    F = dense_fisher(Rm, d, rho)
    beta = rho + 4.0 * np.trace(F) / D
    for i in range(R):
        e_i = 1.0 / (beta / d[i] + 1.0)
        assert 0 < e_i < 1
        np.testing.assert_allclose(Mhat @ Rm[i], (1 - e_i) * (M @ Rm[i]), atol=1e-12 * np.linalg.norm(M))
    null = scipy.linalg.null_space(Rm)
    np.testing.assert_allclose(Mhat @ null, M @ null, atol=1e-12 * np.linalg.norm(M))


def test_fixed_point_with_constant_covariance():
    """P9: with M^T M / N held exactly at V L V^T + s^2 I (rank R), F_t converges to it (Sec. 5.3)."""
    rng = np.random.default_rng(14)
    N, D, R = 40, 10, 3
    V, _ = np.linalg.qr(rng.standard_normal((D, R)))
    lam = np.array([9.0, 4.0, 1.5])
    cov = V @ np.diag(lam) @ V.T + 0.3 * np.eye(D)
    root = scipy.linalg.sqrtm(cov).real
    ng = OnlineNaturalGradient(D, R, num_samples_history=80.0, update_period=1)
    # start from a wrong state so that convergence is not trivial
    ng.precondition(rng.standard_normal((N, D)))
    for _ in range(400):
        Qn, _ = np.linalg.qr(rng.standard_normal((N, D)))      # orthonormal columns
        ng.precondition(math.sqrt(N) * Qn @ root)              # M^T M / N == cov exactly
    np.testing.assert_allclose(dense_fisher(ng.R, ng.d, ng.rho), cov, atol=1e-8)
    # general spectrum: top-R eigenpairs plus the mean of the rest
    evals = np.array([8.0, 5.0, 3.0, 1.0, 0.8, 0.6, 0.5, 0.4, 0.3, 0.2])
    Qf, _ = np.linalg.qr(rng.standard_normal((D, D)))
    cov2 = Qf @ np.diag(evals) @ Qf.T
    root2 = scipy.linalg.sqrtm(cov2).real
    ng2 = OnlineNaturalGradient(D, R, num_samples_history=80.0, update_period=1)
    for _ in range(1500):
        Qn, _ = np.linalg.qr(rng.standard_normal((N, D)))
        ng2.precondition(math.sqrt(N) * Qn @ root2)
    expect = Qf[:, :R] @ np.diag(evals[:R] - evals[R:].mean()) @ Qf[:, :R].T + evals[R:].mean() * np.eye(D)
    np.testing.assert_allclose(dense_fisher(ng2.R, ng2.d, ng2.rho), expect, atol=1e-6)


def test_fisher_stays_spd_and_bounded():
    """P5: rho >= eps, d >= eps, F symmetric positive definite, through zero and tiny inputs."""
    rng = np.random.default_rng(15)
    N, D, R = 20, 9, 3
    ng = OnlineNaturalGradient(D, R, num_samples_history=30.0, update_period=1)
    seq = [data(rng, N, D), np.zeros((N, D)), np.zeros((N, D)), 1e-9 * data(rng, N, D), data(rng, N, D),
           1e4 * data(rng, N, D)]
    for M in seq:
        Mbar, gamma, _ = ng.precondition(M)
        assert np.all(np.isfinite(Mbar)) and math.isfinite(gamma) and gamma > 0
        if not M.any():
            assert gamma == 1.0                                 # zero denominator -> gamma = 1
        assert ng.rho >= ng.epsilon and np.all(ng.d >= ng.epsilon)
        F = dense_fisher(ng.R, ng.d, ng.rho)
        np.testing.assert_allclose(F, F.T, atol=1e-12 * np.trace(F))
        assert np.linalg.eigvalsh(F).min() > 0
        np.testing.assert_allclose(ng.R @ ng.R.T, np.eye(R), atol=2e-3)


@pytest.mark.parametrize("N,D,R", [(30, 11, 3), (9, 14, 3), (12, 12, 4)])
def test_initial_state_is_top_eigenpairs(N, D, R):
    """App. B.3.2 against a dense eigen-decomposition of S_0, for N > D, N < D and N = D."""
    rng = np.random.default_rng(16 + N)
    M0 = data(rng, N, D)
    Rm, d, rho = initial_state(M0, R, 1e-10)
    S0 = M0.T @ M0 / N
    lam, V = np.linalg.eigh(S0)
    lam, V = lam[::-1], V[:, ::-1]
    rho_expect = (np.trace(S0) - lam[:R].sum()) / (D - R)
    assert rho == pytest.approx(rho_expect, rel=1e-10)
    np.testing.assert_allclose(d, lam[:R] - rho_expect, rtol=1e-9)
    F_expect = V[:, :R] @ np.diag(lam[:R] - rho_expect) @ V[:, :R].T + rho_expect * np.eye(D)
    np.testing.assert_allclose(dense_fisher(Rm, d, rho), F_expect, atol=1e-11 * np.trace(S0))
    assert np.trace(dense_fisher(Rm, d, rho)) == pytest.approx(np.trace(S0), rel=1e-12)


def test_initial_state_degenerate_inputs():
    """Zero and rank-deficient first minibatches: floors apply and R_0 is still orthonormal."""
    N, D, R = 10, 8, 3
    Rm, d, rho = initial_state(np.zeros((N, D)), R, 1e-10)
    assert rho == 1e-10 and np.all(d == 1e-10)
    np.testing.assert_allclose(Rm, np.eye(D)[:R], atol=0)        # completion from e_0, e_1, e_2
    # rank one input: first row is the data direction, the others complete the basis
    v = np.arange(1.0, D + 1)
    M0 = np.outer(np.linspace(1, 2, N), v)
    Rm, d, rho = initial_state(M0, R, 1e-10)
    np.testing.assert_allclose(Rm @ Rm.T, np.eye(R), atol=1e-12)
    np.testing.assert_allclose(np.abs(Rm[0]), v / np.linalg.norm(v), atol=1e-12)
    assert d[0] == pytest.approx(np.sum(M0 * M0) / N, rel=1e-10) and np.all(d[1:] == 1e-10)
    for N2, D2 in [(5, 9), (9, 5)]:                                # both eigen routes
        M0 = np.outer(np.ones(N2), np.ones(D2))
        Rm, d, rho = initial_state(M0, 2, 1e-10)
        np.testing.assert_allclose(Rm @ Rm.T, np.eye(2), atol=1e-12)


def test_reorthogonalisation_restores_orthonormal_rows():
    """App. B.3.1 forced: a corrupted R_t makes eigenvalues of Z fall under the floor."""
    rng = np.random.default_rng(17)
    N, D, R = 30, 12, 4
    ng = OnlineNaturalGradient(D, R, num_samples_history=60.0, update_period=1)
    for _ in range(3):
        ng.precondition(data(rng, N, D))
    ng.R[1] *= 1e-4                                              # break R R^T = I
    ng.R[2] += 0.3 * ng.R[0]
    ng.rho = 10.0 * ng.d.max()                                   # large floor
    ng.precondition(data(rng, N, D))
    assert ng.last["floored"] and ng.last["reorthogonalised"]
    np.testing.assert_allclose(ng.R @ ng.R.T, np.eye(R), atol=1e-10)
    assert ng.rho >= ng.epsilon and np.all(ng.d >= ng.epsilon)


def test_reorthogonalisation_of_skewed_rows():
    """A skewed (non-diagonal R R^T) factor comes back orthonormal with the same row space and a
    lower-triangular mixing (row i only mixes rows 0..i, as a Cholesky factor does)."""
    rng = np.random.default_rng(19)
    Q, _ = np.linalg.qr(rng.standard_normal((9, 4)))
    R0 = Q.T
    mix = np.eye(4) + 0.2 * rng.standard_normal((4, 4))
    R_bad = mix @ R0
    R_fix, did = reorthogonalise_if_needed(R_bad)
    assert did
    np.testing.assert_allclose(R_fix @ R_fix.T, np.eye(4), atol=1e-12)
    coeff = R_fix @ np.linalg.pinv(R_bad)                       # R_fix = coeff R_bad
    np.testing.assert_allclose(coeff @ R_bad, R_fix, atol=1e-12)
    np.testing.assert_allclose(np.triu(coeff, 1), 0.0, atol=1e-12)
    R_ok, did = reorthogonalise_if_needed(R0 + 1e-5)
    assert not did and R_ok is not None


def test_two_routes_to_L_agree():
    """H^T H = J W^T (App. B.3): the efficient form gives the same result on both branches N <= D, N > D."""
    rng = np.random.default_rng(18)
    D, R = 12, 3
    for N in (8, 20):
        b = OnlineNaturalGradientEfficient(D, R, num_samples_history=50.0, update_period=1)
        a = OnlineNaturalGradient(D, R, num_samples_history=50.0, update_period=1)
        for _ in range(4):
            M = data(rng, N, D)
            Ma, _, _ = a.precondition(M)
            Mb, _, _ = b.precondition(M)
            np.testing.assert_allclose(Mb, Ma, atol=1e-11 * np.linalg.norm(M))

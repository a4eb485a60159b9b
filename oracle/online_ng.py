"""Online natural-gradient preconditioner, definitional form (float64, NumPy).

TEST INFRASTRUCTURE ONLY - see oracle/__init__.py.

Follows App. B.1 and B.2 of the paper with the low-rank factor kept explicitly:

    F_t = R_t^T D_t R_t + rho_t I          (eq. low:rank; R_t has orthonormal rows)
    G_t = F_t + (alpha tr(F_t) / D) I      (smoothed Fisher factor)
    Xbar_t = gamma_t X_t G_t^{-1},  ||Xbar_t||_F = ||X_t||_F

and the update F_t -> F_{t+1} by one power-method-like step on
T_t = eta S_t + (1 - eta) F_t (App. B.2).  G_t^{-1} is applied through the
Woodbury form the paper states (App. B.3): G^{-1} = (I - R^T E R) / beta with
e_ii = 1 / (beta / d_ii + 1).  The tests check that form against a dense solve.

Readings where the paper leaves a choice (all restated in the design notes):
  * tr(X X^T) is the direct sum of squares (the paper's trace identity holds
    only while R R^T = I).
  * The state built from minibatch 0 is used to precondition minibatch 0 and
    is then updated with minibatch 0 (App. B.5, "on t = 0 ... before running
    the steps below").
  * The top-R eigenpairs of S_0 come from the D x D covariance if D <= N and
    from the N x N Gram matrix otherwise (same non-zero spectrum).
  * Directions of S_0 whose eigenvalue is not above 1e-12 of the largest one
    carry no information; their rows of R_0 are an orthonormal completion built
    by Gram-Schmidt from the standard basis e_0, e_1, ... (first vector whose
    residual exceeds 0.1), and their d is epsilon.
  * App. B.3.1's check is applied to the new factor: O = R_{t+1} R_{t+1}^T, and
    if any entry is off the identity by more than 1e-3, R_{t+1} <- L^{-1} R_{t+1}
    with O = L L^T (this is the paper's M = E^{1/2} L^{-1} E^{-1/2} acting on
    W = E^{1/2} R).
  * Eigenpairs are ordered by decreasing eigenvalue (App. B.4: e_ii sorted from
    greatest to least).
"""
from __future__ import annotations

import math

import numpy as np

ORTHO_COND_LIMIT = 1.0e6      # App. B.3.1: condition number of C_t that triggers the check
ORTHO_TOLERANCE = 1.0e-3      # App. B.3.1: allowed deviation of R R^T from I
NULL_EIG_RATIO = 1.0e-12      # reading: eigenvalues of S_0 at or below this ratio are "zero"
COMPLETION_MIN_RESIDUAL = 0.1  # reading: Gram-Schmidt completion threshold


def forgetting_factor(num_rows: int, num_samples_history: float) -> float:
    """eta = 1 - exp(-N / S)   (App. B.4, eq. eta:ns)."""
    return 1.0 - math.exp(-float(num_rows) / float(num_samples_history))


def smoothing_and_scales(d: np.ndarray, rho: float, alpha: float, dim: int):
    """beta_t (eq. beta2) and the diagonal of E_t (eq. etii)."""
    beta = rho * (1.0 + alpha) + (alpha / dim) * float(np.sum(d))
    e = 1.0 / (beta / d + 1.0)
    return beta, e


def complete_orthonormal_rows(rows: np.ndarray, keep: np.ndarray) -> np.ndarray:
    """Replace rows[i] for keep[i] == False by an orthonormal completion.

    Candidates are the standard basis vectors e_0, e_1, ... taken in order; a
    candidate is orthogonalised (twice) against every row already fixed and
    accepted when its residual norm exceeds COMPLETION_MIN_RESIDUAL.
    """
    rank, dim = rows.shape
    out = rows.copy()
    fixed = [i for i in range(rank) if keep[i]]
    cand = 0
    for i in range(rank):
        if keep[i]:
            continue
        while True:
            if cand >= dim:
                raise ValueError("cannot complete an orthonormal basis")
            v = np.zeros(dim)
            v[cand] = 1.0
            cand += 1
            for _ in range(2):
                for j in fixed:
                    v -= np.dot(out[j], v) * out[j]
            nrm = float(np.linalg.norm(v))
            if nrm > COMPLETION_MIN_RESIDUAL:
                out[i] = v / nrm
                fixed.append(i)
                break
    return out


def reorthogonalise_if_needed(R_new: np.ndarray):
    """App. B.3.1: if R R^T is off the identity by more than 1e-3 anywhere, R <- L^{-1} R with R R^T = L L^T."""
    O = R_new @ R_new.T
    if float(np.max(np.abs(O - np.eye(R_new.shape[0])))) <= ORTHO_TOLERANCE:
        return R_new, False
    L = np.linalg.cholesky(O)
    return np.linalg.solve(L, R_new), True


def initial_state(M0: np.ndarray, rank: int, epsilon: float):
    """R_0, d_0, rho_0 from the first minibatch (App. B.3.2)."""
    M0 = np.asarray(M0, dtype=np.float64)
    N, D = M0.shape
    trace_S0 = float(np.sum(M0 * M0)) / N
    if rank == 0:
        return np.zeros((0, D)), np.zeros(0), max(trace_S0 / D, epsilon)
    if D <= N:
        S0 = (M0.T @ M0) / N
        lam, V = np.linalg.eigh(S0)                   # ascending
        lam = lam[::-1][:rank]
        rows = V[:, ::-1][:, :rank].T.copy()
        lam_max = lam[0]
        keep = (lam > NULL_EIG_RATIO * lam_max) & (lam_max > 0.0)
    else:
        gram = (M0 @ M0.T) / N
        lam, U = np.linalg.eigh(gram)
        lam = lam[::-1][:rank]
        U = U[:, ::-1][:, :rank]
        lam_max = lam[0]
        keep = (lam > NULL_EIG_RATIO * lam_max) & (lam_max > 0.0)
        rows = np.zeros((rank, D))
        for i in range(rank):
            if keep[i]:
                rows[i] = (M0.T @ U[:, i]) / math.sqrt(N * lam[i])
    lam = np.where(keep, lam, 0.0)
    if not np.all(keep):
        rows = complete_orthonormal_rows(rows, keep)
    rho0 = max((trace_S0 - float(np.sum(lam))) / (D - rank), epsilon)
    d0 = np.maximum(epsilon, lam - rho0)
    return rows, d0, rho0


class OnlineNaturalGradient:
    """One instance of the online method (one of the 2I copies of the state)."""

    def __init__(self, dim: int, rank: int, alpha: float = 4.0,
                 num_samples_history: float = 2000.0, epsilon: float = 1.0e-10,
                 update_period: int = 4, always_update_first: int = 10):
        if not (0 <= rank < dim):
            raise ValueError("need 0 <= rank < dim")
        self.dim = dim
        self.rank = rank
        self.alpha = float(alpha)
        self.num_samples_history = float(num_samples_history)
        self.epsilon = float(epsilon)
        self.update_period = int(update_period)
        self.always_update_first = int(always_update_first)
        self.t = 0
        self.R = None        # rank x dim, orthonormal rows
        self.d = None        # diag(D_t)
        self.rho = None
        self.last = {}       # diagnostics of the latest call

    # -- the Fisher-factor model ------------------------------------------------
    def fisher(self) -> np.ndarray:
        """Dense F_t (eq. low:rank); for tests on small dimensions."""
        return self.R.T @ (self.d[:, None] * self.R) + self.rho * np.eye(self.dim)

    def will_update(self) -> bool:
        """App. B.4 / B.5: update on the first ten minibatches and then every J-th."""
        return self.t < self.always_update_first or self.t % self.update_period == 0

    def reset(self) -> None:
        """Forget the state; the next minibatch re-initialises it (App. B.3.2)."""
        self.t = 0
        self.R = self.d = self.rho = None

    # -- one call -----------------------------------------------------------------
    def precondition(self, M: np.ndarray):
        """Return (Mbar, gamma, rownorm2) for one minibatch and advance the state."""
        M = np.asarray(M, dtype=np.float64)
        N, D = M.shape
        if D != self.dim:
            raise ValueError("column count does not match the preconditioner")
        if self.t == 0:
            if self.rank >= min(N, D) and self.rank > 0:
                raise ValueError("need rank < min(rows, dim) at initialisation")
            self.R, self.d, self.rho = initial_state(M, self.rank, self.epsilon)

        eta = forgetting_factor(N, self.num_samples_history)
        R, d, rho = self.R, self.d, self.rho
        beta, e = smoothing_and_scales(d, rho, self.alpha, D)

        # Xhat = beta X G^{-1} = X - (X R^T) E R   (eq. hatxt + Woodbury)
        Mhat = M - ((M @ R.T) * e[None, :]) @ R
        p = np.sum(Mhat * Mhat, axis=1)                       # eq. pi
        tr_M = float(np.sum(np.sum(M * M, axis=1)))           # direct sum of squares, row by row
        tr_Mhat = float(np.sum(p))
        gamma = math.sqrt(tr_M / tr_Mhat) if tr_Mhat > 0.0 else 1.0   # eq. gammat
        Mbar = gamma * Mhat
        rownorm2 = (gamma * gamma) * p
        self.last = dict(eta=eta, beta=beta, e=e.copy(), gamma=gamma, tr_M=tr_M,
                         tr_Mhat=tr_Mhat, updated=False, floored=False, reorthogonalised=False)

        if self.will_update():
            self._update(M, eta, tr_M)
        self.t += 1
        return Mbar, gamma, rownorm2

    def _update(self, M: np.ndarray, eta: float, tr_M: float) -> None:
        N, D = M.shape
        R, d, rho, eps = self.R, self.d, self.rho, self.epsilon
        rank = self.rank
        if rank == 0:
            rho_dash = ((eta / N) * tr_M + (1.0 - eta) * D * rho) / D
            self.rho = max(eps, rho_dash)
            self.last["updated"] = True
            return
        # Y_t = R_t T_t with T_t = eta S_t + (1 - eta) F_t   (eq. yt)
        Y = (eta / N) * ((R @ M.T) @ M) + (1.0 - eta) * ((d + rho)[:, None] * R)
        Z = Y @ Y.T                                           # eq. zt:def
        Z = 0.5 * (Z + Z.T)
        c, U = np.linalg.eigh(Z)                              # eq. zt:eig, ascending
        c = c[::-1].copy()
        U = U[:, ::-1]
        floor = (1.0 - eta) ** 2 * rho ** 2                   # App. B.3 after eq. zt:eig:repeat
        floored = bool(np.any(c < floor))
        c = np.maximum(c, floor)
        sqrt_c = np.sqrt(c)
        rho_dash = ((eta / N) * tr_M + (1.0 - eta) * (D * rho + float(np.sum(d)))
                    - float(np.sum(sqrt_c))) / (D - rank)     # eq. rhodash
        d_new = np.maximum(sqrt_c - rho_dash, eps)            # eq. dt1
        rho_new = max(eps, rho_dash)                          # eq. rhot1
        R_new = (U.T @ Y) / sqrt_c[:, None]                   # eq. rt1:def
        reorth = False
        if floored or c[0] > ORTHO_COND_LIMIT * c[-1]:
            R_new, reorth = reorthogonalise_if_needed(R_new)
        self.R, self.d, self.rho = R_new, d_new, rho_new
        self.last.update(updated=True, floored=floored, reorthogonalised=reorth,
                         c=c.copy(), rho_dash=rho_dash)

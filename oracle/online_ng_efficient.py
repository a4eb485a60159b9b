"""Online natural-gradient preconditioner in the efficient form (float64, NumPy).

TEST INFRASTRUCTURE ONLY - see oracle/__init__.py.

This is the route of App. B.3 as summarised in App. B.5: the state is
W_t = E_t^{1/2} R_t, diag(D_t) and rho_t; one call forms H = X W^T, J = H^T X,
K = J J^T, L = H^T H, the R x R matrix Z_t from K and L (eq. zt:compute), its
eigen-decomposition, and W_{t+1} = A_t B_t (eq. wt1).  The tests require it to
reproduce the definitional form of oracle/online_ng.py step by step, which pins
every formula of App. B.3 independently of any GPU code.
"""
from __future__ import annotations

import math

import numpy as np

from .online_ng import (ORTHO_COND_LIMIT, ORTHO_TOLERANCE, forgetting_factor,
                        initial_state, smoothing_and_scales)


class OnlineNaturalGradientEfficient:
    def __init__(self, dim: int, rank: int, alpha: float = 4.0,
                 num_samples_history: float = 2000.0, epsilon: float = 1.0e-10,
                 update_period: int = 4, always_update_first: int = 10,
                 trace_identity: bool = False):
        if not (0 < rank < dim):
            raise ValueError("need 0 < rank < dim")
        self.dim, self.rank = dim, rank
        self.alpha = float(alpha)
        self.num_samples_history = float(num_samples_history)
        self.epsilon = float(epsilon)
        self.update_period = int(update_period)
        self.always_update_first = int(always_update_first)
        self.trace_identity = bool(trace_identity)   # use eq. trxxt instead of the direct sum
        self.t = 0
        self.W = self.d = self.rho = None
        self.last = {}

    def fisher(self) -> np.ndarray:
        """Dense F_t recovered from W_t = E_t^{1/2} R_t."""
        _, e = smoothing_and_scales(self.d, self.rho, self.alpha, self.dim)
        R = self.W / np.sqrt(e)[:, None]
        return R.T @ (self.d[:, None] * R) + self.rho * np.eye(self.dim)

    def will_update(self) -> bool:
        return self.t < self.always_update_first or self.t % self.update_period == 0

    def precondition(self, M: np.ndarray):
        M = np.asarray(M, dtype=np.float64)
        N, D = M.shape
        alpha, eps, rank = self.alpha, self.epsilon, self.rank
        if self.t == 0:
            R0, self.d, self.rho = initial_state(M, rank, eps)
            _, e0 = smoothing_and_scales(self.d, self.rho, alpha, D)
            self.W = np.sqrt(e0)[:, None] * R0                 # eq. wt:def
        eta = forgetting_factor(N, self.num_samples_history)
        W, d, rho = self.W, self.d, self.rho
        update = self.will_update()

        H = M @ W.T                                            # eq. ht
        Mhat = M - H @ W                                       # eq. hatxt:compute:2
        p = np.sum(Mhat * Mhat, axis=1)                        # eq. pi
        tr_Mhat = float(np.sum(p))
        if update:
            beta, e = smoothing_and_scales(d, rho, alpha, D)
            J = H.T @ M
            K = J @ J.T
            L = H.T @ H if N <= D else W @ J.T                 # App. B.5: two routes to L_t
            L = 0.5 * (L + L.T)
        if update and self.trace_identity:
            tr_M = tr_Mhat - float(np.sum(np.diag(L) * e)) + 2.0 * float(np.trace(L))   # eq. trxxt
        else:
            tr_M = float(np.sum(M * M))
        gamma = math.sqrt(tr_M / tr_Mhat) if tr_Mhat > 0.0 else 1.0
        Mbar = gamma * Mhat
        rownorm2 = gamma * gamma * p

        if update:
            inv_sqrt_e = 1.0 / np.sqrt(e)
            dr = d + rho
            Ks = inv_sqrt_e[:, None] * K * inv_sqrt_e[None, :]
            Ls = inv_sqrt_e[:, None] * L * inv_sqrt_e[None, :]
            Z = ((eta / N) ** 2) * Ks + np.diag(((1.0 - eta) * dr) ** 2) \
                + (eta * (1.0 - eta) / N) * (Ls * dr[None, :] + dr[:, None] * Ls)   # eq. zt:compute
            Z = 0.5 * (Z + Z.T)
            c, U = np.linalg.eigh(Z)
            c = c[::-1].copy()
            U = U[:, ::-1]
            floor = (1.0 - eta) ** 2 * rho ** 2
            floored = bool(np.any(c < floor))
            c = np.maximum(c, floor)
            sqrt_c = np.sqrt(c)
            rho_dash = ((eta / N) * tr_M + (1.0 - eta) * (D * rho + float(np.sum(d)))
                        - float(np.sum(sqrt_c))) / (D - rank)  # eq. rhodash2
            d_new = np.maximum(sqrt_c - rho_dash, eps)
            rho_new = max(eps, rho_dash)
            _, e_new = smoothing_and_scales(d_new, rho_new, alpha, D)
            A = (eta / N) * (np.sqrt(e_new) / sqrt_c)[:, None] * U.T * inv_sqrt_e[None, :]
            B = J + (N * (1.0 - eta) / eta) * (dr[:, None] * W)
            W_new = A @ B                                      # eq. wt1
            reorth = False
            if floored or c[0] > ORTHO_COND_LIMIT * c[-1]:
                s = 1.0 / np.sqrt(e_new)
                O = s[:, None] * (W_new @ W_new.T) * s[None, :]
                if float(np.max(np.abs(O - np.eye(rank)))) > ORTHO_TOLERANCE:
                    Lc = np.linalg.cholesky(O)
                    Mfix = np.sqrt(e_new)[:, None] * np.linalg.inv(Lc) * s[None, :]
                    W_new = Mfix @ W_new
                    reorth = True
            self.W, self.d, self.rho = W_new, d_new, rho_new
            self.last = dict(floored=floored, reorthogonalised=reorth)
        self.t += 1
        return Mbar, gamma, rownorm2

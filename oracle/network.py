"""One worker's NG-SGD minibatch step on a feed-forward net (float64, NumPy).

TEST INFRASTRUCTURE ONLY - see oracle/__init__.py.

The objective is the sum over the frames of a minibatch of log p(y_i | x_i)
(Sec. 2), maximised by gradient ascent.  Gradients are summed over the
minibatch, never divided by its size (Sec. 4.6, App. C.1).  Each affine layer
keeps its bias as the last column of its weight matrix and sees its input with
a 1 appended (Sec. 4.4).  The update of layer i is

    W_i <- W_i + lr * Obar_i^T Xbar_i                      (Sec. 4.6)

where O_i (N x Dout) is the derivative of the objective w.r.t. the affine
output, X_i (N x (Din+1)) the layer input, and the bar marks the output of that
matrix's own online preconditioner (2I instances, App. B.5) or, with
method="simple", the output of the simple method of App. A applied to that
matrix (no state; Fisher factors from the other rows of the same minibatch).  Back-propagation
itself runs on the unmodified derivatives: the natural gradient only modifies
the two matrices that enter the update (App. C.3, last paragraph).

Nonlinearities: tanh, or p-norm with p = 2 over groups of `pnorm_group`
adjacent outputs, y_j = sqrt(sum_k a_k^2) (the paper cites the p-norm paper for
the definition; derivative a_k / y_j, taken as 0 where y_j = 0).

Two stabilisers of the paper's recipe are optional here:
  * `renorm`: the renormalisation layer the paper's p-norm nets carry after
    each p-norm (App. C.8, footnote).  The paper does not define it; the
    reading used is: each row y is divided by max(rms(y), RENORM_FLOOR), with
    rms(y) = sqrt(mean_j y_j^2), so that rows leave with unit rms.
  * `max_change_per_sample` (App. C.3): the update of each layer is scaled by
        a_t = min(1, N * max_change_per_sample / (lr * sum_i ||obar_i|| ||xbar_i||))
    using the rows of the preconditioned matrices (a_t = 1 if the sum is 0).
"""
from __future__ import annotations

import numpy as np

from .online_ng import OnlineNaturalGradient
from .simple_ng import simple_ng

TANH = 0
PNORM = 1
RENORM_FLOOR = 1.0e-20


def append_ones(A: np.ndarray) -> np.ndarray:
    return np.concatenate([A, np.ones((A.shape[0], 1))], axis=1)


def pnorm_forward(A: np.ndarray, group: int) -> np.ndarray:
    N, D = A.shape
    return np.sqrt(np.sum(A.reshape(N, D // group, group) ** 2, axis=2))


def pnorm_backward(dY: np.ndarray, A: np.ndarray, Y: np.ndarray, group: int) -> np.ndarray:
    N, D = A.shape
    safe = np.where(Y > 0.0, Y, 1.0)
    scale = np.where(Y > 0.0, dY / safe, 0.0)
    return (A.reshape(N, D // group, group) * scale[:, :, None]).reshape(N, D)


def renorm_forward(Y: np.ndarray):
    """Rows scaled to unit rms; returns (Y / sigma, sigma) with sigma = max(rms, floor)."""
    sigma = np.maximum(np.sqrt(np.mean(Y * Y, axis=1)), RENORM_FLOOR)
    return Y / sigma[:, None], sigma


def renorm_backward(dYn: np.ndarray, Yn: np.ndarray, sigma: np.ndarray) -> np.ndarray:
    """Derivative through y -> y / rms(y): (dYn - Yn * mean_j(dYn_j Yn_j)) / sigma.

    Rows whose rms sat on the floor were scaled by a constant, so only 1/sigma applies there.
    """
    K = Yn.shape[1]
    proj = np.sum(dYn * Yn, axis=1) / K
    proj = np.where(sigma > RENORM_FLOOR, proj, 0.0)
    return (dYn - Yn * proj[:, None]) / sigma[:, None]


def log_softmax(A: np.ndarray) -> np.ndarray:
    m = np.max(A, axis=1, keepdims=True)
    return A - m - np.log(np.sum(np.exp(A - m), axis=1, keepdims=True))


class NGSGDNetwork:
    """dims[0] is the input dimension, dims[1:] the affine output dimensions.

    nonlin[l] (l = 0 .. n_layers-2) is the nonlinearity after affine layer l;
    the last affine layer feeds a log-softmax.  A p-norm layer divides the
    dimension by `pnorm_group`.
    """

    def __init__(self, dims, nonlin, weights, pnorm_group: int = 10, rank_in: int = 20,
                 rank_out: int = 80, alpha: float = 4.0, num_samples_history: float = 2000.0,
                 epsilon: float = 1.0e-10, update_period: int = 4, natural_gradient: bool = True,
                 renorm: bool = False, max_change_per_sample: float = 0.0, method: str = "online",
                 simple_epsilon: float = 1.0e-20):
        assert method in ("online", "simple")
        self.method = method                 # which estimate of the Fisher factors (Sec. 4.5)
        self.simple_alpha = alpha
        self.simple_epsilon = simple_epsilon
        self.dims = list(dims)
        self.n_layers = len(dims) - 1
        self.nonlin = list(nonlin)
        assert len(self.nonlin) == self.n_layers - 1
        self.pnorm_group = pnorm_group
        self.natural_gradient = natural_gradient
        self.renorm = renorm
        self.max_change_per_sample = float(max_change_per_sample)
        self.in_dims = []
        d_in = dims[0]
        for l in range(self.n_layers):
            self.in_dims.append(d_in)
            if l < self.n_layers - 1:
                d_in = dims[l + 1] // pnorm_group if self.nonlin[l] == PNORM else dims[l + 1]
        self.W = [np.array(w, dtype=np.float64) for w in weights]
        for l in range(self.n_layers):
            assert self.W[l].shape == (dims[l + 1], self.in_dims[l] + 1)
        kw = dict(alpha=alpha, num_samples_history=num_samples_history, epsilon=epsilon,
                  update_period=update_period)
        self.precond_in = [OnlineNaturalGradient(self.in_dims[l] + 1, rank_in, **kw)
                           for l in range(self.n_layers)]
        self.precond_out = [OnlineNaturalGradient(dims[l + 1], rank_out, **kw)
                            for l in range(self.n_layers)]
        self.last = {}

    # -- pieces, exposed for the tests ---------------------------------------------
    def forward(self, x: np.ndarray):
        """Returns (layer inputs with ones column, affine outputs, log-probabilities)."""
        Xin, A = [], []
        self._sigma = [None] * self.n_layers
        cur = np.asarray(x, dtype=np.float64)
        for l in range(self.n_layers):
            Xl = append_ones(cur)
            Al = Xl @ self.W[l].T
            Xin.append(Xl)
            A.append(Al)
            if l < self.n_layers - 1:
                if self.nonlin[l] == TANH:
                    cur = np.tanh(Al)
                else:
                    cur = pnorm_forward(Al, self.pnorm_group)
                    if self.renorm:
                        cur, self._sigma[l] = renorm_forward(cur)
        return Xin, A, log_softmax(A[-1])

    def objective(self, x: np.ndarray, labels: np.ndarray) -> float:
        logp = self.forward(x)[2]
        return float(np.sum(logp[np.arange(len(labels)), labels]))

    def backward(self, Xin, A, logp, labels):
        """Derivatives O_l of the summed objective w.r.t. every affine output."""
        N = len(labels)
        O = [None] * self.n_layers
        Olast = -np.exp(logp)
        Olast[np.arange(N), labels] += 1.0
        O[-1] = Olast
        for l in range(self.n_layers - 1, 0, -1):
            dX = O[l] @ self.W[l][:, :-1]                      # drop the bias column
            Aprev = A[l - 1]
            Yprev = Xin[l][:, :-1]
            if self.nonlin[l - 1] == TANH:
                O[l - 1] = dX * (1.0 - Yprev * Yprev)
            else:
                if self.renorm:
                    sigma = self._sigma[l - 1]
                    dX = renorm_backward(dX, Yprev, sigma)
                    Yprev = Yprev * sigma[:, None]             # the p-norm output before renormalisation
                O[l - 1] = pnorm_backward(dX, Aprev, Yprev, self.pnorm_group)
        return O

    def gradients(self, x, labels):
        """Plain (un-preconditioned) summed gradients O_l^T Xin_l, for the tests."""
        Xin, A, logp = self.forward(x)
        O = self.backward(Xin, A, logp, labels)
        return [O[l].T @ Xin[l] for l in range(self.n_layers)]

    # -- the step ------------------------------------------------------------------
    def step(self, x: np.ndarray, labels: np.ndarray, lr: float) -> float:
        """One NG-SGD minibatch step; returns sum_i log p(y_i | x_i) before the update."""
        labels = np.asarray(labels)
        Xin, A, logp = self.forward(x)
        obj = float(np.sum(logp[np.arange(len(labels)), labels]))
        O = self.backward(Xin, A, logp, labels)
        deltas, Obar_all, Xbar_all, scales = [], [], [], []
        for l in range(self.n_layers):
            if self.natural_gradient and self.method == "simple":
                Obar, _, rn_o = simple_ng(O[l], self.simple_alpha, self.simple_epsilon)
                Xbar, _, rn_x = simple_ng(Xin[l], self.simple_alpha, self.simple_epsilon)
            elif self.natural_gradient:
                Obar, _, rn_o = self.precond_out[l].precondition(O[l])
                Xbar, _, rn_x = self.precond_in[l].precondition(Xin[l])
            else:
                Obar, Xbar = O[l], Xin[l]
                rn_o, rn_x = np.sum(Obar * Obar, axis=1), np.sum(Xbar * Xbar, axis=1)
            a_t = 1.0
            if self.max_change_per_sample > 0.0:
                bound = lr * float(np.sum(np.sqrt(rn_o * rn_x)))          # App. C.3, eq. delta_t_approx
                if bound > 0.0:
                    a_t = min(1.0, len(labels) * self.max_change_per_sample / bound)
            scales.append(a_t)
            delta = a_t * (Obar.T @ Xbar)
            deltas.append(delta)
            Obar_all.append(Obar)
            Xbar_all.append(Xbar)
        for l in range(self.n_layers):
            self.W[l] = self.W[l] + lr * deltas[l]
        self.last = dict(O=O, Xin=Xin, Obar=Obar_all, Xbar=Xbar_all, delta=deltas, logp=logp,
                         max_change_scale=scales)
        return obj

    def reset_preconditioners(self) -> None:
        for p in self.precond_in + self.precond_out:
            p.reset()

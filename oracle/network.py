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
matrix's own online preconditioner (2I instances, App. B.5).  Back-propagation
itself runs on the unmodified derivatives: the natural gradient only modifies
the two matrices that enter the update (App. C.3, last paragraph).

Nonlinearities: tanh, or p-norm with p = 2 over groups of `pnorm_group`
adjacent outputs, y_j = sqrt(sum_k a_k^2) (the paper cites the p-norm paper for
the definition; derivative a_k / y_j, taken as 0 where y_j = 0).
"""
from __future__ import annotations

import numpy as np

from .online_ng import OnlineNaturalGradient

TANH = 0
PNORM = 1


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
                 epsilon: float = 1.0e-10, update_period: int = 4, natural_gradient: bool = True):
        self.dims = list(dims)
        self.n_layers = len(dims) - 1
        self.nonlin = list(nonlin)
        assert len(self.nonlin) == self.n_layers - 1
        self.pnorm_group = pnorm_group
        self.natural_gradient = natural_gradient
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
        cur = np.asarray(x, dtype=np.float64)
        for l in range(self.n_layers):
            Xl = append_ones(cur)
            Al = Xl @ self.W[l].T
            Xin.append(Xl)
            A.append(Al)
            if l < self.n_layers - 1:
                cur = np.tanh(Al) if self.nonlin[l] == TANH else pnorm_forward(Al, self.pnorm_group)
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
        deltas, Obar_all, Xbar_all = [], [], []
        for l in range(self.n_layers):
            if self.natural_gradient:
                Obar, _, _ = self.precond_out[l].precondition(O[l])
                Xbar, _, _ = self.precond_in[l].precondition(Xin[l])
            else:
                Obar, Xbar = O[l], Xin[l]
            delta = Obar.T @ Xbar
            deltas.append(delta)
            Obar_all.append(Obar)
            Xbar_all.append(Xbar)
        for l in range(self.n_layers):
            self.W[l] = self.W[l] + lr * deltas[l]
        self.last = dict(O=O, Xin=Xin, Obar=Obar_all, Xbar=Xbar_all, delta=deltas, logp=logp)
        return obj

    def reset_preconditioners(self) -> None:
        for p in self.precond_in + self.precond_out:
            p.reset()

"""MI355X-native NG-SGD minibatch step (online natural-gradient SGD, arXiv 1410.7455).

Thin ctypes binding over the C ABI of ``libngsgd.so`` (declared in ``include/ngsgd.h``).
Every step of the method runs in the library's HIP kernels; this module only marshals
arguments.  PyTorch supplies device memory and streams.

The shared library is built in-tree by ``paper_1410_7455_amd.build.build()``; importing the
binding without it raises, there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, byref, c_char_p, c_double, c_float, c_int, c_int32, c_int64, c_size_t, c_void_p

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libngsgd.so")

NGSGD_OK = 0
NGSGD_EINVAL = -1
NGSGD_ENOMEM = -2
NGSGD_EHIP = -3
NGSGD_TANH = 0
NGSGD_PNORM = 1
NGSGD_SIDE_INPUT = 0
NGSGD_SIDE_OUTPUT = 1
NGSGD_MAX_RANK = 96
NGSGD_MAX_LAYERS = 16
NGSGD_METHOD_ONLINE = 0
NGSGD_METHOD_SIMPLE = 1


class NgsgdError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = _lib.ngsgd_strerror(code).decode() if _lib is not None else str(code)
        extra = f" (hipError {_lib.ngsgd_last_hip_error()})" if _lib is not None and code == NGSGD_EHIP else ""
        super().__init__(f"{where}: {msg}{extra}")


class ngsgd_config(ctypes.Structure):
    _fields_ = [
        ("n_layers", c_int32), ("dims", POINTER(c_int32)), ("nonlin", POINTER(c_int32)),
        ("pnorm_group", c_int32), ("max_batch", c_int32), ("rank_in", c_int32), ("rank_out", c_int32),
        ("alpha", c_float), ("num_samples_history", c_float), ("epsilon", c_float),
        ("update_period", c_int32), ("always_update_first", c_int32), ("renorm", c_int32),
        ("max_change_per_sample", c_float), ("method", c_int32), ("simple_epsilon", c_float),
        ("side_streams", c_int32),
    ]


# name -> (restype, argtypes); one entry per symbol declared in include/ngsgd.h
_SIGNATURES = {
    "ngsgd_precond_workspace_bytes": (c_int, [c_int32, c_int32, c_int32, POINTER(c_size_t)]),
    "ngsgd_precond_create": (c_int, [c_int32, c_int32, c_int32, c_float, c_float, c_float, c_int32, c_int32,
                                     c_void_p, c_size_t, POINTER(c_void_p)]),
    "ngsgd_precond_destroy": (c_int, [c_void_p]),
    "ngsgd_precond_reset": (c_int, [c_void_p]),
    "ngsgd_precondition": (c_int, [c_void_p, c_void_p, c_int32, c_int32, c_void_p, c_void_p, c_void_p]),
    "ngsgd_precond_get_state": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, POINTER(c_int64), c_void_p]),
    "ngsgd_precond_diagnostics": (c_int, [c_void_p, POINTER(c_int32), POINTER(c_int32), c_void_p]),
    "ngsgd_precond_set_state": (c_int, [c_void_p, c_void_p, c_void_p, c_double, c_int64, c_void_p]),
    "ngsgd_simple_workspace_bytes": (c_int, [c_int32, c_int32, POINTER(c_size_t)]),
    "ngsgd_precondition_simple": (c_int, [c_void_p, c_int32, c_int32, c_int32, c_float, c_float, c_void_p, c_size_t,
                                          c_void_p, c_void_p, c_void_p]),
    "ngsgd_precondition_simple_static": (c_int, [c_void_p, c_int32, c_int32, c_int32, c_float, c_float, c_void_p,
                                                 c_void_p, c_void_p]),
    "ngsgd_workspace_bytes": (c_int, [POINTER(ngsgd_config), POINTER(c_size_t)]),
    "ngsgd_create": (c_int, [POINTER(ngsgd_config), c_void_p, c_size_t, POINTER(c_void_p)]),
    "ngsgd_destroy": (c_int, [c_void_p]),
    "ngsgd_step": (c_int, [c_void_p, c_void_p, c_void_p, c_int32, c_float, c_void_p, c_void_p]),
    "ngsgd_join": (c_int, [c_void_p, c_void_p]),
    "ngsgd_average": (c_int, [POINTER(c_void_p), c_int32, c_int32, c_void_p]),
    "ngsgd_get_params": (c_int, [c_void_p, c_int32, c_void_p, c_void_p]),
    "ngsgd_set_params": (c_int, [c_void_p, c_int32, c_void_p, c_void_p]),
    "ngsgd_net_precond": (c_int, [c_void_p, c_int32, c_int32, POINTER(c_void_p)]),
    "ngsgd_last_preconditioned": (c_int, [c_void_p, c_int32, c_int32, c_void_p, c_void_p]),
    "ngsgd_last_gradient": (c_int, [c_void_p, c_int32, c_void_p, c_void_p]),
    "ngsgd_last_max_change_scale": (c_int, [c_void_p, c_int32, c_void_p, c_void_p]),
    "ngsgd_profile_enable": (c_int, [c_int32]),
    "ngsgd_profile_read": (c_int, [POINTER(c_double), POINTER(c_int64), c_int32]),
    "ngsgd_strerror": (c_char_p, [c_int]),
    "ngsgd_set_wait_limit_us": (c_int, [c_int64]),
    "ngsgd_last_hip_error": (c_int, []),
    "ngsgd_version": (c_int, []),
}

_lib = None


def load_library():
    """Loads libngsgd.so and binds every declared entry point; raises if the library is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_1410_7455_amd.build` "
            "(hipcc, gfx950); there is no CPU fallback")
    try:
        # PyTorch ships its own HIP runtime: load it first, so that the library binds to the same copy as the
        # tensors whose pointers it is given (two runtimes in one process do not know each other's memory)
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(LIB_PATH)
    for name, (restype, argtypes) in _SIGNATURES.items():
        fn = getattr(lib, name)          # AttributeError if the symbol is not exported
        fn.restype = restype
        fn.argtypes = argtypes
    _lib = lib
    return lib


def _check(code: int, where: str) -> None:
    if code != NGSGD_OK:
        raise NgsgdError(code, where)


def _stream_ptr(stream=None):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return c_void_p(s.cuda_stream)


def _ptr(t):
    return c_void_p(0) if t is None else c_void_p(t.data_ptr())


class Preconditioner:
    """One online natural-gradient instance (ngsgd_precond_*) on the current CUDA/HIP device."""

    def __init__(self, dim, rank, max_batch, alpha=4.0, num_samples_history=2000.0, epsilon=1e-10,
                 update_period=4, always_update_first=10, _borrowed=None):
        import torch
        self.lib = load_library()
        self.dim, self.rank, self.max_batch = dim, rank, max_batch
        self._owner = None
        if _borrowed is not None:
            self.handle, self._owner = _borrowed
            self.workspace = None
            return
        nbytes = c_size_t(0)
        _check(self.lib.ngsgd_precond_workspace_bytes(dim, rank, max_batch, byref(nbytes)),
               "ngsgd_precond_workspace_bytes")
        self.workspace = torch.empty(nbytes.value, dtype=torch.uint8, device="cuda")
        h = c_void_p(0)
        _check(self.lib.ngsgd_precond_create(dim, rank, max_batch, alpha, num_samples_history, epsilon,
                                             update_period, always_update_first, _ptr(self.workspace),
                                             nbytes.value, byref(h)), "ngsgd_precond_create")
        self.handle = h

    def close(self):
        if self._owner is None and self.handle is not None:
            self.lib.ngsgd_precond_destroy(self.handle)
        self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def reset(self):
        _check(self.lib.ngsgd_precond_reset(self.handle), "ngsgd_precond_reset")

    def precondition(self, M, gamma=None, rownorm2=None, stream=None):
        """In place on the float32 CUDA tensor M (N x dim, row stride M.stride(0))."""
        assert M.is_cuda and M.dtype.is_floating_point and M.element_size() == 4 and M.stride(1) == 1
        _check(self.lib.ngsgd_precondition(self.handle, _ptr(M), M.shape[0], M.stride(0), _ptr(gamma),
                                           _ptr(rownorm2), _stream_ptr(stream)), "ngsgd_precondition")

    def get_state(self):
        import torch
        W = torch.empty((self.rank, self.dim), dtype=torch.float32, device="cuda")
        d = torch.empty(self.rank, dtype=torch.float64, device="cuda")
        rho = torch.empty(1, dtype=torch.float64, device="cuda")
        t = c_int64(0)
        _check(self.lib.ngsgd_precond_get_state(self.handle, _ptr(W), _ptr(d), _ptr(rho), byref(t),
                                                _stream_ptr()), "ngsgd_precond_get_state")
        torch.cuda.synchronize()
        return W, d, float(rho.item()), t.value

    def diagnostics(self):
        """(flags, Jacobi sweeps) of the latest factor update; waits for the stream."""
        flags, sweeps = c_int32(0), c_int32(0)
        _check(self.lib.ngsgd_precond_diagnostics(self.handle, byref(flags), byref(sweeps), _stream_ptr()),
               "ngsgd_precond_diagnostics")
        return flags.value, sweeps.value

    def set_state(self, R, d, rho, t):
        """R: rank x dim float64 CUDA tensor with orthonormal rows, d: rank float64, rho > 0, t >= 1."""
        assert R.is_cuda and R.dtype.itemsize == 8 and R.is_contiguous() and tuple(R.shape) == (self.rank, self.dim)
        assert d.is_cuda and d.dtype.itemsize == 8 and d.numel() == self.rank
        _check(self.lib.ngsgd_precond_set_state(self.handle, _ptr(R), _ptr(d), float(rho), int(t),
                                                _stream_ptr()), "ngsgd_precond_set_state")


class SimplePreconditioner:
    """The simple method of App. A (ngsgd_precondition_simple): stateless, the workspace is kept for reuse."""

    def __init__(self, max_rows, dim, alpha=4.0, epsilon=1e-20):
        import torch
        self.lib = load_library()
        self.max_rows, self.dim, self.alpha, self.epsilon = max_rows, dim, alpha, epsilon
        nbytes = c_size_t(0)
        _check(self.lib.ngsgd_simple_workspace_bytes(max_rows, dim, byref(nbytes)), "ngsgd_simple_workspace_bytes")
        self.workspace_bytes = nbytes.value
        self.workspace = torch.empty(nbytes.value, dtype=torch.uint8, device="cuda")

    def precondition(self, M, gamma=None, rownorm2=None, stream=None):
        """In place on the float32 CUDA tensor M (N x dim, row stride M.stride(0)), N <= max_rows."""
        assert M.is_cuda and M.element_size() == 4 and M.stride(1) == 1 and M.shape[1] == self.dim
        _check(self.lib.ngsgd_precondition_simple(_ptr(M), M.shape[0], M.shape[1], M.stride(0), self.alpha,
                                                  self.epsilon, _ptr(self.workspace), self.workspace_bytes,
                                                  _ptr(gamma), _ptr(rownorm2), _stream_ptr(stream)),
               "ngsgd_precondition_simple")


def precondition_simple_static(M, alpha=4.0, epsilon=1e-20, gamma=None, rownorm2=None, stream=None):
    """ngsgd_precondition_simple_static: the simple method in place on M with the library's fixed scratch."""
    assert M.is_cuda and M.element_size() == 4 and M.stride(1) == 1
    _check(load_library().ngsgd_precondition_simple_static(_ptr(M), M.shape[0], M.shape[1], M.stride(0), alpha,
                                                           epsilon, _ptr(gamma), _ptr(rownorm2),
                                                           _stream_ptr(stream)),
           "ngsgd_precondition_simple_static")


class Network:
    """One replica (ngsgd_create / ngsgd_step / ...)."""

    def __init__(self, dims, nonlin, max_batch, pnorm_group=10, rank_in=20, rank_out=80, alpha=4.0,
                 num_samples_history=2000.0, epsilon=1e-10, update_period=4, always_update_first=10,
                 renorm=False, max_change_per_sample=0.0, method="online", simple_epsilon=1e-20, side_streams=0):
        import torch
        self.lib = load_library()
        self.method = {"online": NGSGD_METHOD_ONLINE, "simple": NGSGD_METHOD_SIMPLE}[method]
        self.dims = list(dims)
        self.nonlin = list(nonlin)
        self.n_layers = len(dims) - 1
        self.pnorm_group = pnorm_group
        self.max_batch = max_batch
        self.rank_in, self.rank_out = rank_in, rank_out
        self.in_dims = []
        d_in = dims[0]
        for l in range(self.n_layers):
            self.in_dims.append(d_in)
            if l < self.n_layers - 1:
                d_in = dims[l + 1] // pnorm_group if nonlin[l] == NGSGD_PNORM else dims[l + 1]
        self._dims_arr = (c_int32 * len(dims))(*dims)
        self._nonlin_arr = (c_int32 * max(1, len(nonlin)))(*nonlin)
        cfg = ngsgd_config(self.n_layers, self._dims_arr, self._nonlin_arr, pnorm_group, max_batch, rank_in,
                           rank_out, alpha, num_samples_history, epsilon, update_period, always_update_first,
                           1 if renorm else 0, max_change_per_sample, self.method, simple_epsilon, side_streams)
        nbytes = c_size_t(0)
        _check(self.lib.ngsgd_workspace_bytes(byref(cfg), byref(nbytes)), "ngsgd_workspace_bytes")
        self.workspace_bytes = nbytes.value
        self.workspace = torch.empty(nbytes.value, dtype=torch.uint8, device="cuda")
        h = c_void_p(0)
        _check(self.lib.ngsgd_create(byref(cfg), _ptr(self.workspace), nbytes.value, byref(h)), "ngsgd_create")
        self.handle = h
        self._logprob = torch.zeros(1, dtype=torch.float64, device="cuda")

    def close(self):
        if self.handle is not None:
            self.lib.ngsgd_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_params(self, layer, w):
        assert w.is_cuda and w.is_contiguous() and w.element_size() == 4
        assert tuple(w.shape) == (self.dims[layer + 1], self.in_dims[layer] + 1)
        _check(self.lib.ngsgd_set_params(self.handle, layer, _ptr(w), _stream_ptr()), "ngsgd_set_params")

    def get_params(self, layer):
        import torch
        w = torch.empty((self.dims[layer + 1], self.in_dims[layer] + 1), dtype=torch.float32, device="cuda")
        _check(self.lib.ngsgd_get_params(self.handle, layer, _ptr(w), _stream_ptr()), "ngsgd_get_params")
        return w

    def step(self, x, labels, lr, logprob_out=None, stream=None):
        """Enqueues one minibatch step; the sum of log-probabilities lands in `logprob_out` (1 float64)."""
        assert x.is_cuda and x.is_contiguous() and x.element_size() == 4 and x.shape[1] == self.dims[0]
        assert labels.is_cuda and labels.is_contiguous() and labels.element_size() == 4
        out = self._logprob if logprob_out is None else logprob_out
        _check(self.lib.ngsgd_step(self.handle, _ptr(x), _ptr(labels), x.shape[0], float(lr), _ptr(out),
                                   _stream_ptr(stream)), "ngsgd_step")
        return out

    def join(self, stream=None):
        """Makes the stream wait for the factor updates the network has in flight on its internal streams."""
        _check(self.lib.ngsgd_join(self.handle, _stream_ptr(stream)), "ngsgd_join")

    def precond(self, layer, side):
        h = c_void_p(0)
        _check(self.lib.ngsgd_net_precond(self.handle, layer, side, byref(h)), "ngsgd_net_precond")
        if not h.value:
            return None
        dim = self.in_dims[layer] + 1 if side == NGSGD_SIDE_INPUT else self.dims[layer + 1]
        rank = self.rank_in if side == NGSGD_SIDE_INPUT else self.rank_out
        return Preconditioner(dim, rank, self.max_batch, _borrowed=(h, self))

    def last_preconditioned(self, layer, side, n_rows):
        import torch
        dim = self.in_dims[layer] + 1 if side == NGSGD_SIDE_INPUT else self.dims[layer + 1]
        out = torch.empty((n_rows, dim), dtype=torch.float32, device="cuda")
        _check(self.lib.ngsgd_last_preconditioned(self.handle, layer, side, _ptr(out), _stream_ptr()),
               "ngsgd_last_preconditioned")
        return out

    def last_gradient(self, layer):
        import torch
        out = torch.empty((self.dims[layer + 1], self.in_dims[layer] + 1), dtype=torch.float32, device="cuda")
        _check(self.lib.ngsgd_last_gradient(self.handle, layer, _ptr(out), _stream_ptr()), "ngsgd_last_gradient")
        return out

    def last_max_change_scale(self, layer):
        import torch
        out = torch.empty(1, dtype=torch.float64, device="cuda")
        _check(self.lib.ngsgd_last_max_change_scale(self.handle, layer, _ptr(out), _stream_ptr()),
               "ngsgd_last_max_change_scale")
        return out


PROFILE_CATEGORIES = ["gemm_fwd", "gemm_bwd", "gemm_upd", "precond_h", "precond_j", "precond_xhat", "precond_kl",
                      "precond_small", "precond_wnew", "elementwise", "precond_misc", "init", "simple_gram",
                      "simple_inverse", "simple_apply", "precond_fused"]


def profile_enable(on: bool) -> None:
    _check(load_library().ngsgd_profile_enable(1 if on else 0), "ngsgd_profile_enable")


def profile_read():
    """{category: (milliseconds, bracketed launch groups)} since the last read."""
    n = len(PROFILE_CATEGORIES)
    ms = (c_double * n)()
    cnt = (c_int64 * n)()
    _check(load_library().ngsgd_profile_read(ms, cnt, n), "ngsgd_profile_read")
    return {name: (ms[i], cnt[i]) for i, name in enumerate(PROFILE_CATEGORIES)}


def set_wait_limit_us(microseconds: int) -> None:
    """ngsgd_set_wait_limit_us: bound of the fused apply kernel's wait between workgroups."""
    _check(load_library().ngsgd_set_wait_limit_us(int(microseconds)), "ngsgd_set_wait_limit_us")


def average(networks, reset_preconditioners=True, stream=None):
    """ngsgd_average over replicas living on the same device."""
    lib = load_library()
    arr = (c_void_p * len(networks))(*[n.handle for n in networks])
    _check(lib.ngsgd_average(arr, len(networks), 1 if reset_preconditioners else 0, _stream_ptr(stream)),
           "ngsgd_average")

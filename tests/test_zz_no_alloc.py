"""GPU test of the entry point that allocates nothing (ngsgd_precondition_simple_static), through the C ABI.

Its output is compared with ngsgd_precondition_simple (the same computation with a caller-provided workspace) and
with the float64 oracle, at the bar of the other parity tests (1e-4 relative Frobenius), on two calls in a row, the
second on a smaller matrix: the library's fixed scratch keeps the first call's contents.
"""
import ctypes
from ctypes import c_float, c_int32, c_size_t, c_void_p

import numpy as np
import pytest

from oracle.simple_ng import simple_ng

pytestmark = pytest.mark.gpu

TOL = 1.0e-4


def rel(a, b):
    return float(np.linalg.norm(np.asarray(a, np.float64) - np.asarray(b, np.float64)) /
                 max(np.linalg.norm(np.asarray(b, np.float64)), 1e-300))


def matrix(rng, N, D):
    scales = 0.97 ** np.arange(D) + 0.02
    x = rng.standard_normal((N, D)) * scales[None, :] + 0.3 * np.sin(np.arange(D))[None, :]
    return x[:, rng.permutation(D)].astype(np.float32)


def test_static_scratch_matches_workspace_variant_on_two_calls_in_a_row(ngsgd):
    import torch
    lib = ngsgd.load_library()
    stream = c_void_p(torch.cuda.current_stream().cuda_stream)
    rng = np.random.default_rng(7455)
    for N, D in ((300, 1000), (120, 77)):        # row space first, then a smaller column-space problem
        print(f"static scratch case N={N} D={D}", flush=True)
        M = matrix(rng, N, D)
        ld = D + (-D) % 4
        bufs, gammas, norms = [], [], []
        for which in ("workspace", "static"):
            buf = torch.zeros((N, ld), dtype=torch.float32, device="cuda")
            buf[:, :D] = torch.from_numpy(M).cuda()
            gamma = torch.zeros(1, dtype=torch.float32, device="cuda")
            rn2 = torch.zeros(N, dtype=torch.float32, device="cuda")
            if which == "workspace":
                nbytes = c_size_t(0)
                assert lib.ngsgd_simple_workspace_bytes(N, D, ctypes.byref(nbytes)) == 0
                ws = torch.empty(nbytes.value, dtype=torch.uint8, device="cuda")
                rc = lib.ngsgd_precondition_simple(c_void_p(buf.data_ptr()), c_int32(N), c_int32(D), c_int32(ld),
                                                   c_float(4.0), c_float(1e-20), c_void_p(ws.data_ptr()),
                                                   c_size_t(nbytes.value), c_void_p(gamma.data_ptr()),
                                                   c_void_p(rn2.data_ptr()), stream)
            else:
                torch.cuda.synchronize()
                before = torch.cuda.memory_allocated()
                rc = lib.ngsgd_precondition_simple_static(c_void_p(buf.data_ptr()), c_int32(N), c_int32(D),
                                                          c_int32(ld), c_float(4.0), c_float(1e-20),
                                                          c_void_p(gamma.data_ptr()), c_void_p(rn2.data_ptr()),
                                                          stream)
                assert torch.cuda.memory_allocated() == before
            assert rc == 0, (which, rc)
            torch.cuda.synchronize()
            bufs.append(buf[:, :D].cpu().numpy())
            gammas.append(float(gamma.item()))
            norms.append(rn2.cpu().numpy())
        want, g_o, rn_o = simple_ng(M.astype(np.float64))
        assert rel(bufs[1], bufs[0]) < TOL and rel(bufs[1], want) < TOL, (N, D)
        assert gammas[1] == pytest.approx(gammas[0], rel=1e-4) and gammas[1] == pytest.approx(g_o, rel=1e-4)
        assert rel(norms[1], norms[0]) < 2e-4 and rel(norms[1], rn_o) < 2e-4


def test_static_scratch_rejects_what_does_not_fit(ngsgd):
    import torch
    lib = ngsgd.load_library()
    stream = c_void_p(torch.cuda.current_stream().cuda_stream)
    N, D = 1024, 8000          # needs 51 MiB of scratch: over the fixed 16 MiB
    buf = torch.ones((N, D), dtype=torch.float32, device="cuda")
    rc = lib.ngsgd_precondition_simple_static(c_void_p(buf.data_ptr()), c_int32(N), c_int32(D), c_int32(D),
                                              c_float(4.0), c_float(1e-20), None, None, stream)
    assert rc == ngsgd.NGSGD_ENOMEM
    torch.cuda.synchronize()
    assert bool((buf == 1.0).all())          # nothing was enqueued
    rc = lib.ngsgd_precondition_simple_static(None, c_int32(4), c_int32(4), c_int32(4), c_float(4.0), c_float(1e-20),
                                              None, None, stream)
    assert rc == ngsgd.NGSGD_EINVAL

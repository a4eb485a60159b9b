"""GPU parity of the fused apply path (calls that do not update their factor, App. B.5 "without updating"):
ngsgd_precondition through the C ABI against the float64 oracle on the same seeded inputs.

The fused kernel lets the workgroups of a block of 64 rows wait for each other's share of H = X W^T; the wait is
bounded and a workgroup that gives up forms its H rows itself.  Both routes are held to the same bar (1e-4 relative
Frobenius): the ordinary one, and the slow one forced from the host with a wait limit of zero.
"""
import numpy as np
import pytest

import workloads
from oracle.online_ng import OnlineNaturalGradient

pytestmark = pytest.mark.gpu

TOL = 1.0e-4


def rel(a, b):
    return float(np.linalg.norm(np.asarray(a, np.float64) - np.asarray(b, np.float64)) /
                 max(np.linalg.norm(np.asarray(b, np.float64)), 1e-300))


def data(rng, N, D, decay=0.97, mean=0.3):
    scales = decay ** np.arange(D) + 0.02
    x = rng.standard_normal((N, D)) * scales[None, :] + mean * np.sin(np.arange(D))[None, :]
    return x[:, rng.permutation(D)].astype(np.float32)


def gpu_call(torch, pre, M, ld):
    N, D = M.shape
    buf = torch.full((N, ld), 777.0, dtype=torch.float32, device="cuda")   # padding holds garbage on purpose
    buf[:, :D] = torch.from_numpy(M).cuda()
    gamma = torch.zeros(1, dtype=torch.float32, device="cuda")
    rn2 = torch.zeros(N, dtype=torch.float32, device="cuda")
    pre.precondition(buf, gamma, rn2)
    torch.cuda.synchronize()
    out = buf.cpu().numpy()
    if ld > D:
        assert np.all(out[:, D:] == 777.0), "columns beyond dim must not be touched"
    return out[:, :D], float(gamma.item()), rn2.cpu().numpy()


SHAPES = [(100, 333, 7), (64, 160, 1), (65, 161, 33), (129, 40, 4), (300, 1000, 96), (37, 50, 20), (200, 3001, 20),
          (256, 640, 80), (90, 2000, 81)]


@pytest.mark.parametrize("wait_us", [2000, 0])
@pytest.mark.parametrize("N,D,R", SHAPES)
def test_calls_without_update_match_oracle(ngsgd, N, D, R, wait_us):
    """Schedule: calls 0, 1 update (always_update_first = 2), 2 and 3 apply only, 4 updates, 5..7 apply only; the
    apply-only calls take the fused kernel.  Rows vary (fewer rows than the first call, a single row)."""
    import torch
    rng = np.random.default_rng(7000 + 13 * N + D + R)
    kw = dict(num_samples_history=600.0, update_period=4, always_update_first=2)
    ora = OnlineNaturalGradient(D, R, **kw)
    pre = ngsgd.Preconditioner(D, R, max_batch=N, **kw)
    ngsgd.set_wait_limit_us(wait_us)
    try:
        for step in range(8):
            n = {3: max(1, N - 9), 6: 1}.get(step, N)
            M = data(rng, n, D)
            print(f"fused apply case N={n} D={D} R={R} step={step} wait_us={wait_us}", flush=True)
            expect, g_o, rn_o = ora.precondition(M)
            got, g_g, rn_g = gpu_call(torch, pre, M, ld=D + (-D) % 4 + (8 if step % 2 else 0))
            assert rel(got, expect) < TOL, f"step {step}"
            assert g_g == pytest.approx(g_o, rel=1e-4)
            assert rel(rn_g, rn_o) < 2e-4
            assert abs(np.linalg.norm(got.astype(np.float64)) / np.linalg.norm(M.astype(np.float64)) - 1.0) < 1e-5
    finally:
        ngsgd.set_wait_limit_us(2000)


@pytest.mark.parametrize("which", ["input", "output"])
def test_c2_full_size_without_update(ngsgd, which):
    """BASELINE configs[2] shapes at full size, apply-only calls between periodic updates."""
    import torch
    spec = workloads.c2_input_side() if which == "input" else workloads.c2_output_side()
    kw = dict(num_samples_history=spec.num_samples_history, update_period=4, always_update_first=3)
    ora = OnlineNaturalGradient(spec.dim, spec.rank, **kw)
    pre = ngsgd.Preconditioner(spec.dim, spec.rank, max_batch=spec.rows, **kw)
    ld = (spec.dim + 3) // 4 * 4
    for step in range(8):
        print(f"fused apply full size {spec.name} step={step}", flush=True)
        M = workloads.spectrum_matrix(spec, step)
        expect, g_o, rn_o = ora.precondition(M)
        got, g_g, rn_g = gpu_call(torch, pre, M, ld)
        assert rel(got, expect) < TOL, f"step {step}"
        assert g_g == pytest.approx(g_o, rel=1e-4)
        assert rel(rn_g, rn_o) < 2e-4

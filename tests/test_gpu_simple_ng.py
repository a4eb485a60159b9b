"""GPU parity: the simple natural-gradient method (App. A) through the C ABI against the float64 oracle.

Bar: 1e-4 relative Frobenius error per preconditioned matrix and per gradient, as for the online method.
Small cases are compared with the definition (one hold-out solve per row); sizes that routine cannot reach
are compared with the oracle's efficient form, which the CPU tests pin to the definition.
"""
import numpy as np
import pytest

import workloads
from oracle.network import NGSGDNetwork
from oracle.simple_ng import simple_ng, simple_ng_definitional

pytestmark = pytest.mark.gpu

TOL = 1.0e-4


def rel(a, b):
    return float(np.linalg.norm(np.asarray(a, np.float64) - np.asarray(b, np.float64)) /
                 max(np.linalg.norm(np.asarray(b, np.float64)), 1e-300))


def data(rng, N, D, decay=0.97, mean=0.3):
    scales = decay ** np.arange(D) + 0.02
    x = rng.standard_normal((N, D)) * scales[None, :] + mean * np.sin(np.arange(D))[None, :]
    return x[:, rng.permutation(D)].astype(np.float32)


def gpu_call(torch, pre, M, ld=None):
    N, D = M.shape
    ld = D + (-D) % 4 if ld is None else ld
    buf = torch.full((N, ld), 777.0, dtype=torch.float32, device="cuda")   # padding holds garbage on purpose
    buf[:, :D] = torch.from_numpy(M).cuda()
    gamma = torch.zeros(1, dtype=torch.float32, device="cuda")
    rn2 = torch.zeros(N, dtype=torch.float32, device="cuda")
    pre.precondition(buf[:, :D], gamma, rn2)                                # a view: row stride ld
    torch.cuda.synchronize()
    out = buf.cpu().numpy()
    if ld > D:
        assert np.all(out[:, D:] == 777.0), "columns beyond dim must not be touched"
    return out[:, :D], float(gamma.item()), rn2.cpu().numpy()


@pytest.mark.parametrize("N,D", [(40, 7), (33, 32), (32, 33), (100, 45), (70, 150), (2, 9), (65, 64)])
def test_small_shapes_match_the_definition(ngsgd, N, D):
    """Column space (N > D) and row space (N <= D), one and several pivot blocks, ragged edges."""
    import torch
    rng = np.random.default_rng(1000 + 37 * N + D)
    M = data(rng, N, D)
    pre = ngsgd.SimplePreconditioner(N, D)
    got, g_g, rn_g = gpu_call(torch, pre, M)
    want, g_o, rn_o = simple_ng_definitional(M.astype(np.float64))
    assert rel(got, want) < TOL
    assert g_g == pytest.approx(g_o, rel=1e-4)
    assert rel(rn_g, rn_o) < 2e-4
    assert abs(np.linalg.norm(got.astype(np.float64)) / np.linalg.norm(M.astype(np.float64)) - 1.0) < 1e-5


@pytest.mark.parametrize("N,D", [(200, 301), (333, 77), (130, 520), (257, 1000)])
def test_medium_shapes_and_reuse(ngsgd, N, D):
    """Several tiles and pivot blocks; the same workspace serves calls with fewer rows and a padded ld."""
    import torch
    rng = np.random.default_rng(2000 + N + D)
    pre = ngsgd.SimplePreconditioner(N, D)
    for rows, ld in ((N, None), (N - 37, D + (-D) % 4 + 8), (N, None)):
        M = data(rng, rows, D)
        got, g_g, rn_g = gpu_call(torch, pre, M, ld)
        want, g_o, rn_o = simple_ng(M.astype(np.float64))
        assert rel(got, want) < TOL, (rows, ld)
        assert g_g == pytest.approx(g_o, rel=1e-4)
        assert rel(rn_g, rn_o) < 2e-4


def test_degenerate_inputs(ngsgd):
    """Zero matrix (gamma = 1, output 0), identical rows (output = input), rows on distinct axes (output = input)."""
    import torch
    pre = ngsgd.SimplePreconditioner(48, 40)
    got, g, rn = gpu_call(torch, pre, np.zeros((48, 40), np.float32))
    assert not got.any() and g == 1.0 and not rn.any()
    x = np.linspace(-1.0, 2.0, 40).astype(np.float32)
    M = np.tile(x, (48, 1))
    got, g, _ = gpu_call(torch, pre, M)
    assert rel(got, M) < TOL
    n2 = float(x.astype(np.float64) @ x.astype(np.float64))
    assert g == pytest.approx(4.0 * n2 / 40 + n2, rel=1e-4)
    M = np.zeros((30, 40), np.float32)
    M[np.arange(30), np.arange(30)] = np.linspace(0.5, 4.0, 30)
    got, _, _ = gpu_call(torch, pre, M)
    assert rel(got, M) < TOL


@pytest.mark.parametrize("which", ["input", "output"])
def test_c2_full_size_shapes(ngsgd, which):
    """The two matrix shapes of BASELINE configs[2] (512 x 3001 with a ones column, 512 x 5000), row space."""
    import torch
    spec = workloads.c2_input_side() if which == "input" else workloads.c2_output_side()
    pre = ngsgd.SimplePreconditioner(spec.rows, spec.dim)
    for step in range(2):
        M = workloads.spectrum_matrix(spec, step)
        got, g_g, rn_g = gpu_call(torch, pre, M)
        want, g_o, rn_o = simple_ng(M.astype(np.float64))
        assert rel(got, want) < TOL, f"step {step}"
        assert g_g == pytest.approx(g_o, rel=1e-4)
        assert rel(rn_g, rn_o) < 2e-4


def make_pair(ngsgd, spec, renorm=False, max_change=0.0):
    import torch
    weights = workloads.initial_weights(spec)
    ora = NGSGDNetwork(spec.dims, spec.nonlin, weights, spec.pnorm_group, spec.rank_in, spec.rank_out, spec.alpha,
                       spec.num_samples_history, spec.epsilon, spec.update_period, renorm=renorm,
                       max_change_per_sample=max_change, method="simple")
    gpu = ngsgd.Network(spec.dims, spec.nonlin, spec.minibatch, spec.pnorm_group, spec.rank_in, spec.rank_out,
                        spec.alpha, spec.num_samples_history, spec.epsilon, spec.update_period, renorm=renorm,
                        max_change_per_sample=max_change, method="simple")
    for l, w in enumerate(weights):
        gpu.set_params(l, torch.from_numpy(np.ascontiguousarray(w, dtype=np.float32)).cuda())
    return ora, gpu


def run_and_compare(ngsgd, spec, ora, gpu, steps, rows=None):
    import torch
    for t in range(steps):
        x, y = workloads.minibatch(spec, t, rows=rows)
        obj_o = ora.step(x, y, spec.lr)
        out = gpu.step(torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda(), spec.lr)
        torch.cuda.synchronize()
        n = len(y)
        assert abs(float(out.item()) - obj_o) / n < 1e-3, f"step {t}"
        for l in range(spec.n_layers):
            xo = gpu.last_preconditioned(l, ngsgd.NGSGD_SIDE_INPUT, n).cpu().numpy()
            oo = gpu.last_preconditioned(l, ngsgd.NGSGD_SIDE_OUTPUT, n).cpu().numpy()
            grad = gpu.last_gradient(l).cpu().numpy()
            e_x, e_o = rel(xo, ora.last["Xbar"][l]), rel(oo, ora.last["Obar"][l])
            assert e_x < TOL and e_o < TOL, f"step {t} layer {l}: Xbar {e_x:.2e} Obar {e_o:.2e}"
            assert rel(grad, ora.last["delta"][l]) < TOL, f"step {t} layer {l}: gradient"
            if ora.max_change_per_sample > 0.0:
                mc = float(gpu.last_max_change_scale(l).item())
                assert mc == pytest.approx(ora.last["max_change_scale"][l], rel=1e-4)
        # the update itself, then both sides continue from the oracle's weights (one step's accuracy at a time)
        for l in range(spec.n_layers):
            assert rel(gpu.get_params(l).cpu().numpy(), ora.W[l]) < TOL
            gpu.set_params(l, torch.from_numpy(np.ascontiguousarray(ora.W[l], dtype=np.float32)).cuda())


def test_network_steps_small_nets(ngsgd):
    """C0 (tanh) free of stabilisers, and the reduced p-norm net with renormalisation and max-change."""
    spec = workloads.c0_tiny()
    ora, gpu = make_pair(ngsgd, spec)
    run_and_compare(ngsgd, spec, ora, gpu, 4)
    assert gpu.precond(0, ngsgd.NGSGD_SIDE_INPUT) is None            # no online factors are kept
    spec = workloads.small_pnorm()
    ora, gpu = make_pair(ngsgd, spec, renorm=True, max_change=0.075)
    run_and_compare(ngsgd, spec, ora, gpu, 3)
    run_and_compare(ngsgd, spec, ora, gpu, 1, rows=spec.minibatch - 9)


def test_c1_full_size_step(ngsgd):
    """BASELINE configs[1] at full size with the simple method, in the configuration bench.py times."""
    spec = workloads.c1_pnorm()
    ora, gpu = make_pair(ngsgd, spec, renorm=True, max_change=0.075)
    run_and_compare(ngsgd, spec, ora, gpu, 2)

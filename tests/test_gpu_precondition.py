"""GPU parity: ngsgd_precondition (through the C ABI) against the float64 oracle, same seeded inputs.

Bar: 1e-4 relative Frobenius error per preconditioned matrix.  The factor itself is not unique (sign and
rotation of eigenvectors), so states are compared through what is unique: rho, the sorted diagonal D, and the
action X -> X - X W^T W on a probe.
"""
import math

import numpy as np
import pytest

import workloads
from oracle.online_ng import OnlineNaturalGradient, smoothing_and_scales

pytestmark = pytest.mark.gpu

TOL = 1.0e-4


def rel(a, b):
    return float(np.linalg.norm(np.asarray(a, np.float64) - np.asarray(b, np.float64)) /
                 max(np.linalg.norm(np.asarray(b, np.float64)), 1e-300))


def data(rng, N, D, decay=0.97, mean=0.3):
    scales = decay ** np.arange(D) + 0.02
    x = rng.standard_normal((N, D)) * scales[None, :] + mean * np.sin(np.arange(D))[None, :]
    mix = rng.permutation(D)
    return x[:, mix].astype(np.float32)


def gpu_call(torch, pre, M, ld=None):
    N, D = M.shape
    ld = D + (-D) % 4 if ld is None else ld
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


def probe_action_oracle(ora, P):
    _, e = smoothing_and_scales(ora.d, ora.rho, ora.alpha, ora.dim)
    return P - ((P @ ora.R.T) * e[None, :]) @ ora.R


def compare_states(torch, pre, ora, rng):
    W, d, rho, t = pre.get_state()
    W = W.cpu().numpy().astype(np.float64)
    d = d.cpu().numpy()
    assert t == ora.t
    assert rho == pytest.approx(ora.rho, rel=2e-4)
    live = ora.d > 1e-6 * ora.d.max()
    np.testing.assert_allclose(np.sort(d)[::-1][live], np.sort(ora.d)[::-1][live], rtol=5e-4)
    P = rng.standard_normal((16, ora.dim))
    assert rel(P - (P @ W.T) @ W, probe_action_oracle(ora, P)) < TOL


def upload_state(torch, pre, ora):
    pre.set_state(torch.from_numpy(np.ascontiguousarray(ora.R)).cuda(), torch.from_numpy(ora.d.copy()).cuda(),
                  ora.rho, ora.t)


@pytest.mark.parametrize("N,D,R,period", [(200, 301, 20, 1), (96, 1000, 80, 1), (333, 77, 5, 2), (130, 520, 90, 1),
                                           (64, 41, 4, 1), (150, 400, 96, 1), (120, 333, 95, 1), (40, 9, 1, 1)])
def test_from_shared_state_matches_oracle(ngsgd, N, D, R, period):
    """Oracle warms up, its state is uploaded, then both process the same matrices (apply and update paths)."""
    import torch
    rng = np.random.default_rng(1000 + D)
    kw = dict(num_samples_history=500.0, update_period=period, always_update_first=2)
    ora = OnlineNaturalGradient(D, R, **kw)
    for _ in range(3):
        ora.precondition(data(rng, N, D))
    pre = ngsgd.Preconditioner(D, R, max_batch=N + 7, **kw)
    upload_state(torch, pre, ora)
    compare_states(torch, pre, ora, rng)
    for step in range(6):
        n = N if step != 3 else N - 5                       # a smaller minibatch in the middle (App. B.5)
        M = data(rng, n, D)
        expect, g_o, rn_o = ora.precondition(M)
        got, g_g, rn_g = gpu_call(torch, pre, M, ld=D + (-D) % 4 + (8 if step % 2 else 0))
        assert rel(got, expect) < TOL, f"step {step}"
        assert g_g == pytest.approx(g_o, rel=1e-4)
        assert rel(rn_g, rn_o) < 2e-4
        assert abs(np.linalg.norm(got.astype(np.float64)) / np.linalg.norm(M.astype(np.float64)) - 1.0) < 1e-5
    compare_states(torch, pre, ora, rng)


@pytest.mark.parametrize("N,D,R", [(128, 301, 20), (96, 700, 40), (257, 64, 8), (80, 80, 12)])
def test_free_running_from_device_initialisation(ngsgd, N, D, R):
    """Both sides build their state from the first minibatch (App. B.3.2) and then run the paper's schedule."""
    import torch
    rng = np.random.default_rng(2000 + D)
    kw = dict(num_samples_history=800.0, update_period=4, always_update_first=10)
    ora = OnlineNaturalGradient(D, R, **kw)
    pre = ngsgd.Preconditioner(D, R, max_batch=N, **kw)
    for step in range(14):
        M = data(rng, N, D)
        expect, g_o, _ = ora.precondition(M)
        got, g_g, _ = gpu_call(torch, pre, M)
        assert rel(got, expect) < TOL, f"step {step}"
        assert g_g == pytest.approx(g_o, rel=1e-4)
        if step in (0, 9, 13):
            compare_states(torch, pre, ora, rng)


def test_degenerate_first_minibatches(ngsgd):
    """Zero and rank-deficient first inputs: floors, gamma = 1 on a zero matrix, completion of R_0."""
    import torch
    rng = np.random.default_rng(3)
    N, D, R = 64, 100, 6
    kw = dict(num_samples_history=300.0, update_period=1)
    # (a) zeros first, then data
    ora = OnlineNaturalGradient(D, R, **kw)
    pre = ngsgd.Preconditioner(D, R, max_batch=N, **kw)
    seq = [np.zeros((N, D), np.float32), np.zeros((N, D), np.float32)] + [data(rng, N, D) for _ in range(4)]
    for step, M in enumerate(seq):
        expect, g_o, _ = ora.precondition(M)
        got, g_g, _ = gpu_call(torch, pre, M)
        if not M.any():
            assert g_g == 1.0 and not got.any()
        else:
            assert rel(got, expect) < TOL, f"step {step}"
    compare_states(torch, pre, ora, rng)
    # (b) first minibatch of rank 2 (< R), for both eigen routes
    for n_rows, dim in [(64, 100), (120, 40)]:
        ora = OnlineNaturalGradient(dim, R, **kw)
        pre = ngsgd.Preconditioner(dim, R, max_batch=n_rows, **kw)
        basis = rng.standard_normal((2, dim))
        first = (rng.standard_normal((n_rows, 2)) @ basis).astype(np.float32)
        for step, M in enumerate([first] + [data(rng, n_rows, dim) for _ in range(4)]):
            expect, _, _ = ora.precondition(M)
            got, _, _ = gpu_call(torch, pre, M)
            assert rel(got, expect) < TOL, f"route {dim} step {step}"


@pytest.mark.parametrize("N,D,R,spread", [(96, 200, 6, 1e5), (96, 200, 6, None), (96, 200, 13, None),
                                          (128, 300, 40, None), (160, 400, 80, None), (200, 500, 96, None)])
def test_forced_reorthogonalisation(ngsgd, N, D, R, spread):
    """A skewed factor with an ill-conditioned D_t makes cond(C_t) exceed 1e6, which triggers the check of
    App. B.3.1, and the check then finds R R^T off the identity.

    With R R^T != I the efficient form of App. B.3 (which the GPU implements) is no longer the same map as the
    definitional form, so the reference here is the oracle's efficient-form routine, which follows the paper's
    W-space formulas including the Cholesky fix.
    """
    import torch
    from oracle.online_ng_efficient import OnlineNaturalGradientEfficient
    rng = np.random.default_rng(4)   # (one rank per instantiation of the correction kernel)
    kw = dict(num_samples_history=300.0, update_period=1)
    warm = OnlineNaturalGradient(D, R, **kw)
    for _ in range(3):
        warm.precondition(data(rng, N, D))
    R_bad = warm.R.copy()
    R_bad[1] *= 0.5
    R_bad[2] += 0.3 * R_bad[0]
    d_bad = warm.d.copy()
    rho_bad = warm.rho
    # cond(C_t) ~ ((d_0 + rho) / (d_min + rho))^2 just past the 1e6 of App. B.3.1; at rank 6 also a d_0 a hundred
    # thousand times larger (at higher ranks that mostly tests how float32 factors carry the spread through the
    # trace identities: rho then differs in the second digit)
    d_bad[0] = d_bad[0] * spread if spread else 3.0e3 * (d_bad.min() + rho_bad)
    eff = OnlineNaturalGradientEfficient(D, R, **kw)
    _, e = smoothing_and_scales(d_bad, rho_bad, 4.0, D)
    eff.W, eff.d, eff.rho, eff.t = np.sqrt(e)[:, None] * R_bad, d_bad.copy(), rho_bad, warm.t
    pre = ngsgd.Preconditioner(D, R, max_batch=N, **kw)
    pre.set_state(torch.from_numpy(R_bad).cuda(), torch.from_numpy(d_bad.copy()).cuda(), rho_bad, warm.t)
    M = data(rng, N, D)
    expect, _, _ = eff.precondition(M)
    got, _, _ = gpu_call(torch, pre, M)
    assert eff.last["reorthogonalised"]
    assert rel(got, expect) < TOL
    W, d, rho, _ = pre.get_state()
    W = W.cpu().numpy().astype(np.float64)
    _, e = smoothing_and_scales(d.cpu().numpy(), rho, 4.0, D)
    Rg = W / np.sqrt(e)[:, None]
    np.testing.assert_allclose(Rg @ Rg.T, np.eye(R), atol=1e-5)      # orthonormal again
    assert rho == pytest.approx(eff.rho, rel=2e-4)
    P = rng.standard_normal((16, D))
    assert rel(P - (P @ W.T) @ W, P - (P @ eff.W.T) @ eff.W) < TOL
    for _ in range(3):
        M = data(rng, N, D)
        expect, _, _ = eff.precondition(M)
        got, _, _ = gpu_call(torch, pre, M)
        assert rel(got, expect) < TOL


def test_rank_zero_and_argument_errors(ngsgd):
    import torch
    rng = np.random.default_rng(5)
    M = data(rng, 50, 36)
    pre0 = ngsgd.Preconditioner(36, 0, max_batch=64)
    got, g, rn = gpu_call(torch, pre0, M)
    np.testing.assert_array_equal(got, M)
    assert g == 1.0
    np.testing.assert_allclose(rn, np.sum(M.astype(np.float64) ** 2, axis=1), rtol=1e-5)
    pre = ngsgd.Preconditioner(36, 8, max_batch=64)
    buf = torch.zeros((70, 36), dtype=torch.float32, device="cuda")
    with pytest.raises(ngsgd.NgsgdError) as err:
        pre.precondition(buf)                                  # N > max_batch
    assert err.value.code == ngsgd.NGSGD_EINVAL
    with pytest.raises(ngsgd.NgsgdError):
        pre.precondition(buf[:8])                              # first call needs N > rank
    with pytest.raises(ngsgd.NgsgdError):
        pre.precondition(torch.zeros((20, 38), dtype=torch.float32, device="cuda")[:, :36])   # ld not a multiple of 4
    with pytest.raises(ngsgd.NgsgdError):
        ngsgd.Preconditioner(36, 36, max_batch=64)             # rank >= dim
    assert pre.get_state()[3] == 0                             # failed calls did not advance the state


@pytest.mark.parametrize("which", ["input", "output"])
def test_c2_full_size_shapes(ngsgd, which):
    """BASELINE's preconditioner microbenchmark shapes (512x3001 rank 20, 512x5000 rank 80), successive updates,
    in the configuration bench.py times (update on every call)."""
    import torch
    spec = workloads.c2_input_side() if which == "input" else workloads.c2_output_side()
    kw = dict(num_samples_history=spec.num_samples_history, update_period=spec.update_period)
    ora = OnlineNaturalGradient(spec.dim, spec.rank, **kw)
    pre = ngsgd.Preconditioner(spec.dim, spec.rank, max_batch=spec.rows, **kw)
    rng = np.random.default_rng(6)
    for step in range(12):
        M = workloads.spectrum_matrix(spec, step)
        expect, g_o, rn_o = ora.precondition(M)
        got, g_g, rn_g = gpu_call(torch, pre, M)
        assert rel(got, expect) < TOL, f"step {step}"
        assert g_g == pytest.approx(g_o, rel=1e-4)
        assert rel(rn_g, rn_o) < 2e-4
        # the device-side eigen-solver reports what it did: it must have converged within its sweep budget
        flags, sweeps = pre.diagnostics()
        assert flags & 8 == 0, f"step {step}: the Jacobi iteration did not converge (flags {flags})"
        assert 1 <= sweeps <= 20
    compare_states(torch, pre, ora, rng)


@pytest.mark.parametrize("which", ["input", "output"])
def test_c2_thousand_successive_updates(ngsgd, which):
    """BASELINE configs[2] as stated: 1000 successive online updates at full size, free running on both sides
    (each builds its state from the first matrix and then follows its own recursion), the factor updated on every
    call.  A pool of 16 matrices is cycled, as in bench.py.  Every 50th call the preconditioned matrix, gamma, rho,
    the sorted D and the action of the factor on a probe are compared; the first mismatch stops the test."""
    import torch
    spec = workloads.c2_input_side() if which == "input" else workloads.c2_output_side()
    kw = dict(num_samples_history=spec.num_samples_history, update_period=spec.update_period)
    ora = OnlineNaturalGradient(spec.dim, spec.rank, **kw)
    pre = ngsgd.Preconditioner(spec.dim, spec.rank, max_batch=spec.rows, **kw)
    pool = [workloads.spectrum_matrix(spec, t) for t in range(16)]
    ld = (spec.dim + 3) // 4 * 4
    dev_pool = []
    for M in pool:
        buf = torch.zeros((spec.rows, ld), dtype=torch.float32, device="cuda")
        buf[:, :spec.dim] = torch.from_numpy(M).cuda()
        dev_pool.append(buf)
    work = torch.empty_like(dev_pool[0])
    gamma = torch.zeros(1, dtype=torch.float32, device="cuda")
    rng = np.random.default_rng(8)
    worst = 0.0
    for step in range(spec.steps):
        expect, g_o, _ = ora.precondition(pool[step % 16])
        work.copy_(dev_pool[step % 16])
        pre.precondition(work, gamma)
        if step % 50 == 49 or step == spec.steps - 1:
            print(f"c2 long run {spec.name} call {step}", flush=True)
            torch.cuda.synchronize()
            err = rel(work[:, :spec.dim].cpu().numpy(), expect)
            worst = max(worst, err)
            assert err < TOL, f"call {step}"
            assert float(gamma.item()) == pytest.approx(g_o, rel=1e-4)
            compare_states(torch, pre, ora, rng)
            flags, sweeps = pre.diagnostics()
            assert flags & 8 == 0 and 1 <= sweeps <= 20, f"call {step}: flags {flags}, sweeps {sweeps}"
    assert ora.t == spec.steps == 1000
    print(f"c2 long run {spec.name}: worst relative error of the preconditioned matrix {worst:.2e}")


def test_eigenvalues_under_the_floor(ngsgd):
    """The eigenvalues of Z_t cannot fall below (1 - eta)^2 rho_t^2 for a factor with orthonormal rows (App. B.3), so
    with consistent state the floor only catches rounding.  It fires for real when the stored factor has lost its
    orthogonality: eq. zt:compute then no longer describes a Gram matrix and Z_t can even be indefinite.  A mixed
    (non-orthonormal) factor is installed for which the oracle's W-space routine reports a floored eigenvalue, and
    the device must then raise its floor flag (bit 1), run the orthogonality check the floor asks for, repair the
    factor (bit 2) and agree with that routine on the output, on the state and on the calls that follow.  (As in
    the forced re-orthogonalisation test, the reference is the efficient form: with R R^T != I the definitional
    form is a different map.)"""
    import torch
    from oracle.online_ng_efficient import OnlineNaturalGradientEfficient
    rng = np.random.default_rng(4)
    N, D, R = 96, 200, 6
    kw = dict(num_samples_history=300.0, update_period=1)
    warm = OnlineNaturalGradient(D, R, **kw)
    for _ in range(3):
        warm.precondition(data(rng, N, D))
    M = data(rng, N, D)
    eta = 1.0 - math.exp(-N / 300.0)
    search = np.random.default_rng(40)
    chosen = None
    for _ in range(400):        # seeded search on the CPU for a mildly indefinite case
        R_bad = (np.eye(R) + 1.5 * search.standard_normal((R, R))) @ warm.R
        d_bad = warm.d * np.exp(search.uniform(-3.0, 3.0, R))
        rho_bad = warm.rho * math.exp(search.uniform(-1.0, 2.0))
        eff = OnlineNaturalGradientEfficient(D, R, **kw)
        _, e = smoothing_and_scales(d_bad, rho_bad, 4.0, D)
        eff.W, eff.d, eff.rho, eff.t = np.sqrt(e)[:, None] * R_bad, d_bad.copy(), rho_bad, warm.t
        expect, _, _ = eff.precondition(M)
        if eff.last["floored"] and eff.last["reorthogonalised"]:
            chosen = (R_bad, d_bad, rho_bad, eff, expect)
            break
    assert chosen is not None, "the search found no floored case"
    R_bad, d_bad, rho_bad, eff, expect = chosen
    pre = ngsgd.Preconditioner(D, R, max_batch=N, **kw)
    pre.set_state(torch.from_numpy(R_bad.copy()).cuda(), torch.from_numpy(d_bad.copy()).cuda(), rho_bad, warm.t)
    got, _, _ = gpu_call(torch, pre, M)
    flags, sweeps = pre.diagnostics()
    assert flags & 2, "the device did not floor an eigenvalue of Z_t"
    assert flags & 4 and not flags & 1, "the floor must trigger the orthogonality check, which repairs this factor"
    assert flags & 8 == 0 and 1 <= sweeps <= 20
    assert rel(got, expect) < TOL
    W, d, rho, _ = pre.get_state()
    W = W.cpu().numpy().astype(np.float64)
    assert rho == pytest.approx(eff.rho, rel=2e-4)
    live = np.sort(eff.d)[::-1] > 1e-6 * eff.d.max()      # (a floored eigenvalue leaves d_i at epsilon)
    np.testing.assert_allclose(np.sort(d.cpu().numpy())[::-1][live], np.sort(eff.d)[::-1][live], rtol=5e-4)
    P = rng.standard_normal((16, D))
    assert rel(P - (P @ W.T) @ W, P - (P @ eff.W.T) @ eff.W) < TOL
    for _ in range(3):
        M = data(rng, N, D)
        expect, _, _ = eff.precondition(M)
        got, _, _ = gpu_call(torch, pre, M)
        assert rel(got, expect) < TOL

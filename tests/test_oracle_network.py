"""Pins for the float64 oracle of the network step and of parameter averaging."""
import math

import numpy as np
import pytest

import workloads
from oracle.averaging import average_parameters, job_learning_rate
from oracle.network import (PNORM, TANH, NGSGDNetwork, log_softmax, pnorm_backward,
                            pnorm_forward)


def tiny_net(rng, nonlin, ng=True, rank_in=2, rank_out=3, zero_softmax=False):
    group = 3
    dims = [5, 12, 9, 7]
    in_dims = [5, 12 // group if nonlin[0] == PNORM else 12, 9 // group if nonlin[1] == PNORM else 9]
    weights = [rng.standard_normal((dims[l + 1], in_dims[l] + 1)) / math.sqrt(in_dims[l]) for l in range(3)]
    if zero_softmax:
        weights[-1][:] = 0.0
    return NGSGDNetwork(dims, nonlin, weights, pnorm_group=group, rank_in=rank_in, rank_out=rank_out,
                        num_samples_history=40.0, update_period=1, natural_gradient=ng)


@pytest.mark.parametrize("nonlin", [[TANH, TANH], [PNORM, PNORM], [PNORM, TANH]])
def test_gradients_match_central_differences(nonlin):
    """P11: backward pass against finite differences of sum_i log p(y_i | x_i)."""
    rng = np.random.default_rng(21)
    net = tiny_net(rng, nonlin)
    x = rng.standard_normal((6, 5))
    y = rng.integers(0, 7, 6)
    grads = net.gradients(x, y)
    h = 1e-6
    for l in range(net.n_layers):
        num = np.zeros_like(net.W[l])
        for idx in np.ndindex(*net.W[l].shape):
            old = net.W[l][idx]
            net.W[l][idx] = old + h
            fp = net.objective(x, y)
            net.W[l][idx] = old - h
            fm = net.objective(x, y)
            net.W[l][idx] = old
            num[idx] = (fp - fm) / (2 * h)
        np.testing.assert_allclose(grads[l], num, atol=2e-7 * max(1.0, np.abs(num).max()))


def test_softmax_and_derivative_properties():
    rng = np.random.default_rng(22)
    A = 30.0 * rng.standard_normal((9, 11))
    lp = log_softmax(A)
    np.testing.assert_allclose(np.exp(lp).sum(axis=1), 1.0, rtol=1e-13)
    net = tiny_net(rng, [TANH, TANH])
    x = rng.standard_normal((8, 5))
    y = rng.integers(0, 7, 8)
    Xin, Aff, logp = net.forward(x)
    O = net.backward(Xin, Aff, logp, y)
    np.testing.assert_allclose(O[-1].sum(axis=1), 0.0, atol=1e-14)   # onehot - softmax
    assert all(np.all(X[:, -1] == 1.0) for X in Xin)                 # appended ones column
    # zero softmax weights: every class has probability 1 / #classes (App. C.7 initialisation)
    net0 = tiny_net(rng, [PNORM, PNORM], zero_softmax=True)
    assert net0.objective(x, y) == pytest.approx(-8 * math.log(7), rel=1e-14)


def test_pnorm_definition_and_zero_group():
    A = np.array([[3.0, 4.0, 0.0, 0.0, 0.0, 0.0, 1.0, 2.0, 2.0]])
    Y = pnorm_forward(A, 3)
    np.testing.assert_allclose(Y, [[5.0, 0.0, 3.0]])
    dA = pnorm_backward(np.array([[1.0, 7.0, -2.0]]), A, Y, 3)
    np.testing.assert_allclose(dA, [[0.6, 0.8, 0.0, 0.0, 0.0, 0.0, -2 / 3, -4 / 3, -4 / 3]])


def test_rank_zero_step_is_plain_sgd():
    """P4 at network level: with R = 0 on both sides NG-SGD equals SGD with summed gradients."""
    rng = np.random.default_rng(23)
    a = tiny_net(np.random.default_rng(5), [TANH, PNORM], ng=True, rank_in=0, rank_out=0)
    b = tiny_net(np.random.default_rng(5), [TANH, PNORM], ng=False)
    for _ in range(3):
        x = rng.standard_normal((10, 5))
        y = rng.integers(0, 7, 10)
        g = b.gradients(x, y)
        Wb = [w.copy() for w in b.W]
        oa = a.step(x, y, 0.01)
        ob = b.step(x, y, 0.01)
        assert oa == pytest.approx(ob, rel=1e-14)
        for l in range(3):
            np.testing.assert_allclose(b.W[l], Wb[l] + 0.01 * g[l], atol=1e-14)   # summed, not averaged
            np.testing.assert_allclose(a.W[l], b.W[l], atol=1e-13)


def test_step_update_is_product_of_preconditioned_factors():
    """W += lr Obar^T Xbar with each factor rescaled to the norm of its input (Sec. 4.6, 4.7)."""
    rng = np.random.default_rng(24)
    net = tiny_net(rng, [PNORM, TANH])
    from oracle.online_ng import OnlineNaturalGradient
    kw = dict(num_samples_history=40.0, update_period=1)
    shadow_in = [OnlineNaturalGradient(net.in_dims[l] + 1, 2, **kw) for l in range(3)]
    shadow_out = [OnlineNaturalGradient(net.dims[l + 1], 3, **kw) for l in range(3)]
    for _ in range(4):
        x = rng.standard_normal((12, 5))
        y = rng.integers(0, 7, 12)
        W0 = [w.copy() for w in net.W]
        obj_before = net.objective(x, y)
        obj = net.step(x, y, 0.02)
        assert obj == pytest.approx(obj_before, rel=1e-14)              # objective is taken before the update
        for l in range(3):
            Ob = shadow_out[l].precondition(net.last["O"][l])[0]      # each matrix has its own instance
            Xb = shadow_in[l].precondition(net.last["Xin"][l])[0]
            np.testing.assert_allclose(net.W[l], W0[l] + 0.02 * Ob.T @ Xb, atol=1e-14)
            assert np.linalg.norm(Ob) == pytest.approx(np.linalg.norm(net.last["O"][l]), rel=1e-12)
            assert np.linalg.norm(Xb) == pytest.approx(np.linalg.norm(net.last["Xin"][l]), rel=1e-12)
    assert all(p.t == 4 for p in net.precond_in + net.precond_out)


def test_simple_method_step():
    """method="simple" (App. A): the update is built from the definitional hold-one-out factors of the same
    minibatch, keeps no state, and tends to the plain SGD step under heavy smoothing."""
    from oracle.simple_ng import simple_ng_definitional
    rng = np.random.default_rng(31)
    dims, group = [5, 12, 9, 7], 3
    weights = [rng.standard_normal((12, 6)) / 2, rng.standard_normal((9, 5)) / 2, rng.standard_normal((7, 10)) / 3]
    mk = lambda **kw: NGSGDNetwork(dims, [PNORM, TANH], [w.copy() for w in weights], pnorm_group=group, rank_in=2, rank_out=3, **kw)
    net = mk(method="simple")
    x = rng.standard_normal((14, 5))
    y = rng.integers(0, 7, 14)
    W0 = [w.copy() for w in net.W]
    net.step(x, y, 0.02)
    for l in range(3):
        Ob = simple_ng_definitional(net.last["O"][l])[0]
        Xb = simple_ng_definitional(net.last["Xin"][l])[0]
        np.testing.assert_allclose(net.W[l], W0[l] + 0.02 * Ob.T @ Xb, atol=1e-12)
    assert all(p.t == 0 for p in net.precond_in + net.precond_out)       # the online state is not touched
    heavy, plain = mk(method="simple", alpha=1e10), mk(natural_gradient=False)
    heavy.step(x, y, 0.02)
    plain.step(x, y, 0.02)
    for l in range(3):
        np.testing.assert_allclose(heavy.W[l], plain.W[l], atol=1e-7)


def test_small_learning_rate_step_increases_objective():
    rng = np.random.default_rng(25)
    net = tiny_net(rng, [TANH, TANH])
    x = rng.standard_normal((16, 5))
    y = rng.integers(0, 7, 16)
    before = net.objective(x, y)
    net.step(x, y, 1e-3)
    assert net.objective(x, y) > before


def test_parameter_averaging():
    """P12: mean of identical replicas is the replica; the mean is linear; state is rebuilt afterwards."""
    rng = np.random.default_rng(26)
    nets = [tiny_net(np.random.default_rng(9), [TANH, TANH]) for _ in range(3)]
    ref = [w.copy() for w in nets[0].W]
    average_parameters(nets)
    for net in nets:
        for l in range(3):
            np.testing.assert_allclose(net.W[l], ref[l], rtol=0, atol=4e-16)   # (3w)/3 rounds once
    for k, net in enumerate(nets):
        for l in range(3):
            net.W[l] = ref[l] + (k + 1.0)
        net.step(rng.standard_normal((8, 5)), rng.integers(0, 7, 8), 0.0)
        assert net.precond_in[0].t == 1
    snapshot = [[w.copy() for w in net.W] for net in nets]
    average_parameters(nets)
    for net in nets:
        for l in range(3):
            np.testing.assert_allclose(net.W[l], sum(s[l] for s in snapshot) / 3.0, atol=1e-15)
            np.testing.assert_allclose(net.W[l], ref[l] + 2.0, atol=1e-13)
        assert all(p.t == 0 and p.R is None for p in net.precond_in + net.precond_out)


def test_job_learning_rate_keeps_the_effective_rate():
    """Sec. 3.1: with the jobs' rate n times the effective rate, one averaged SGD step of n jobs from common weights
    equals one step at the effective rate on the sum of the jobs' gradients (checked on plain SGD, rank 0)."""
    n_jobs, eff = 3, 0.004
    lr = job_learning_rate(eff, n_jobs)
    assert lr == pytest.approx(0.012)
    with pytest.raises(ValueError):
        job_learning_rate(eff, 0)
    rng = np.random.default_rng(31)
    nets = [tiny_net(np.random.default_rng(9), [TANH, PNORM], ng=False) for _ in range(n_jobs)]
    start = [w.copy() for w in nets[0].W]
    total = [np.zeros_like(w) for w in start]
    for net in nets:
        x, y = rng.standard_normal((8, 5)), rng.integers(0, 7, 8)
        for l, g in enumerate(net.gradients(x, y)):
            total[l] += g
        net.step(x, y, lr)
    average_parameters(nets, reset_preconditioners=False)
    for l in range(3):
        np.testing.assert_allclose(nets[0].W[l], start[l] + eff * total[l], atol=1e-14)


def test_workload_generators_are_seeded_and_shaped():
    spec = workloads.c1_pnorm()
    assert spec.in_dims == [360, 300, 300, 300, 300] and spec.n_params() == 5_297_000
    assert workloads.c3_wide_tanh().n_params() == 38_276_928
    spec0 = workloads.c0_tiny()
    x1, y1 = workloads.minibatch(spec0, 3)
    x2, y2 = workloads.minibatch(spec0, 3)
    np.testing.assert_array_equal(x1, x2)
    np.testing.assert_array_equal(y1, y2)
    assert x1.shape == (64, 40) and x1.dtype == np.float32 and y1.dtype == np.int32 and y1.max() < 50
    w = workloads.initial_weights(spec)
    assert [a.shape for a in w] == [(3000, 361), (3000, 301), (3000, 301), (3000, 301), (5000, 301)]
    assert not w[-1].any() and np.all(w[0][:, -1] == 0)
    assert np.std(w[1][:, :-1]) == pytest.approx(1 / math.sqrt(300), rel=0.02)
    ps = workloads.c2_input_side()
    m = workloads.spectrum_matrix(ps, 0, rows=64)
    assert m.shape == (64, 3001) and np.all(m[:, -1] == 1.0)
    po = workloads.c2_output_side()
    m = workloads.spectrum_matrix(po, 1, rows=2048).astype(np.float64)
    sv = np.linalg.svd(m, compute_uv=False)
    # singular values follow ~ 1/k: the leading ratio s1/s8 is near 8
    assert 5.0 < sv[0] / sv[7] < 12.0


# ---- renormalisation layer (App. C.8, footnote) and maximum parameter change (App. C.3) ---------------------------
from oracle.network import RENORM_FLOOR, renorm_backward, renorm_forward


def renorm_net(rng, nonlin=(PNORM, PNORM), **kw):
    group = 3
    dims = [5, 12, 9, 7]
    in_dims = [5, 12 // group if nonlin[0] == PNORM else 12, 9 // group if nonlin[1] == PNORM else 9]
    weights = [rng.standard_normal((dims[l + 1], in_dims[l] + 1)) / math.sqrt(in_dims[l]) for l in range(3)]
    return NGSGDNetwork(dims, list(nonlin), weights, pnorm_group=group, rank_in=2, rank_out=3,
                        num_samples_history=40.0, update_period=1, **kw)


def test_renorm_forward_hand_example_unit_rms_and_scale_invariance():
    """Rows leave with unit rms, whatever their scale; a zero row stays zero (its divisor is the floor)."""
    Y = np.array([[3.0, 4.0], [0.0, 0.0], [1.0e-3, 0.0]])
    Yn, sigma = renorm_forward(Y)
    # row 0: rms = sqrt((9 + 16) / 2) = 5 / sqrt(2); row 2: rms = 1e-3 / sqrt(2)
    np.testing.assert_allclose(sigma, [5.0 / math.sqrt(2.0), RENORM_FLOOR, 1.0e-3 / math.sqrt(2.0)], rtol=1e-15)
    np.testing.assert_allclose(Yn, [[0.6 * math.sqrt(2.0), 0.8 * math.sqrt(2.0)], [0.0, 0.0], [math.sqrt(2.0), 0.0]],
                               rtol=1e-15)
    rng = np.random.default_rng(41)
    Y = np.abs(rng.standard_normal((7, 11))) * np.exp(rng.uniform(-20, 20, (7, 1)))   # rows on very different scales
    Yn, sigma = renorm_forward(Y)
    np.testing.assert_allclose(np.sqrt(np.mean(Yn * Yn, axis=1)), 1.0, rtol=1e-14)
    np.testing.assert_allclose(Yn * sigma[:, None], Y, rtol=1e-14)
    np.testing.assert_allclose(renorm_forward(37.5 * Y)[0], Yn, rtol=1e-14)


def test_renorm_backward_matches_central_differences():
    """d/dY of sum(C * renorm(Y)) against finite differences, row by row."""
    rng = np.random.default_rng(42)
    Y = np.abs(rng.standard_normal((4, 6))) + 0.1
    C = rng.standard_normal((4, 6))
    Yn, sigma = renorm_forward(Y)
    ana = renorm_backward(C, Yn, sigma)
    num = np.zeros_like(Y)
    h = 1e-6
    for idx in np.ndindex(*Y.shape):
        Yp, Ym = Y.copy(), Y.copy()
        Yp[idx] += h
        Ym[idx] -= h
        num[idx] = (np.sum(C * renorm_forward(Yp)[0]) - np.sum(C * renorm_forward(Ym)[0])) / (2 * h)
    np.testing.assert_allclose(ana, num, atol=1e-8)
    # the derivative of a scale-invariant map is orthogonal to its argument
    np.testing.assert_allclose(np.sum(ana * Y, axis=1), 0.0, atol=1e-13)


def test_renorm_net_gradients_match_central_differences_with_a_row_on_the_floor():
    """Backward pass through p-norm + renorm against finite differences of the objective.  Frame 0 is all zero and
    the first layer has no bias, so its p-norm outputs are exactly zero and its divisor sits on the floor: that
    frame's derivative w.r.t. the first affine output is zero (finite), and the objective does not depend on the
    first layer's input weights through it (its bias column is left out: the objective has a kink there)."""
    rng = np.random.default_rng(43)
    net = renorm_net(rng, renorm=True)
    net.W[0][:, -1] = 0.0
    x = rng.standard_normal((6, 5))
    x[0] = 0.0
    y = rng.integers(0, 7, 6)
    Xin, A, logp = net.forward(x)
    assert net._sigma[0][0] == RENORM_FLOOR and np.all(net._sigma[0][1:] > 1e-3)
    O = net.backward(Xin, A, logp, y)
    assert np.all(np.isfinite(O[0])) and not O[0][0].any()
    grads = net.gradients(x, y)
    h = 1e-6
    for l in range(net.n_layers):
        num = np.zeros_like(net.W[l])
        for idx in np.ndindex(*net.W[l].shape):
            if l == 0 and idx[1] == net.W[0].shape[1] - 1:
                num[idx] = grads[l][idx]
                continue
            old = net.W[l][idx]
            net.W[l][idx] = old + h
            fp = net.objective(x, y)
            net.W[l][idx] = old - h
            fm = net.objective(x, y)
            net.W[l][idx] = old
            num[idx] = (fp - fm) / (2 * h)
        np.testing.assert_allclose(grads[l], num, atol=2e-7 * max(1.0, np.abs(num).max()))


def test_renorm_makes_the_output_invariant_to_the_scale_of_pnorm_layers():
    """App. C.8 (footnote): with the renormalisation layers the network output does not change when the
    parameters of a p-norm layer are multiplied by a nonzero constant; without them it does."""
    rng = np.random.default_rng(44)
    x = rng.standard_normal((9, 5))
    for renorm in (True, False):
        net = renorm_net(np.random.default_rng(7), renorm=renorm)
        ref = net.forward(x)[2]
        for l, s in ((0, 3.7), (1, 0.02)):
            net.W[l] *= s
        out = net.forward(x)[2]
        if renorm:
            np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12)
        else:
            assert np.abs(out - ref).max() > 1e-2


def one_layer_net(W, **kw):
    return NGSGDNetwork([W.shape[1] - 1, W.shape[0]], [], [W], rank_in=0, rank_out=0, natural_gradient=False, **kw)


def test_max_change_scale_from_hand_computed_row_norms():
    """App. C.3 on a softmax layer with zero weights: O = onehot - 1/3 has row norm sqrt(6)/3, the inputs
    [3, 4, 1] and [0, 0, 1] have norms sqrt(26) and 1, so with lr = 0.5, N = 2 and 0.075 per sample
    a = 2 * 0.075 / (0.5 * (sqrt(6)/3) * (sqrt(26) + 1))."""
    x = np.array([[3.0, 4.0], [0.0, 0.0]])
    y = np.array([2, 0])
    lr = 0.5
    net = one_layer_net(np.zeros((3, 3)), max_change_per_sample=0.075)
    net.step(x, y, lr)
    a = net.last["max_change_scale"][0]
    expect = 0.15 / (0.5 * (math.sqrt(6.0) / 3.0) * (math.sqrt(26.0) + 1.0))
    assert expect < 1.0 and a == pytest.approx(expect, rel=1e-14)
    O = np.array([[-1 / 3, -1 / 3, 2 / 3], [2 / 3, -1 / 3, -1 / 3]])
    X1 = np.array([[3.0, 4.0, 1.0], [0.0, 0.0, 1.0]])
    np.testing.assert_allclose(net.W[0], lr * expect * O.T @ X1, atol=1e-15)
    # the bound of eq. delta_t_approx: ||a lr O^T X||_F <= a lr sum_i ||o_i|| ||x_i|| = N * 0.075 when active
    assert np.linalg.norm(net.W[0]) <= 2 * 0.075
    assert a * lr * np.sum(np.linalg.norm(O, axis=1) * np.linalg.norm(X1, axis=1)) == pytest.approx(0.15, rel=1e-14)


def test_max_change_scale_is_one_when_inactive_or_degenerate():
    x = np.array([[3.0, 4.0], [0.0, 0.0]])
    y = np.array([2, 0])
    # small learning rate: the bound lr * sum(...) = 1e-3 * 4.98 is under N * 0.075
    net = one_layer_net(np.zeros((3, 3)), max_change_per_sample=0.075)
    net.step(x, y, 1.0e-3)
    assert net.last["max_change_scale"][0] == 1.0
    # a single class: log p = 0 and O = 0, the sum is zero and the scale stays 1
    net = one_layer_net(np.zeros((1, 3)), max_change_per_sample=0.075)
    net.step(x, np.array([0, 0]), 10.0)
    assert net.last["max_change_scale"][0] == 1.0 and not net.W[0].any()
    # disabled
    net = one_layer_net(np.zeros((3, 3)), max_change_per_sample=0.0)
    net.step(x, y, 100.0)
    assert net.last["max_change_scale"][0] == 1.0


def test_max_change_uses_the_preconditioned_rows_and_bounds_the_update():
    """With natural gradient the limit is applied on top of the modified matrices (App. C.3): a_l follows from the
    row norms of Obar_l and Xbar_l, and ||a_l lr Obar_l^T Xbar_l||_F never exceeds N * 0.075."""
    rng = np.random.default_rng(45)
    net = renorm_net(rng, nonlin=(PNORM, TANH), renorm=True, max_change_per_sample=0.075)
    lr, N = 0.8, 12
    active = 0
    for _ in range(5):
        x = rng.standard_normal((N, 5))
        y = rng.integers(0, 7, N)
        W0 = [w.copy() for w in net.W]
        net.step(x, y, lr)
        for l in range(3):
            Ob, Xb = net.last["Obar"][l], net.last["Xbar"][l]
            s = lr * np.sum(np.linalg.norm(Ob, axis=1) * np.linalg.norm(Xb, axis=1))
            a = net.last["max_change_scale"][l]
            assert a == pytest.approx(min(1.0, N * 0.075 / s), rel=1e-12)
            change = net.W[l] - W0[l]
            np.testing.assert_allclose(change, a * lr * Ob.T @ Xb, atol=1e-14)
            assert np.linalg.norm(change) <= N * 0.075 * (1 + 1e-12)
            active += a < 1.0
    assert active >= 5   # the limit did bind in this run

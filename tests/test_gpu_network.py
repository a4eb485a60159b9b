"""GPU parity: ngsgd_step / ngsgd_average (through the C ABI) against the float64 oracle.

Bars (the benchmark spec): 1e-4 relative Frobenius error per preconditioned matrix and per gradient on the
same seeded inputs; 1e-3 absolute on the mean per-frame log-probability after 10 free-running steps.
"""
import numpy as np
import pytest

import workloads
from oracle.averaging import average_parameters
from oracle.network import NGSGDNetwork

pytestmark = pytest.mark.gpu

TOL = 1.0e-4


def rel(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def make_pair(ngsgd, spec, renorm=False, max_change=0.0, weights=None, max_batch=None, side_streams=0):
    import torch
    weights = workloads.initial_weights(spec) if weights is None else weights
    ora = NGSGDNetwork(spec.dims, spec.nonlin, weights, spec.pnorm_group, spec.rank_in, spec.rank_out, spec.alpha,
                       spec.num_samples_history, spec.epsilon, spec.update_period, renorm=renorm,
                       max_change_per_sample=max_change)
    gpu = ngsgd.Network(spec.dims, spec.nonlin, max_batch or spec.minibatch, spec.pnorm_group, spec.rank_in,
                        spec.rank_out, spec.alpha, spec.num_samples_history, spec.epsilon, spec.update_period,
                        renorm=renorm, max_change_per_sample=max_change, side_streams=side_streams)
    for l, w in enumerate(weights):
        gpu.set_params(l, torch.from_numpy(np.ascontiguousarray(w, dtype=np.float32)).cuda())
    return ora, gpu


def sync_from_oracle(ngsgd, spec, ora, gpu):
    """Loads the oracle's weights and all 2I factor states into the GPU replica (oracle -> GPU only)."""
    import torch
    for l in range(spec.n_layers):
        gpu.set_params(l, torch.from_numpy(np.ascontiguousarray(ora.W[l], dtype=np.float32)).cuda())
        for side, pre_o in ((ngsgd.NGSGD_SIDE_INPUT, ora.precond_in[l]), (ngsgd.NGSGD_SIDE_OUTPUT, ora.precond_out[l])):
            h = gpu.precond(l, side)
            if h is not None:
                h.set_state(torch.from_numpy(np.ascontiguousarray(pre_o.R)).cuda(),
                            torch.from_numpy(pre_o.d.copy()).cuda(), pre_o.rho, pre_o.t)
    torch.cuda.synchronize()


def singular_values(M):
    M = np.asarray(M, np.float64)
    G = M @ M.T if M.shape[0] <= M.shape[1] else M.T @ M
    return np.sqrt(np.maximum(np.linalg.eigvalsh(G)[::-1], 0.0))


def run_and_compare(ngsgd, spec, ora, gpu, steps, check_every=1, rows=None, tol=TOL, logp_tol=1e-3,
                    ambiguous_first=(), first_step=0, sync_every_step=False):
    """`ambiguous_first`: (layer, side) pairs whose first minibatch has a degenerate spectrum at the rank cut
    (e.g. onehot - uniform derivatives with repeated labels), so that the top-R eigenvectors are not unique.
    For those the first output is checked through what is unique (its singular values), and afterwards the
    oracle's state is loaded into the GPU so that the following steps can be compared element by element.
    `sync_every_step`: compare step by step from shared state (the oracle's weights and factors are loaded into
    the GPU after every step), which separates the accuracy of one step from the divergence that training
    dynamics add to any two trajectories."""
    import torch
    worst = dict(pre=0.0, grad=0.0, logp=0.0)
    for t in range(first_step, first_step + steps):
        x, y = workloads.minibatch(spec, t, rows=rows)
        obj_o = ora.step(x, y, spec.lr)
        out = gpu.step(torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda(), spec.lr)
        torch.cuda.synchronize()
        obj_g = float(out.item())
        n = len(y)
        worst["logp"] = max(worst["logp"], abs(obj_g - obj_o) / n)
        assert abs(obj_g - obj_o) / n < logp_tol, f"step {t}: mean log-prob {obj_g / n} vs {obj_o / n}"
        if t % check_every == 0 or t == steps - 1:
            for l in range(spec.n_layers):
                xo = gpu.last_preconditioned(l, ngsgd.NGSGD_SIDE_INPUT, n).cpu().numpy()
                oo = gpu.last_preconditioned(l, ngsgd.NGSGD_SIDE_OUTPUT, n).cpu().numpy()
                grad = gpu.last_gradient(l).cpu().numpy()
                if t == 0 and ((l, ngsgd.NGSGD_SIDE_OUTPUT) in ambiguous_first or
                               (l, ngsgd.NGSGD_SIDE_INPUT) in ambiguous_first):
                    for got, want in ((xo, ora.last["Xbar"][l]), (oo, ora.last["Obar"][l])):
                        sg, sw = singular_values(got), singular_values(want)
                        assert np.max(np.abs(sg - sw)) < tol * sw[0], f"layer {l}: spectrum of the output differs"
                        assert abs(np.linalg.norm(got.astype(np.float64)) / np.linalg.norm(want) - 1.0) < tol
                    continue
                e_x, e_o = rel(xo, ora.last["Xbar"][l]), rel(oo, ora.last["Obar"][l])
                e_g = rel(grad, ora.last["delta"][l])
                worst["pre"] = max(worst["pre"], e_x, e_o)
                worst["grad"] = max(worst["grad"], e_g)
                assert e_x < tol and e_o < tol, f"step {t} layer {l}: Xbar {e_x:.2e} Obar {e_o:.2e}"
                assert e_g < tol, f"step {t} layer {l}: gradient {e_g:.2e}"
                mc = float(gpu.last_max_change_scale(l).item())
                assert mc == pytest.approx(ora.last["max_change_scale"][l], rel=1e-4)
        if sync_every_step and t < first_step + steps - 1:
            for l in range(spec.n_layers):          # the update itself, before it is overwritten by the sync
                assert rel(gpu.get_params(l).cpu().numpy(), ora.W[l]) < tol
            sync_from_oracle(ngsgd, spec, ora, gpu)
        elif t == 0 and ambiguous_first:
            sync_from_oracle(ngsgd, spec, ora, gpu)
    for l in range(spec.n_layers):
        assert rel(gpu.get_params(l).cpu().numpy(), ora.W[l]) < tol
    return worst


def test_c0_ten_steps_free_running(ngsgd):
    """BASELINE configs[0]: tiny tanh MLP, minibatch 64, ranks 4 / 8, lr 0.01, 10 steps from the seed."""
    spec = workloads.c0_tiny()
    ora, gpu = make_pair(ngsgd, spec)
    worst = run_and_compare(ngsgd, spec, ora, gpu, spec.steps)
    print("c0 worst errors", worst)


def test_small_pnorm_net_with_renorm_and_max_change(ngsgd):
    """Reduced p-norm net with ragged sizes: p-norm, renormalisation, max-change, zero-initialised softmax."""
    spec = workloads.small_pnorm()
    ora, gpu = make_pair(ngsgd, spec, renorm=True, max_change=0.075)
    run_and_compare(ngsgd, spec, ora, gpu, spec.steps)
    assert min(ora.last["max_change_scale"]) <= 1.0


def test_small_pnorm_net_plain(ngsgd):
    """Same net without the stabilisers, smaller last minibatch, update period 1."""
    spec = workloads.small_pnorm()
    spec.update_period = 1
    spec.lr = 0.002
    ora, gpu = make_pair(ngsgd, spec)
    run_and_compare(ngsgd, spec, ora, gpu, 5)
    # the smaller minibatch is what the last two steps are for, not five steps' worth of accumulated divergence
    # (without the stabilisers the last layer's gradient is a sum that nearly cancels): continue from shared state
    sync_from_oracle(ngsgd, spec, ora, gpu)
    run_and_compare(ngsgd, spec, ora, gpu, 2, rows=spec.minibatch - 9)


@pytest.mark.parametrize("side_streams", [0, 1, 3])
def test_small_pnorm_net_past_the_always_update_phase(ngsgd, side_streams):
    """Sixteen steps without any synchronisation of state: steps 10, 11 only apply the factors, step 12 is the first
    periodic update and step 13 is the step that follows one, which the library orders around the factor updates
    still in flight (the layers whose factors are ready are preconditioned and updated first).  With the default
    three internal streams, with one (a single group of factors) and with two."""
    spec = workloads.small_pnorm()
    ora, gpu = make_pair(ngsgd, spec, renorm=True, max_change=0.075, side_streams=side_streams)
    worst = run_and_compare(ngsgd, spec, ora, gpu, 16)
    print("small p-norm net, 16 steps free running, side_streams", side_streams, worst)


@pytest.mark.parametrize("dims,nonlin", [([40, 50], []), ([40, 120, 50], [workloads.PNORM])])
def test_shallow_networks(ngsgd, dims, nonlin):
    """One affine layer (softmax regression: no backward pass, one group of factors) and two (the first layer's
    derivatives are the only ones the backward pass produces): 14 steps free running, through the always-update
    phase, a periodic update and the step after it."""
    spec = workloads.NetSpec("shallow", 7, dims, nonlin, 10, 64, 4, 8, 0.01, 14, softmax_zero_init=False,
                             label_law="uniform", splice=1, base_dim=40)
    ora, gpu = make_pair(ngsgd, spec, renorm=True, max_change=0.075)
    worst = run_and_compare(ngsgd, spec, ora, gpu, 14)
    print("shallow network", dims, worst)


def test_deepest_network(ngsgd):
    """The most layers the library takes (16, i.e. 32 factor instances: more than one grouped launch holds),
    alternating tanh and p-norm layers: 6 steps free running, then step by step from shared state (rounding
    differences grow through 16 layers: free running, the first layer's derivatives are 1.3e-4 apart after ten
    steps)."""
    dims = [40] + [64] * 15 + [30]
    nonlin = [workloads.TANH, workloads.PNORM] * 7 + [workloads.TANH]
    assert len(dims) - 1 == ngsgd.NGSGD_MAX_LAYERS
    spec = workloads.NetSpec("deep", 8, dims, nonlin, 2, 64, 4, 8, 0.01, 14, softmax_zero_init=False,
                             label_law="uniform", splice=1, base_dim=40)
    ora, gpu = make_pair(ngsgd, spec, renorm=True, max_change=0.075)
    worst = run_and_compare(ngsgd, spec, ora, gpu, 6)
    print("16-layer network, free running", worst)
    sync_from_oracle(ngsgd, spec, ora, gpu)
    worst = run_and_compare(ngsgd, spec, ora, gpu, 8, first_step=6, sync_every_step=True)
    print("16-layer network, step by step", worst)


@pytest.mark.parametrize("rows", [1, 2, 5, 63])
def test_tiny_minibatches_after_the_first(ngsgd, rows):
    """Once the factors exist a minibatch may be as small as one row (less than one tile, fewer rows than the
    rank): two such steps from shared state, the first of them an update step."""
    spec = workloads.small_pnorm()
    spec.update_period = 1
    ora, gpu = make_pair(ngsgd, spec, renorm=True, max_change=0.075)
    run_and_compare(ngsgd, spec, ora, gpu, 2)
    sync_from_oracle(ngsgd, spec, ora, gpu)
    worst = run_and_compare(ngsgd, spec, ora, gpu, 2, first_step=2, rows=rows, sync_every_step=True)
    print("minibatch of", rows, "rows", worst)


def test_rank_zero_is_plain_sgd(ngsgd):
    spec = workloads.c0_tiny()
    spec.rank_in = spec.rank_out = 0
    ora, gpu = make_pair(ngsgd, spec)
    run_and_compare(ngsgd, spec, ora, gpu, 3)
    assert gpu.precond(0, ngsgd.NGSGD_SIDE_INPUT) is None


def test_c1_full_size_first_steps(ngsgd):
    """BASELINE configs[1] at full size (360 -> 4 x p-norm 3000/300 -> 5000, minibatch 512, ranks 20 / 80) in the
    configuration bench.py times: renormalised p-norm layers and the max-change limit."""
    spec = workloads.c1_pnorm()
    ora, gpu = make_pair(ngsgd, spec, renorm=True, max_change=0.075)
    # zero-initialised softmax: the first derivatives are onehot - 1/5000 with many repeated labels, whose
    # covariance has equal eigenvalues across the rank-80 cut
    worst = run_and_compare(ngsgd, spec, ora, gpu, 4, ambiguous_first={(spec.n_layers - 1, ngsgd.NGSGD_SIDE_OUTPUT)})
    print("c1 worst errors, free running", worst)
    # further into training, step by step from shared state: steps 4..13 cover the always-update phase, two
    # apply-only steps (10, 11), and the first periodic update (12)
    sync_from_oracle(ngsgd, spec, ora, gpu)
    worst = run_and_compare(ngsgd, spec, ora, gpu, 10, first_step=4, sync_every_step=True)
    print("c1 worst errors, step by step", worst)
    # steps 14..17 free running from shared state: 16 is a periodic update whose factor updates are still in flight
    # when step 17 is enqueued, so step 17 takes the library's path around them at full size
    sync_from_oracle(ngsgd, spec, ora, gpu)
    worst = run_and_compare(ngsgd, spec, ora, gpu, 4, first_step=14)
    print("c1 worst errors, steps 14..17 free running", worst)


def test_wide_layers_ragged_minibatch(ngsgd):
    """Layers as wide as those of configs[1] with a minibatch that is no multiple of any tile (500 rows): the
    twelve-wavefront 64 x 96 tiles of the forward and backward products with a ragged row tile, ragged column tiles
    and a K tail, and the last row block of the fused apply kernel (500 = 7 x 64 + 52) at ranks 20 and 80."""
    import dataclasses
    base = workloads.c1_pnorm()
    spec = dataclasses.replace(base, name="wide_ragged", index=11, dims=[360, 3000, 3000, 5000], nonlin=base.nonlin[:2],
                               minibatch=500)
    ora, gpu = make_pair(ngsgd, spec, renorm=True, max_change=0.075)
    worst = run_and_compare(ngsgd, spec, ora, gpu, 3, ambiguous_first={(spec.n_layers - 1, ngsgd.NGSGD_SIDE_OUTPUT)})
    print("wide ragged worst errors, free running", worst)
    # past the always-update phase, step by step from shared state: apply-only steps (fused kernel) and an update
    sync_from_oracle(ngsgd, spec, ora, gpu)
    worst = run_and_compare(ngsgd, spec, ora, gpu, 10, first_step=3, sync_every_step=True)
    print("wide ragged worst errors, step by step", worst)


def test_c3_wide_tanh_first_steps(ngsgd):
    """BASELINE configs[3] at full size (440 -> 6 x tanh 2048 -> 8000, minibatch 1024, ranks 20 / 80): the tanh
    kernels, 2049-wide inputs and an 8000-way softmax (the widest row the softmax kernel keeps in registers)."""
    spec = workloads.c3_wide_tanh()
    ora, gpu = make_pair(ngsgd, spec)
    worst = run_and_compare(ngsgd, spec, ora, gpu, 2, ambiguous_first={(spec.n_layers - 1, ngsgd.NGSGD_SIDE_OUTPUT)})
    print("c3 worst errors, free running", worst)
    sync_from_oracle(ngsgd, spec, ora, gpu)
    worst = run_and_compare(ngsgd, spec, ora, gpu, 3, first_step=2, sync_every_step=True)
    print("c3 worst errors, step by step", worst)


def test_step_argument_errors(ngsgd):
    import torch
    spec = workloads.c0_tiny()
    _, gpu = make_pair(ngsgd, spec)
    x, y = workloads.minibatch(spec, 0, rows=80)
    with pytest.raises(ngsgd.NgsgdError):
        gpu.step(torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda(), 0.01)       # N > max_batch
    x, y = workloads.minibatch(spec, 0, rows=6)
    with pytest.raises(ngsgd.NgsgdError):
        gpu.step(torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda(), 0.01)       # N <= rank on the first step
    torch.cuda.synchronize()


def test_kernel_group_timing(ngsgd):
    """The event brackets of ngsgd_profile_*: categories and launch counts of a step, and the error that a read
    returns when more launch groups ran than the library keeps (instead of sums that silently miss some)."""
    import torch
    spec = workloads.c0_tiny()
    _, gpu = make_pair(ngsgd, spec)
    x, y = workloads.minibatch(spec, 0)
    x, y = torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda()
    out = torch.zeros(1, dtype=torch.float64, device="cuda")
    for _ in range(12):                      # past the always-update phase
        gpu.step(x, y, spec.lr, out)
    ngsgd.profile_enable(True)
    gpu.step(x, y, spec.lr, out)             # t = 12: an update step
    gpu.step(x, y, spec.lr, out)             # t = 13: apply only
    gpu.join()
    prof = ngsgd.profile_read()
    assert prof["gemm_fwd"][1] == 2 * spec.n_layers and prof["gemm_bwd"][1] == 2 * (spec.n_layers - 1)
    # the update step takes H, J and Xhat as separate products, the apply-only step the fused pass
    assert prof["precond_small"][1] >= 1 and prof["precond_xhat"][1] >= 1 and prof["precond_fused"][1] >= 1
    assert all(ms >= 0.0 for ms, _ in prof.values()) and prof["gemm_fwd"][0] > 0.0
    assert sum(c for _, c in ngsgd.profile_read().values()) == 0          # a read clears the record
    for _ in range(2000):                    # about 20 groups per step: more than the 32768 the library keeps
        gpu.step(x, y, spec.lr, out)
    gpu.join()
    with pytest.raises(ngsgd.NgsgdError):
        ngsgd.profile_read()
    ngsgd.profile_enable(False)
    torch.cuda.synchronize()


def test_average_replicas(ngsgd):
    """Sec. 3.1: every replica ends with the arithmetic mean; preconditioners restart as new processes do."""
    import torch
    spec = workloads.c0_tiny()
    pairs = [make_pair(ngsgd, spec) for _ in range(3)]
    for r, (ora, gpu) in enumerate(pairs):
        for t in range(2):
            x, y = workloads.minibatch(spec, t, replica=r)
            ora.step(x, y, spec.lr)
            gpu.step(torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda(), spec.lr)
    before = [[g.get_params(l).cpu().numpy().astype(np.float64) for l in range(spec.n_layers)] for _, g in pairs]
    average_parameters([o for o, _ in pairs])
    ngsgd.average([g for _, g in pairs], reset_preconditioners=True)
    torch.cuda.synchronize()
    for _, g in pairs:
        for l in range(spec.n_layers):
            got = g.get_params(l).cpu().numpy()
            mean = sum(b[l] for b in before) / 3.0
            np.testing.assert_allclose(got, mean, rtol=0, atol=2e-7 * np.abs(mean).max())
            assert rel(got, pairs[0][0].W[l]) < TOL
        assert g.precond(0, ngsgd.NGSGD_SIDE_OUTPUT).get_state()[3] == 0
    # replicas continue (re-initialising their factors) and still match the oracle
    for r, (ora, gpu) in enumerate(pairs[:2]):
        x, y = workloads.minibatch(spec, 5, replica=r)
        obj_o = ora.step(x, y, spec.lr)
        out = gpu.step(torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda(), spec.lr)
        torch.cuda.synchronize()
        assert abs(float(out.item()) - obj_o) / len(y) < 1e-3
        for l in range(spec.n_layers):
            assert rel(gpu.last_gradient(l).cpu().numpy(), ora.last["delta"][l]) < TOL


def test_average_replicas_on_their_own_streams(ngsgd):
    """Replicas stepped on streams of their own, averaged on another stream and stepped again, with no host
    synchronisation in between: the averaging call orders itself behind each replica's latest step (and its factor
    updates), and each replica's next step behind the averaged weights."""
    import torch
    spec = workloads.c0_tiny()   # (its first minibatch has no equal eigenvalues across the rank cut: free running)
    pairs = [make_pair(ngsgd, spec, side_streams=1) for _ in range(3)]
    streams = [torch.cuda.Stream() for _ in pairs]
    data = [[workloads.minibatch(spec, t, replica=r) for t in range(7)] for r in range(len(pairs))]
    dev = [[(torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda()) for x, y in d] for d in data]
    outs = [torch.zeros(1, dtype=torch.float64, device="cuda") for _ in pairs]
    torch.cuda.synchronize()
    for r, (ora, gpu) in enumerate(pairs):
        with torch.cuda.stream(streams[r]):
            for t in range(6):
                gpu.step(*dev[r][t], spec.lr, outs[r], stream=streams[r])
        for t in range(6):
            ora.step(*data[r][t], spec.lr)
    ngsgd.average([g for _, g in pairs], reset_preconditioners=True)      # on the default stream, at once
    average_parameters([o for o, _ in pairs])
    for r, (ora, gpu) in enumerate(pairs):                                  # and on, on the replicas' streams
        with torch.cuda.stream(streams[r]):
            gpu.step(*dev[r][6], spec.lr, outs[r], stream=streams[r])
        obj_o = ora.step(*data[r][6], spec.lr)
        streams[r].synchronize()
        assert abs(float(outs[r].item()) - obj_o) / len(data[r][6][1]) < 1e-3
    torch.cuda.synchronize()
    for ora, gpu in pairs:
        for l in range(spec.n_layers):
            assert rel(gpu.get_params(l).cpu().numpy(), ora.W[l]) < TOL


def test_back_to_back_steps_equal_synchronised_steps(ngsgd):
    """The factor updates of a step overlap the following steps on internal streams: steps enqueued back to back
    must give what steps separated by a device synchronisation give.
    (Both are GPU runs; sums over split products use atomics, so they agree to rounding, not bit for bit.)"""
    import torch
    spec = workloads.small_pnorm()
    batches = [workloads.minibatch(spec, t) for t in range(14)]
    batches = [(torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda()) for x, y in batches]
    finals = []
    for synchronise in (False, True):
        _, gpu = make_pair(ngsgd, spec, renorm=True, max_change=0.075)
        out = torch.zeros(1, dtype=torch.float64, device="cuda")
        objs = []
        for t, (x, y) in enumerate(batches):
            gpu.step(x, y, spec.lr, out)
            if synchronise:
                torch.cuda.synchronize()
            objs.append(out.clone())
        gpu.join()                                   # the caller's stream now covers the last factor updates too
        torch.cuda.current_stream().synchronize()
        finals.append(([gpu.get_params(l).cpu().numpy() for l in range(spec.n_layers)],
                       np.array([float(o.item()) for o in objs])))
    (w_free, o_free), (w_sync, o_sync) = finals
    np.testing.assert_allclose(o_free, o_sync, rtol=1e-5)
    for a, b in zip(w_free, w_sync):
        assert rel(a, b) < 1e-5

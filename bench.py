"""Benchmark of the NG-SGD minibatch step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

A step is one pass of the whole hot path (forward, objective, backward, natural-gradient
preconditioning of both matrices of every layer, rank-N update) over one synthetic minibatch of the
speech-shaped p-norm DNN workload (BASELINE configs[1]: 360 -> 4 x (affine 3000, p-norm 10 -> 300) ->
5000-way softmax, minibatch 512, ranks 20 / 80, fp32), with the renormalisation layer and the
max-change limit of the paper's recipe enabled.  Inputs are resident in HBM before the timed region.

Prints ONE JSON line on stdout; progress and the breakdown go to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_F32_TFLOPS = 157.3      # MI355X dense fp32 matrix peak
PEAK_HBM_GBS = 8000.0             # MI355X HBM3E
POOL = 16                         # distinct minibatches resident on the GPU, cycled


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def gemm_flops_per_step(spec, n):
    fwd = sum(2.0 * n * (spec.in_dims[l] + 1) * spec.dims[l + 1] for l in range(spec.n_layers))
    bwd = sum(2.0 * n * spec.in_dims[l] * spec.dims[l + 1] for l in range(1, spec.n_layers))
    return dict(gemm_fwd=fwd, gemm_bwd=bwd, gemm_upd=fwd)


def gemm_bytes_per_step(spec, n):
    """Operands read once and the result written once (the update also reads the weights it adds to)."""
    fwd = sum(4.0 * (n * (spec.in_dims[l] + 1) + (spec.in_dims[l] + 1) * spec.dims[l + 1] + n * spec.dims[l + 1])
              for l in range(spec.n_layers))
    bwd = sum(4.0 * (n * spec.dims[l + 1] + spec.in_dims[l] * spec.dims[l + 1] + n * spec.in_dims[l])
              for l in range(1, spec.n_layers))
    upd = sum(4.0 * (n * spec.dims[l + 1] + n * (spec.in_dims[l] + 1) + 2 * (spec.in_dims[l] + 1) * spec.dims[l + 1])
              for l in range(spec.n_layers))
    return dict(gemm_fwd=fwd, gemm_bwd=bwd, gemm_upd=upd)


def precond_flops(n, d, r, update):
    f = 2.0 * n * d * r * 2            # H and Xhat
    if update:
        f += 2.0 * n * d * r           # J
        f += 2.0 * r * r * d + 2.0 * r * r * n + 2.0 * r * r * d   # K, L, W_{t+1}
    return f


def precond_bytes(n, d, r, update):
    # read X once, write Xbar once, read W (and write it when the factor is updated)
    return 4.0 * (2.0 * n * d + (2.0 if update else 1.0) * r * d)


def measured_traffic_per_launch(category):
    """HBM bytes per launch of a layer-GEMM category, from the committed rocprofv3 --pmc summary (FETCH_SIZE and
    WRITE_SIZE runs of this file, scaled by a plain copy of known size; see the summary for the commands).
    None when the summary is missing or does not list the kernels."""
    import re
    # template arguments after the tile shape: A K-contiguous, B K-contiguous, epilogue, sum of squares, chunk, fp64
    pattern = {"gemm_fwd": r"gemm_kernel<\d+, \d+, 32, \d, \d, true, true, 0, false, 0, false",
               "gemm_bwd": r"gemm_kernel<\d+, \d+, 32, \d, \d, true, false, 0, false, 4, false",
               "gemm_upd": r"gemm_kernel<\d+, \d+, 32, \d, \d, false, false, 0, false, 0, false"}.get(category)
    path = os.path.join(ROOT, "profiles", "step_c1_pnorm_hbm_traffic.txt")
    if pattern is None or not os.path.exists(path):
        return None
    calls = total = 0.0
    for line in open(path):
        if re.search(pattern, line):
            cols = line.split()
            try:
                n, read_mb, write_mb = float(cols[-5]), float(cols[-2]), float(cols[-1])
            except (ValueError, IndexError):
                continue
            calls += n
            total += n * (read_mb + write_mb) * 1e6
    return total / calls if calls > 0 else None


def run_step_bench(args):
    import numpy as np
    import torch

    import paper_1410_7455_amd as ng
    import workloads

    spec = workloads.c1_pnorm()
    n = spec.minibatch
    net = ng.Network(spec.dims, spec.nonlin, n, spec.pnorm_group, spec.rank_in, spec.rank_out, spec.alpha,
                     spec.num_samples_history, spec.epsilon, spec.update_period, renorm=True,
                     max_change_per_sample=0.075)
    for l, w in enumerate(workloads.initial_weights(spec)):
        net.set_params(l, torch.from_numpy(w).cuda())
    pool = []
    for t in range(POOL):
        x, y = workloads.minibatch(spec, t)
        pool.append((torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda()))
    logp = torch.zeros(1, dtype=torch.float64, device="cuda")
    torch.cuda.synchronize()

    step_no = 0
    for _ in range(args.warmup):
        x, y = pool[step_no % POOL]
        net.step(x, y, spec.lr, logp)
        step_no += 1
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        x, y = pool[step_no % POOL]
        net.step(x, y, spec.lr, logp)
        step_no += 1
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    final_logp = float(logp.item()) / n
    ms_per_step = elapsed * 1e3 / args.steps
    frames_per_s = n * args.steps / elapsed
    log(f"[bench] {args.steps} steps in {elapsed:.3f} s -> {ms_per_step:.3f} ms/step, {frames_per_s:,.0f} frames/s, "
        f"mean log-prob of last minibatch {final_logp:.4f}")
    if not np.isfinite(final_logp):
        raise RuntimeError("training diverged: the benchmark number would be meaningless")

    # second pass with per-category HIP events on the launch stream (same steps, same shapes); bounded so that the
    # library's event pool (65536 events, about 70 per step) always holds every launch group of the pass
    prof_steps = min(args.steps, 400)
    ng.profile_enable(True)
    for _ in range(prof_steps):
        x, y = pool[step_no % POOL]
        net.step(x, y, spec.lr, logp)
        step_no += 1
    torch.cuda.synchronize()
    prof = ng.profile_read()
    ng.profile_enable(False)
    flops = gemm_flops_per_step(spec, n)
    total_ms = sum(ms for ms, _ in prof.values())
    breakdown = {}
    for name, (ms, cnt) in prof.items():
        if cnt == 0:
            continue
        entry = dict(ms_per_step=ms / prof_steps, launches_per_step=cnt / prof_steps, share=ms / total_ms)
        if name in flops:
            entry["tflops"] = flops[name] * prof_steps / (ms * 1e-3) / 1e12
        breakdown[name] = entry
        log(f"[bench]   {name:14s} {entry['ms_per_step'] * 1e3:9.1f} us/step  {entry['share'] * 100:5.1f} %"
            + (f"  {entry['tflops']:6.1f} TFLOP/s" if "tflops" in entry else ""))
    dominant = max((k for k in breakdown if k in flops), key=lambda k: breakdown[k]["ms_per_step"])
    ms, cnt = prof[dominant]
    achieved = flops[dominant] * prof_steps / (ms * 1e-3) / 1e12
    roofline = dict(bound="mfma", kernel=dominant, achieved=achieved, peak=PEAK_MFMA_F32_TFLOPS, unit="TFLOP/s",
                    frac=achieved / PEAK_MFMA_F32_TFLOPS, traffic=measured_traffic_per_launch(dominant),
                    traffic_unit="bytes of HBM traffic per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, from profiles/)",
                    algorithmic_bytes_per_launch=gemm_bytes_per_step(spec, n)[dominant] * prof_steps / cnt,
                    flops_per_launch=flops[dominant] * prof_steps / cnt, avg_launch_us=ms * 1e3 / cnt,
                    all_gemms_tflops=sum(flops.values()) * prof_steps /
                    (sum(prof[k][0] for k in flops) * 1e-3) / 1e12)
    return spec, ms_per_step, frames_per_s, roofline, breakdown, final_logp


def run_precond_bench(calls=200):
    """BASELINE configs[2]: the preconditioner alone, successive online updates (update on every call)."""
    import torch

    import paper_1410_7455_amd as ng
    import workloads

    out = []
    for spec in (workloads.c2_input_side(), workloads.c2_output_side()):
        ld = (spec.dim + 3) // 4 * 4
        pre = ng.Preconditioner(spec.dim, spec.rank, spec.rows, update_period=spec.update_period)
        pool = []
        for t in range(POOL):
            buf = torch.zeros((spec.rows, ld), dtype=torch.float32, device="cuda")
            buf[:, :spec.dim] = torch.from_numpy(workloads.spectrum_matrix(spec, t)).cuda()
            pool.append(buf)
        work = torch.empty_like(pool[0])
        for t in range(12):                      # initialisation and the first updates are not timed
            work.copy_(pool[t % POOL])
            pre.precondition(work)
        torch.cuda.synchronize()
        starts = [torch.cuda.Event(enable_timing=True) for _ in range(calls)]
        stops = [torch.cuda.Event(enable_timing=True) for _ in range(calls)]
        for t in range(calls):
            work.copy_(pool[t % POOL])
            starts[t].record()
            pre.precondition(work)
            stops[t].record()
        torch.cuda.synchronize()
        us = sum(s.elapsed_time(e) for s, e in zip(starts, stops)) * 1e3 / calls
        nbytes = precond_bytes(spec.rows, spec.dim, spec.rank, True)
        fl = precond_flops(spec.rows, spec.dim, spec.rank, True)
        gbs = nbytes / (us * 1e-6) / 1e9
        tfl = fl / (us * 1e-6) / 1e12
        entry = dict(workload=spec.name, us_per_call=us, algorithmic_bytes=nbytes, achieved_gbs=gbs,
                     hbm_frac=gbs / PEAK_HBM_GBS, flops=fl, achieved_tflops=tfl,
                     mfma_frac=tfl / PEAK_MFMA_F32_TFLOPS, update_every_call=True)
        log(f"[bench] precondition {spec.name}: {us:.1f} us/call, {gbs:.0f} GB/s algorithmic "
            f"({entry['hbm_frac'] * 100:.1f} % of HBM peak), {tfl:.2f} TFLOP/s")
        out.append(entry)
        del pre
    return out


def run_wide_bench(steps=40, warmup=12):
    """BASELINE configs[3]: the wider tanh DNN (440 -> 6 x tanh 2048 -> 8000, minibatch 1024, ranks 20 / 80),
    whose layer products (1024 x 2049 x 2048) are large enough to fill the chip several times over."""
    import torch

    import paper_1410_7455_amd as ng
    import workloads

    spec = workloads.c3_wide_tanh()
    n = spec.minibatch
    net = ng.Network(spec.dims, spec.nonlin, n, spec.pnorm_group, spec.rank_in, spec.rank_out, spec.alpha,
                     spec.num_samples_history, spec.epsilon, spec.update_period, max_change_per_sample=0.075)
    for l, w in enumerate(workloads.initial_weights(spec)):
        net.set_params(l, torch.from_numpy(w).cuda())
    pool = []
    for t in range(4):
        x, y = workloads.minibatch(spec, t)
        pool.append((torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda()))
    logp = torch.zeros(1, dtype=torch.float64, device="cuda")
    for t in range(warmup):
        net.step(*pool[t % 4], spec.lr, logp)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(steps):
        net.step(*pool[(warmup + t) % 4], spec.lr, logp)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    final_logp = float(logp.item()) / n
    ng.profile_enable(True)
    for t in range(steps):
        net.step(*pool[t % 4], spec.lr, logp)
    torch.cuda.synchronize()
    prof = ng.profile_read()
    ng.profile_enable(False)
    flops = gemm_flops_per_step(spec, n)
    gemm = {k: dict(ms_per_step=prof[k][0] / steps, tflops=flops[k] * steps / (prof[k][0] * 1e-3) / 1e12) for k in flops}
    all_tf = sum(flops.values()) * steps / (sum(prof[k][0] for k in flops) * 1e-3) / 1e12
    log(f"[bench] configs[3] wide tanh net: {elapsed * 1e3 / steps:.3f} ms/step, {n * steps / elapsed:,.0f} frames/s, "
        f"layer GEMMs {all_tf:.1f} TFLOP/s ({all_tf / PEAK_MFMA_F32_TFLOPS * 100:.0f} % of fp32 matrix peak): "
        + ", ".join(f"{k} {v['tflops']:.1f}" for k, v in gemm.items()) + f"; mean log-prob {final_logp:.4f}")
    del net
    return dict(workload="configs[3] wider tanh DNN: 440 -> 6x tanh 2048 -> 8000, minibatch 1024, ranks 20/80, "
                         "update period 4, max-change 0.075, lr 0.01",
                value=n * steps / elapsed, unit="frames/s", ms_per_step=elapsed * 1e3 / steps, steps=steps,
                final_mean_logprob=final_logp, gemm=gemm, all_gemms_tflops=all_tf,
                all_gemms_mfma_frac=all_tf / PEAK_MFMA_F32_TFLOPS)


def run_simple_bench(steps=60, warmup=5, calls=40):
    """The simple method of App. A on the same workloads: the configs[1] step with every one of the 2I matrices
    preconditioned from the other rows of its own minibatch (no factor state), and the two configs[2] matrix
    shapes through ngsgd_precondition_simple alone.  The paper's own comparison (Sec. 6): 208 s per outer
    iteration with the simple method against 93 s with the online method and 88 s for plain SGD, on a K20."""
    import torch

    import paper_1410_7455_amd as ng
    import workloads

    spec = workloads.c1_pnorm()
    n = spec.minibatch
    net = ng.Network(spec.dims, spec.nonlin, n, spec.pnorm_group, spec.rank_in, spec.rank_out, spec.alpha,
                     spec.num_samples_history, spec.epsilon, spec.update_period, renorm=True,
                     max_change_per_sample=0.075, method="simple")
    for l, w in enumerate(workloads.initial_weights(spec)):
        net.set_params(l, torch.from_numpy(w).cuda())
    pool = []
    for t in range(POOL):
        x, y = workloads.minibatch(spec, t)
        pool.append((torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda()))
    logp = torch.zeros(1, dtype=torch.float64, device="cuda")
    for t in range(warmup):
        net.step(*pool[t % POOL], spec.lr, logp)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(steps):
        net.step(*pool[(warmup + t) % POOL], spec.lr, logp)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    final_logp = float(logp.item()) / n
    ng.profile_enable(True)
    for t in range(steps):
        net.step(*pool[t % POOL], spec.lr, logp)
    torch.cuda.synchronize()
    prof = ng.profile_read()
    ng.profile_enable(False)
    breakdown = {k: dict(ms_per_step=ms / steps, launches_per_step=c / steps) for k, (ms, c) in prof.items() if c}
    log(f"[bench] simple method (App. A): {elapsed * 1e3 / steps:.3f} ms/step, {n * steps / elapsed:,.0f} frames/s, "
        f"mean log-prob of last minibatch {final_logp:.4f}; "
        + ", ".join(f"{k} {v['ms_per_step'] * 1e3:.0f} us" for k, v in breakdown.items() if k.startswith("simple")))
    del net
    shapes = []
    for ps in (workloads.c2_input_side(), workloads.c2_output_side()):
        ld = (ps.dim + 3) // 4 * 4
        pre = ng.SimplePreconditioner(ps.rows, ps.dim)
        mats = []
        for t in range(4):
            buf = torch.zeros((ps.rows, ld), dtype=torch.float32, device="cuda")
            buf[:, :ps.dim] = torch.from_numpy(workloads.spectrum_matrix(ps, t)).cuda()
            mats.append(buf)
        work = torch.empty_like(mats[0])
        for t in range(3):
            work.copy_(mats[t % 4])
            pre.precondition(work[:, :ps.dim])
        torch.cuda.synchronize()
        starts = [torch.cuda.Event(enable_timing=True) for _ in range(calls)]
        stops = [torch.cuda.Event(enable_timing=True) for _ in range(calls)]
        for t in range(calls):
            work.copy_(mats[t % 4])
            starts[t].record()
            pre.precondition(work[:, :ps.dim])
            stops[t].record()
        torch.cuda.synchronize()
        us = sum(a.elapsed_time(b) for a, b in zip(starts, stops)) * 1e3 / calls
        m = min(ps.rows, ps.dim)
        big = max(ps.rows, ps.dim)
        mp = (m + 31) // 32 * 32
        fl = 2.0 * m * m * big + 2.0 * mp ** 3 + 2.0 * ps.rows * ps.dim * m     # Gram, inverse, Q
        nbytes = 8.0 * ps.rows * ps.dim                                            # X read once, Xbar written once
        entry = dict(workload=ps.name.replace("_r20", "").replace("_r80", ""), us_per_call=us, flops=fl,
                     achieved_tflops=fl / (us * 1e-6) / 1e12, algorithmic_bytes=nbytes,
                     achieved_gbs=nbytes / (us * 1e-6) / 1e9, inverse_size=m)
        log(f"[bench] simple method {entry['workload']}: {us:.1f} us/call, {entry['achieved_tflops']:.2f} TFLOP/s, "
            f"{entry['achieved_gbs']:.0f} GB/s algorithmic")
        shapes.append(entry)
        del pre
    return dict(workload="configs[1] step and configs[2] matrix shapes with the simple method (App. A)",
                value=n * steps / elapsed, unit="frames/s", ms_per_step=elapsed * 1e3 / steps, steps=steps,
                final_mean_logprob=final_logp, breakdown=breakdown, precondition=shapes,
                paper_context="K20, seconds per outer iteration: plain SGD 88, online NG-SGD 93, simple NG-SGD 208")


def run_replica_bench(replicas=8, rounds=4, steps_per_round=400):
    """BASELINE configs[4]: `replicas` copies of the configs[1] network resident on the one GPU, each
    stepping on its own HIP stream over its own data shard, parameters averaged on the device between rounds
    (which also resets the preconditioners, as the paper's re-spawned jobs do).  A single step leaves much of the
    chip idle (a few hundred tiles for 256 compute units); independent replicas fill it.  The labels of the
    synthetic data are independent of the inputs, so a replica can only learn the prior and memorise its own
    minibatches: the log-probabilities after averaging say nothing about the method."""
    import torch

    import paper_1410_7455_amd as ng
    import workloads

    spec = workloads.c1_pnorm()
    n = spec.minibatch
    nets, streams, pools, logps = [], [], [], []
    weights = workloads.initial_weights(spec)
    for r in range(replicas):
        net = ng.Network(spec.dims, spec.nonlin, n, spec.pnorm_group, spec.rank_in, spec.rank_out, spec.alpha,
                         spec.num_samples_history, spec.epsilon, spec.update_period, renorm=True,
                         max_change_per_sample=0.075, side_streams=1)   # many networks on one GPU: one stream each
        for l, w in enumerate(weights):
            net.set_params(l, torch.from_numpy(w).cuda())
        nets.append(net)
        streams.append(torch.cuda.Stream())
        logps.append(torch.zeros(1, dtype=torch.float64, device="cuda"))
        pool = []
        for t in range(4):
            x, y = workloads.minibatch(spec, t, replica=r)
            pool.append((torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda()))
        pools.append(pool)
    torch.cuda.synchronize()

    def steps_on_streams(steps, t0):
        for t in range(t0, t0 + steps):
            for r in range(replicas):
                with torch.cuda.stream(streams[r]):
                    nets[r].step(*pools[r][t % 4], spec.lr, logps[r])
        torch.cuda.synchronize()

    steps_on_streams(12, 0)               # first initialisation of all factors: not timed
    t_steady = t_avg = t_reinit = 0.0
    step_no = 12
    t_begin = time.perf_counter()
    for k in range(rounds):
        t0 = time.perf_counter()
        steps_on_streams(steps_per_round, step_no)
        t1 = time.perf_counter()
        ng.average(nets, reset_preconditioners=True)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        steps_on_streams(1, step_no + steps_per_round)   # rebuilds every factor from this minibatch (App. B.3.2)
        t3 = time.perf_counter()
        step_no += steps_per_round + 1
        t_steady += t1 - t0
        t_avg += t2 - t1
        t_reinit += t3 - t2
    elapsed = time.perf_counter() - t_begin
    steady = n * replicas * rounds * steps_per_round / t_steady
    overall = n * replicas * rounds * (steps_per_round + 1) / elapsed
    last = [float(l.item()) / n for l in logps]
    log(f"[bench] {replicas} interleaved replicas: {steady:,.0f} frames/s aggregate between averaging points "
        f"({rounds} x {steps_per_round} steps each), averaging {t_avg * 1e3 / rounds:.2f} ms, re-initialisation step "
        f"{t_reinit * 1e3 / rounds:.1f} ms, {overall:,.0f} frames/s overall; last mean log-probs "
        f"{min(last):.3f} .. {max(last):.3f}")
    return dict(workload="configs[4]: replicas of configs[1] interleaved on HIP streams, on-device averaging every "
                         f"{steps_per_round} minibatches with preconditioner reset, {rounds} rounds",
                replicas=replicas, rounds=rounds, steps_per_round=steps_per_round, value=steady, unit="frames/s",
                ms_per_replica_step=t_steady * 1e3 / (replicas * rounds * steps_per_round),
                averaging_ms=t_avg * 1e3 / rounds, reinitialisation_step_ms=t_reinit * 1e3 / rounds,
                overall_frames_per_s=overall)


def run_cpu_baseline(max_steps=120, budget_s=20.0):
    """The float64 oracle as it stands, timed on the host cores on a bounded sample of the same workload."""
    import workloads
    from oracle.network import NGSGDNetwork

    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count() or 1])
    except Exception:
        threads = os.cpu_count() or 1
    spec = workloads.c1_pnorm()
    net = NGSGDNetwork(spec.dims, spec.nonlin, workloads.initial_weights(spec), spec.pnorm_group, spec.rank_in,
                       spec.rank_out, spec.alpha, spec.num_samples_history, spec.epsilon, spec.update_period,
                       renorm=True, max_change_per_sample=0.075)
    batches = [workloads.minibatch(spec, t) for t in range(max_steps + 1)]
    net.step(*batches[0], spec.lr)          # state initialisation (eigen-decompositions) is not timed
    done = 0
    t0 = time.perf_counter()
    while done < max_steps and time.perf_counter() - t0 < budget_s:
        net.step(*batches[done + 1], spec.lr)
        done += 1
    elapsed = time.perf_counter() - t0
    value = spec.minibatch * done / elapsed
    log(f"[bench] oracle (float64 NumPy, {threads} threads): {done} steps in {elapsed:.1f} s -> {value:,.0f} frames/s")
    return dict(value=value, unit="frames/s", cores=threads, kind="oracle",
                sample=f"{done} steps of the same workload after 1 untimed initialisation step")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-precond", action="store_true")
    ap.add_argument("--no-replicas", action="store_true")
    ap.add_argument("--no-wide", action="store_true", help="skip the configs[3] leg (wider tanh DNN)")
    ap.add_argument("--no-simple", action="store_true", help="skip the simple-method leg (App. A)")
    ap.add_argument("--precond-only", action="store_true",
                    help="run only the preconditioner microbenchmark (BASELINE configs[2]); used for its profile")
    ap.add_argument("--simple-only", action="store_true",
                    help="run only the simple-method leg (App. A); used for its profile")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device-to-device copy (the known-size reference for scaling "
                         "the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py measures one GPU: this build has no multi-GPU path (replicas only exchange parameters "
            "at averaging points).  Run with --gpus 1.")
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        log("bench.py needs a GPU")
        sys.exit(1)
    torch.cuda.set_device(0)
    if args.precond_only:
        print(json.dumps({"precondition_roofline": run_precond_bench()}), flush=True)
        return
    if args.simple_only:
        print(json.dumps({"simple_method": run_simple_bench()}), flush=True)
        return
    spec, ms_per_step, frames_per_s, roofline, breakdown, final_logp = run_step_bench(args)
    if args.calibrate_copy:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    precond = None if args.no_precond else run_precond_bench()
    wide = None if args.no_wide else run_wide_bench()
    simple = None if args.no_simple else run_simple_bench()
    replica = None if args.no_replicas else run_replica_bench()
    cpu = None if args.no_cpu_baseline else run_cpu_baseline()
    result = {
        "metric": "NG-SGD training frames/sec (p-norm DNN, mb 512) + precondition % roofline",
        "value": frames_per_s,
        "unit": "frames/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": "configs[1] speech-shaped p-norm DNN: 360 -> 4x(3000 -> p-norm 300) -> 5000, "
                        "minibatch 512, ranks 20/80, update period 4, renorm + max-change 0.075, lr 0.01",
            "minibatch": spec.minibatch,
            "params": spec.n_params(),
            "pool_minibatches": POOL,
            "final_mean_logprob": final_logp,
        },
        "roofline": roofline,
        "cpu_baseline": cpu,
        "precondition_roofline": precond,
        "wide_tanh_net": wide,
        "simple_method": simple,
        "replica_interleaving": replica,
        "breakdown": breakdown,
    }
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()

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
POOL = 16                         # distinct matrices / minibatches resident on the GPU, cycled (side legs)
REPLICA_POOL = 64                 # distinct minibatches per replica in the interleaving leg, cycled
MAX_FRESH = 4096                  # most distinct minibatches the main leg keeps resident (0.74 MB each)


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
                n, read_mb, write_mb = float(cols[-7]), float(cols[-2]), float(cols[-1])
            except (ValueError, IndexError):
                continue
            calls += n
            total += n * (read_mb + write_mb) * 1e6
    return total / calls if calls > 0 else None


def machine_peaks():
    """Peaks re-derived on the box that runs the measurement, next to the data-sheet values the fractions use:
    fp32 matrix peak = compute units x clock x 256 flop / clock / unit (both read from `rocminfo`), and the
    bandwidth of a plain device-to-device copy of 1 GiB (read + write bytes over its HIP-event time)."""
    import re
    import subprocess

    import torch

    out = dict(datasheet_mfma_f32_tflops=PEAK_MFMA_F32_TFLOPS, datasheet_hbm_gbs=PEAK_HBM_GBS)
    try:
        txt = subprocess.run(["rocminfo"], capture_output=True, text=True, timeout=60).stdout
        gpu = txt[txt.index("gfx9"):] if "gfx9" in txt else txt
        cus = int(re.search(r"Compute Unit:\s+(\d+)", gpu).group(1))
        mhz = int(re.search(r"Max Clock Freq\. \(MHz\):\s+(\d+)", gpu).group(1))
        out.update(compute_units=cus, max_clock_mhz=mhz, derived_mfma_f32_tflops=cus * mhz * 1e6 * 256 / 1e12)
    except Exception as e:   # rocminfo missing or its format changed: the data-sheet values still stand
        out["rocminfo_error"] = str(e)[:200]
    src = torch.ones(256 * 1024 * 1024, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    times = []
    for _ in range(5):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        dst.copy_(src)
        b.record()
        torch.cuda.synchronize()
        times.append(a.elapsed_time(b))
    times.sort()
    out["measured_copy_gbs"] = 2.0 * src.numel() * 4 / (times[len(times) // 2] * 1e-3) / 1e9
    del src, dst
    log(f"[bench] machine: {out.get('compute_units')} CUs at {out.get('max_clock_mhz')} MHz -> "
        f"{out.get('derived_mfma_f32_tflops', float('nan')):.1f} TFLOP/s fp32 matrix peak (data sheet "
        f"{PEAK_MFMA_F32_TFLOPS}); 1 GiB copy {out['measured_copy_gbs']:.0f} GB/s read+write (data sheet HBM "
        f"{PEAK_HBM_GBS:.0f})")
    return out


def step_work(spec, n, update_period):
    """Algorithmic work of one step averaged over an update period: flops and HBM bytes of the layer GEMMs and of
    the 2I preconditioner calls (one call in `update_period` also updates its factor)."""
    gf, gb = gemm_flops_per_step(spec, n), gemm_bytes_per_step(spec, n)
    pf = pb = 0.0
    for l in range(spec.n_layers):
        for d, r in ((spec.in_dims[l] + 1, spec.rank_in), (spec.dims[l + 1], spec.rank_out)):
            pf += ((update_period - 1) * precond_flops(n, d, r, False) + precond_flops(n, d, r, True)) / update_period
            pb += ((update_period - 1) * precond_bytes(n, d, r, False) + precond_bytes(n, d, r, True)) / update_period
    return dict(gemm_flops=sum(gf.values()), gemm_bytes=sum(gb.values()), precond_flops=pf, precond_bytes=pb)


def timed_repetitions(net, pool, spec, logp, step_no, steps, reps):
    """`reps` repetitions of `steps` steps, each bracketed by a pair of HIP events on the stream the steps are
    launched on (the stop event behind ngsgd_join, so that it also covers the factor updates on the network's own
    streams) and by device synchronisations with a host clock.  Returns the per-repetition milliseconds by both
    clocks and the advanced step counter."""
    import torch
    ev_ms, wall_ms = [], []
    for _ in range(reps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        a.record()
        for _ in range(steps):
            x, y = pool[step_no % len(pool)]
            net.step(x, y, spec.lr, logp)
            step_no += 1
        net.join()
        b.record()
        torch.cuda.synchronize()
        wall_ms.append((time.perf_counter() - t0) * 1e3)
        ev_ms.append(a.elapsed_time(b))
    return ev_ms, wall_ms, step_no


def median(v):
    v = sorted(v)
    return v[len(v) // 2] if len(v) % 2 else 0.5 * (v[len(v) // 2 - 1] + v[len(v) // 2])


def run_step_bench(args):
    import numpy as np
    import torch

    import paper_1410_7455_amd as ng
    import workloads

    spec = workloads.c1_pnorm()
    n = spec.minibatch
    always_first = 10                    # App. B.4: the factors are updated on each of the first 10 minibatches
    net = ng.Network(spec.dims, spec.nonlin, n, spec.pnorm_group, spec.rank_in, spec.rank_out, spec.alpha,
                     spec.num_samples_history, spec.epsilon, spec.update_period, renorm=True,
                     max_change_per_sample=0.075)
    for l, w in enumerate(workloads.initial_weights(spec)):
        net.set_params(l, torch.from_numpy(w).cuda())
    # Untimed: at least --warmup steps, and whatever it takes to leave the start-up phase of the schedule (state
    # initialisation at t = 0, a factor update on every one of the first 10 steps) and to start the timed region on
    # a step whose factors are due, so that every repetition sees the same mix: one updating step per period.
    period = spec.update_period
    untimed = max(args.warmup, always_first + 2)
    untimed = (untimed + period - 1) // period * period
    prof_steps = max(period, min(args.steps, 400) // period * period)
    # A fresh minibatch for every step (resident in HBM before the clock starts), as in training: a small pool that
    # is revisited is memorised within a few hundred steps, the derivatives collapse, the R x R eigen-problems get
    # easy and the step gets faster than it is on data.  Beyond MAX_FRESH steps the pool is cycled.
    POOL = min(MAX_FRESH, untimed + args.reps * args.steps + 8 * period + prof_steps)
    pool = []
    for t in range(POOL):
        x, y = workloads.minibatch(spec, t)
        pool.append((torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda()))
    logp = torch.zeros(1, dtype=torch.float64, device="cuda")
    torch.cuda.synchronize()
    step_no = 0
    for _ in range(untimed):
        x, y = pool[step_no % POOL]
        net.step(x, y, spec.lr, logp)
        step_no += 1
    torch.cuda.synchronize()
    ev_ms, wall_ms, step_no = timed_repetitions(net, pool, spec, logp, step_no, args.steps, args.reps)
    final_logp = float(logp.item()) / n
    per_step = [m / args.steps for m in ev_ms]
    ms_per_step = median(per_step)
    frames_per_s = n / (ms_per_step * 1e-3)
    timing = dict(repetitions=args.reps, steps_per_repetition=args.steps, untimed_steps=untimed,
                  whole_update_periods=args.steps % period == 0, clock="HIP events on the launch stream",
                  ms_per_step_median=ms_per_step, ms_per_step_min=min(per_step), ms_per_step_max=max(per_step),
                  ms_per_step_host_clock_median=median(wall_ms) / args.steps)
    log(f"[bench] {args.reps} x {args.steps} steps after {untimed} untimed: median {ms_per_step:.4f} ms/step "
        f"(min {min(per_step):.4f}, max {max(per_step):.4f}; host clock {timing['ms_per_step_host_clock_median']:.4f}) "
        f"-> {frames_per_s:,.0f} frames/s, mean log-prob of last minibatch {final_logp:.4f}")
    if not np.isfinite(final_logp):
        raise RuntimeError("training diverged: the benchmark number would be meaningless")

    # Per-step time by position in the update period (the updating step, the step after it, ...): one event pair
    # per step, so slightly longer than the back-to-back figure above.
    by_phase = [[] for _ in range(period)]
    for _ in range(8 * period):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        x, y = pool[step_no % POOL]
        net.step(x, y, spec.lr, logp)
        b.record()
        by_phase[step_no % period].append((a, b))
        step_no += 1
    torch.cuda.synchronize()
    timing["ms_by_step_in_period"] = [median([a.elapsed_time(b) for a, b in ph]) for ph in by_phase]
    log("[bench]   ms by step in the update period (0 = the step that updates the factors): "
        + ", ".join(f"{v:.3f}" for v in timing["ms_by_step_in_period"]))

    # second pass with per-category HIP events on the launch stream (same steps, same shapes); bounded so that the
    # library's event pool (65536 events, about 70 per step) always holds every launch group of the pass
    ng.profile_enable(True)
    for _ in range(prof_steps):
        x, y = pool[step_no % POOL]
        net.step(x, y, spec.lr, logp)
        step_no += 1
    torch.cuda.synchronize()
    prof = ng.profile_read()
    ng.profile_enable(False)
    flops = gemm_flops_per_step(spec, n)
    breakdown = {}
    for name, (ms, cnt) in prof.items():
        if cnt == 0:
            continue
        # the groups overlap (side streams), so the shares of the wall step need not add up to one
        entry = dict(ms_per_step=ms / prof_steps, launches_per_step=cnt / prof_steps,
                     share_of_wall_step=ms / prof_steps / ms_per_step)
        if name in flops:
            entry["tflops"] = flops[name] * prof_steps / (ms * 1e-3) / 1e12
        breakdown[name] = entry
        log(f"[bench]   {name:14s} {entry['ms_per_step'] * 1e3:9.1f} us/step  {entry['share_of_wall_step'] * 100:5.1f} %"
            + (f"  {entry['tflops']:6.1f} TFLOP/s" if "tflops" in entry else ""))
    dominant = max((k for k in breakdown if k in flops), key=lambda k: breakdown[k]["ms_per_step"])
    ms, cnt = prof[dominant]
    achieved = flops[dominant] * prof_steps / (ms * 1e-3) / 1e12
    roofline = dict(bound="mfma", kernel=dominant, achieved=achieved, peak=PEAK_MFMA_F32_TFLOPS, unit="TFLOP/s",
                    frac=achieved / PEAK_MFMA_F32_TFLOPS, traffic=measured_traffic_per_launch(dominant),
                    traffic_unit="bytes of HBM traffic per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE); read from the "
                                 "committed summary under profiles/, not measured in this run",
                    algorithmic_bytes_per_launch=gemm_bytes_per_step(spec, n)[dominant] * prof_steps / cnt,
                    flops_per_launch=flops[dominant] * prof_steps / cnt, avg_launch_us=ms * 1e3 / cnt,
                    all_gemms_tflops=sum(flops.values()) * prof_steps /
                    (sum(prof[k][0] for k in flops) * 1e-3) / 1e12)
    roofline["all_gemms_frac"] = roofline["all_gemms_tflops"] / PEAK_MFMA_F32_TFLOPS
    # whole step: frames/s if every flop ran at the fp32 matrix peak and every algorithmic byte at the HBM peak
    work = step_work(spec, n, period)
    t_flops = (work["gemm_flops"] + work["precond_flops"]) / (PEAK_MFMA_F32_TFLOPS * 1e12)
    t_bytes = (work["gemm_bytes"] + work["precond_bytes"]) / (PEAK_HBM_GBS * 1e9)
    at_peak = n / max(t_flops, t_bytes)
    step_roofline = dict(bound="mfma" if t_flops >= t_bytes else "hbm", flops_per_step=work["gemm_flops"] + work["precond_flops"],
                         bytes_per_step=work["gemm_bytes"] + work["precond_bytes"], frames_per_s_at_peak=at_peak,
                         frac=frames_per_s / at_peak)
    log(f"[bench]   whole step: {step_roofline['flops_per_step'] / 1e9:.2f} GFLOP, {step_roofline['bytes_per_step'] / 1e6:.0f} MB "
        f"algorithmic -> {at_peak:,.0f} frames/s at peak; achieved fraction {step_roofline['frac']:.3f}")
    timing["distinct_minibatches"] = POOL
    return spec, ms_per_step, frames_per_s, roofline, breakdown, final_logp, timing, step_roofline


def run_precond_bench(calls=200, reps=5):
    """BASELINE configs[2]: the preconditioner alone.  Two figures per shape: successive online updates (the factor
    is updated on every call, as configs[2] states) and the call without a factor update (App. B.5, "without
    updating": what three of four training steps run).  Median over `reps` repetitions of `calls` calls, each
    repetition bracketed by HIP events on the launch stream; the untimed refill of the work matrix between calls
    is inside the bracket of the repetition and subtracted through a repetition of refills alone."""
    import torch

    import paper_1410_7455_amd as ng
    import workloads

    out = []
    for spec in (workloads.c2_input_side(), workloads.c2_output_side()):
        ld = (spec.dim + 3) // 4 * 4
        pool = []
        for t in range(POOL):
            buf = torch.zeros((spec.rows, ld), dtype=torch.float32, device="cuda")
            buf[:, :spec.dim] = torch.from_numpy(workloads.spectrum_matrix(spec, t)).cuda()
            pool.append(buf)
        work = torch.empty_like(pool[0])

        def bracket(fn):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            a.record()
            for t in range(calls):
                work.copy_(pool[t % POOL])
                fn()
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) * 1e3 / calls

        refill_us = median([bracket(lambda: None) for _ in range(reps)])
        for update in (True, False):
            period = spec.update_period if update else 1 << 30
            pre = ng.Preconditioner(spec.dim, spec.rank, spec.rows, update_period=period)
            for t in range(12):                      # initialisation and the first (always updating) calls: untimed
                work.copy_(pool[t % POOL])
                pre.precondition(work)
            us_all = [bracket(lambda: pre.precondition(work)) - refill_us for _ in range(reps)]
            us = median(us_all)
            nbytes = precond_bytes(spec.rows, spec.dim, spec.rank, update)
            fl = precond_flops(spec.rows, spec.dim, spec.rank, update)
            gbs = nbytes / (us * 1e-6) / 1e9
            tfl = fl / (us * 1e-6) / 1e12
            t_roof = max(nbytes / (PEAK_HBM_GBS * 1e9), fl / (PEAK_MFMA_F32_TFLOPS * 1e12)) * 1e6
            entry = dict(workload=spec.name, update_every_call=update, us_per_call=us, us_per_call_min=min(us_all),
                         us_per_call_max=max(us_all), refill_us=refill_us, algorithmic_bytes=nbytes,
                         achieved_gbs=gbs, hbm_frac=gbs / PEAK_HBM_GBS, flops=fl, achieved_tflops=tfl,
                         mfma_frac=tfl / PEAK_MFMA_F32_TFLOPS, roofline_us=t_roof, roofline_frac=t_roof / us)
            log(f"[bench] precondition {spec.name} ({'update every call' if update else 'no factor update'}): "
                f"{us:.1f} us/call (min {min(us_all):.1f}, max {max(us_all):.1f}), {gbs:.0f} GB/s algorithmic "
                f"({entry['hbm_frac'] * 100:.1f} % of HBM peak), {tfl:.2f} TFLOP/s; roofline {t_roof:.1f} us "
                f"-> {entry['roofline_frac'] * 100:.0f} %")
            out.append(entry)
            del pre
    return out


def run_c0_bench(reps=5):
    """BASELINE configs[0]: the tiny tanh net, its 10 steps from the seed (state initialisation on the first step,
    a factor update on every step), timed as a whole; median over fresh networks."""
    import torch

    import paper_1410_7455_amd as ng
    import workloads

    spec = workloads.c0_tiny()
    n = spec.minibatch
    batches = [tuple(torch.from_numpy(a).cuda() for a in workloads.minibatch(spec, t)) for t in range(spec.steps)]
    logp = torch.zeros(1, dtype=torch.float64, device="cuda")
    times = []
    for _ in range(reps + 1):
        net = ng.Network(spec.dims, spec.nonlin, n, spec.pnorm_group, spec.rank_in, spec.rank_out, spec.alpha,
                         spec.num_samples_history, spec.epsilon, spec.update_period)
        for l, w in enumerate(workloads.initial_weights(spec)):
            net.set_params(l, torch.from_numpy(w).cuda())
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for x, y in batches:
            net.step(x, y, spec.lr, logp)
        net.join()
        b.record()
        torch.cuda.synchronize()
        times.append(a.elapsed_time(b))
        del net
    ms = median(times[1:])               # the first network also pays one-time kernel loading
    final = float(logp.item()) / n
    log(f"[bench] configs[0] tiny tanh net: {spec.steps} steps in {ms:.2f} ms -> {n * spec.steps / (ms * 1e-3):,.0f} "
        f"frames/s, mean log-prob of step {spec.steps - 1}: {final:.4f}")
    return dict(workload="configs[0] tiny tanh MLP 40 -> 128 -> 128 -> 50, minibatch 64, ranks 4/8, 10 steps from seed "
                         "(initialisation and a factor update on every step included)",
                value=n * spec.steps / (ms * 1e-3), unit="frames/s", ms_total=ms, steps=spec.steps,
                final_mean_logprob=final)


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
        for t in range(REPLICA_POOL):
            x, y = workloads.minibatch(spec, t, replica=r)
            pool.append((torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda()))
        pools.append(pool)
    torch.cuda.synchronize()

    def steps_on_streams(steps, t0):
        for t in range(t0, t0 + steps):
            for r in range(replicas):
                with torch.cuda.stream(streams[r]):
                    nets[r].step(*pools[r][t % REPLICA_POOL], spec.lr, logps[r])
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


def run_cpu_baseline(max_steps=120, budget_s=16.0, single_thread_budget_s=8.0):
    """The float64 oracle as it stands, timed on the host cores on a bounded sample of the same workload: with the
    BLAS library's default thread count, then with one thread for scale; and the 10 steps of configs[0]."""
    import workloads
    from oracle.network import NGSGDNetwork

    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count() or 1])
    except Exception:
        threadpool_limits = None
        threads = os.cpu_count() or 1
    spec = workloads.c1_pnorm()
    net = NGSGDNetwork(spec.dims, spec.nonlin, workloads.initial_weights(spec), spec.pnorm_group, spec.rank_in,
                       spec.rank_out, spec.alpha, spec.num_samples_history, spec.epsilon, spec.update_period,
                       renorm=True, max_change_per_sample=0.075)
    batches = [workloads.minibatch(spec, t) for t in range(max_steps + 1)]
    net.step(*batches[0], spec.lr)          # state initialisation (eigen-decompositions) is not timed

    def run(budget, first):
        done = 0
        t0 = time.perf_counter()
        while first + done < max_steps and time.perf_counter() - t0 < budget:
            net.step(*batches[first + done + 1], spec.lr)
            done += 1
        return done, time.perf_counter() - t0

    max_steps -= 12                         # keep some minibatches for the single-thread run
    done, elapsed = run(budget_s, 0)
    max_steps += 12
    value = spec.minibatch * done / elapsed
    log(f"[bench] oracle (float64 NumPy, {threads} threads): {done} steps in {elapsed:.1f} s -> {value:,.0f} frames/s")
    out = dict(value=value, unit="frames/s", cores=threads, kind="oracle",
               sample=f"{done} steps of the same workload after 1 untimed initialisation step")
    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            d1, e1 = run(single_thread_budget_s, done)
        if d1 > 0:
            out["single_thread"] = dict(value=spec.minibatch * d1 / e1, unit="frames/s", cores=1,
                                        sample=f"the next {d1} steps with the BLAS library limited to one thread")
            log(f"[bench] oracle, 1 thread: {d1} steps in {e1:.1f} s -> {out['single_thread']['value']:,.0f} frames/s")
    spec0 = workloads.c0_tiny()
    net0 = NGSGDNetwork(spec0.dims, spec0.nonlin, workloads.initial_weights(spec0), spec0.pnorm_group, spec0.rank_in,
                        spec0.rank_out, spec0.alpha, spec0.num_samples_history, spec0.epsilon, spec0.update_period)
    b0 = [workloads.minibatch(spec0, t) for t in range(spec0.steps)]
    t0 = time.perf_counter()
    for x, y in b0:
        net0.step(x, y, spec0.lr)
    e0 = time.perf_counter() - t0
    out["configs0"] = dict(value=spec0.minibatch * spec0.steps / e0, unit="frames/s", cores=threads,
                           sample=f"all {spec0.steps} steps of configs[0], initialisation included")
    log(f"[bench] oracle, configs[0]: {spec0.steps} steps in {e0 * 1e3:.1f} ms -> {out['configs0']['value']:,.0f} frames/s")
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--reps", type=int, default=5, help="repetitions of the timed --steps steps (the median is reported)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-precond", action="store_true")
    ap.add_argument("--no-replicas", action="store_true")
    ap.add_argument("--no-wide", action="store_true", help="skip the configs[3] leg (wider tanh DNN)")
    ap.add_argument("--no-simple", action="store_true", help="skip the simple-method leg (App. A)")
    ap.add_argument("--precond-only", action="store_true",
                    help="run only the preconditioner microbenchmark (BASELINE configs[2]); used for its profile")
    ap.add_argument("--wide-only", action="store_true",
                    help="run only the configs[3] leg (wider tanh DNN); used for its profile")
    ap.add_argument("--simple-only", action="store_true",
                    help="run only the simple-method leg (App. A); used for its profile")
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
    # (the 1 GiB device-to-device copy timed here is also the known-size reference for scaling the FETCH_SIZE /
    # WRITE_SIZE counters of a rocprofv3 --pmc run of this file: it reads 1 GiB and writes 1 GiB)
    peaks = machine_peaks()
    if args.precond_only:
        print(json.dumps({"precondition_roofline": run_precond_bench(), "machine_peaks": peaks}), flush=True)
        return
    if args.wide_only:
        print(json.dumps({"wide_tanh_net": run_wide_bench(), "machine_peaks": peaks}), flush=True)
        return
    if args.simple_only:
        print(json.dumps({"simple_method": run_simple_bench(), "machine_peaks": peaks}), flush=True)
        return
    spec, ms_per_step, frames_per_s, roofline, breakdown, final_logp, timing, step_roofline = run_step_bench(args)
    precond = None if args.no_precond else run_precond_bench()
    tiny = run_c0_bench()
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
            "distinct_minibatches": timing["distinct_minibatches"],
            "final_mean_logprob": final_logp,
        },
        "timing": timing,
        "roofline": roofline,
        "step_roofline": step_roofline,
        "machine_peaks": peaks,
        "cpu_baseline": cpu,
        "precondition_roofline": precond,
        "tiny_tanh_net": tiny,
        "wide_tanh_net": wide,
        "simple_method": simple,
        "replica_interleaving": replica,
        "breakdown": breakdown,
    }
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()

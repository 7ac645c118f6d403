#!/usr/bin/env python3
"""Benchmark of the HALP epoch on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4|c2|c1]

A "step" is one whole outer iteration of Algorithm 4 (full-gradient pass, bit
centering, T inner steps, update of w~) through `halp_epoch` over one batch of
synthetic input.  The default workload is the batched-chains configuration
(R=256 independent linear-regression instances, N=16384, d=512, b=8, T=N): it
is the one both halves of the metric are quoted on (the chip-filling inner loop
and an 8.6 GB HBM-resident gradient pass).  Inputs are generated on the device
and are resident in HBM before the timed region starts.

Prints ONE JSON line.  `value` is int8 feature-updates per second over whole
epochs (R*T*d updates per epoch, gradient pass included in the time).
`roofline` describes the inner-loop kernel (the dominant one; `roofline_chip_filled` the
same kernel with 2048 chains, eight per CU), and
`roofline_full_gradient` the gradient pass of the same epochs; both durations
come from HIP events recorded by the library on the launch stream inside the
timed region.  `roofline.latency` holds the latency floor of that inner loop (one
chain per CU: the step's dependent chain run alone by the library's micro-kernel) and
the share of it the measured loop reaches.  `full_gradient_c5` is the gradient pass
alone on the 16.4 GB logistic configuration (N=1e6, d=4096), with the step rate of that
configuration's minibatch inner loop (B=64, b=16; T=2000 of its 1e6 steps per epoch)
beside it; `side_inner_loops` the inner-loop step rates of the single-chain and the
10-class configurations at reduced step counts (`inner_variant` 2 = register-resident
kernel), `softmax_gradient_pass` the 10-class gradient pass at an HBM-resident row
count.  Every `traffic` field is read from a committed rocprofv3 counter summary
(`traffic_source`), not measured by the run.  `cpu_baseline` is the oracle timed on
the host cores on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
ALU_PEAK_LANEOPS = 256 * 64 * 2.4e9   # 256 CUs x 64 lanes/clk x 2.4 GHz, 32-bit integer lane-ops/s
# algorithmic lane-ops per feature-update at b = 8: 1/4 dot MAC + 1 update
# multiply-add + 4 (add rounding bits, shift, add z, clamp) + 60/16 Philox4x32-10 share
LANEOPS_PER_UPDATE_B8 = 0.25 + 1.0 + 4.0 + 60.0 / 16.0

WORKLOADS = {
    # name: R, N, d, T, alpha, mu, noise
    "c4": dict(R=256, N=16384, d=512, T=16384, alpha=0.1, mu=0.02, noise=0.1),
    # mu of c2: swept with the oracle over 20 epochs (0.01 .. 0.5); 0.3 lowers the loss every epoch
    "c2": dict(R=1, N=100000, d=1024, T=100000, alpha=1e-3, mu=0.3, noise=0.1),
    "c1": dict(R=1, N=1000, d=64, T=2000, alpha=0.01, mu=1.0, noise=0.01),
}


def traffic_source(workload):
    """Where a `traffic` figure of this line comes from: a committed counter summary, not this run."""
    rel = f"profiles/{workload}_hbm_traffic.md"
    return (f"{rel} (rocprofv3 FETCH_SIZE / WRITE_SIZE of an earlier run of this workload, "
            "not measured by this run)") if os.path.exists(os.path.join(ROOT, rel)) else None


def measured_traffic(kernel, workload):
    """HBM bytes per launch from the committed rocprofv3 counter summary, or None."""
    path = os.path.join(ROOT, "profiles", f"{workload}_hbm_traffic.md")
    try:
        for line in open(path):
            t = line.split()
            if len(t) == 4 and t[0] == "traffic_bytes_per_launch" and t[1] == kernel and t[2] == workload:
                return int(t[3])
    except OSError:
        pass
    return None


def make_problem(hp, inp, torch, cfg, seed=0):
    R, N, d = cfg["R"], cfg["N"], cfg["d"]
    share = bool(cfg.get("share_data"))
    Rd = 1 if share else R
    X, y, _ = inp.linreg_chains_device(Rd, N, d, seed=seed, noise=cfg["noise"])
    delta_d = float(X.abs().max().item()) / 127.0
    st = hp.alloc_state(N, d, R=R, b=8)
    Xq = torch.zeros((Rd, N, d), dtype=torch.int8, device="cuda")
    alg = {"lpsvrg": hp.ALG_LPSVRG, "svrg": hp.ALG_SVRG}.get(cfg.get("algorithm"), hp.ALG_HALP)
    h = hp.Halp(N, d, R=R, b=8, T=cfg["T"], alpha=cfg["alpha"], mu=cfg["mu"], delta_d=delta_d,
                seed=seed, share_data=share, algorithm=alg, delta=cfg.get("delta", 0.0))
    h.bind(X=X, Xq=Xq, y=y, **st)
    h.quantize_data()
    torch.cuda.synchronize()
    return h, X, Xq, y, st, delta_d


def cpu_baseline(cfg, X, Xq, y, delta_d, seed, budget_chains):
    """The oracle as it stands on the host cores: whole epochs of sampled chains, one chain per
    thread (ctypes releases the GIL)."""
    from oracle import ref

    R, N, d, T = cfg["R"], cfg["N"], cfg["d"], cfg["T"]
    cores = min(16, os.cpu_count() or 1)
    chains = list(range(0, R, max(1, R // budget_chains)))[:budget_chains]
    src = [0 if cfg.get("share_data") else r for r in chains]
    host = [(X[r].cpu().numpy(), Xq[r].cpu().numpy(), y[r].cpu().numpy()) for r in src]
    ref.lib()

    def one(k):
        r = chains[k]
        prob = ref.make_problem(N, d, b=8, alpha=cfg["alpha"], mu=cfg["mu"], delta_d=delta_d,
                                seed=seed + r)
        return ref.epoch(prob, host[k][0], host[k][1], host[k][2], np.zeros((1, d), np.float32), 0, T)

    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=cores) as ex:
        list(ex.map(one, range(len(chains))))
    dt = time.perf_counter() - t0
    return dict(value=len(chains) * T * d / dt, unit="feature-updates/s", cores=min(cores, len(chains)),
                kind="oracle",
                sample=f"{len(chains)} of the {R} chains, one full epoch each (N={N}, d={d}, T={T}), "
                       f"{dt:.1f} s wall")


def chip_filled_inner_loop(hp, inp, torch, cfg, chains=2048, epochs=3):
    """The inner-loop kernel of the headline workload with 8 chains per CU (the chains share chain
    0's data and differ in their seeds): the throughput-bound figure beside the latency-bound
    one of 256 chains."""
    c = dict(cfg)
    c["R"], c["share_data"] = chains, True
    h, X, Xq, y, st, _ = make_problem(hp, inp, torch, c)
    for k in range(2):
        h.epoch(k)
    h.set_option(hp.OPT_TIMING, 1)
    for k in range(epochs):
        h.epoch(2 + k)
    s = h.get_stats(0)
    upd = chains * c["T"] * c["d"]
    out = dict(chains=chains, ms=s.ms_inner_loop, feature_updates_per_s=upd / (s.ms_inner_loop * 1e-3),
               achieved=upd * LANEOPS_PER_UPDATE_B8 / (s.ms_inner_loop * 1e-3) / 1e12,
               peak=ALU_PEAK_LANEOPS / 1e12, unit="Tlane-op/s",
               frac=upd * LANEOPS_PER_UPDATE_B8 / (s.ms_inner_loop * 1e-3) / ALU_PEAK_LANEOPS,
               steps_per_s_per_chain=c["T"] / (s.ms_inner_loop * 1e-3))
    h.close()
    del X, Xq, y, st
    return out


def step_latency_floor(hp, torch, T, inner_ms, waves=4, steps=65536):
    """The dependent chain of one 8-bit step run alone by the library's micro-kernel, one workgroup
    per CU, and the share of it the measured inner loop reaches.  waves = 4: the several-wave form
    (multiply-adds, DPP fold, one LDS word per wave and a barrier, the fp64 path of gamma, the
    update).  waves = 1: the form with one chain wave (a row of 512 coordinates in four strips per
    lane: packed dots, DPP fold, fp64 path, packed update, one LDS store; records from an LDS
    ring, one barrier per 8 steps)."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    out = torch.empty(cus * waves * 64, dtype=torch.int32, device="cuda")
    hp.debug_step_latency(waves, 8192, cus, out)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    best = None
    for _ in range(3):
        torch.cuda.synchronize()
        e0.record()
        hp.debug_step_latency(waves, steps, cus, out)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        best = ms if best is None else min(best, ms)
    ns = best * 1e6 / steps
    what = ("critical path of a step (dot, DPP fold, LDS word + barrier, fp64 scalar path, update) "
            "measured alone" if waves > 1 else
            "the chain wave's step (packed dots, DPP fold, fp64 scalar path, packed update, LDS store of "
            "the unclamped strips; records from an LDS ring) measured alone")
    return dict(kernel="step_latency_kernel" if waves > 1 else "step_latency_lone_kernel",
                waves_per_chain=waves, chain_ns_per_step=ns,
                bound_ms=ns * T * 1e-6, achieved_ms=inner_ms, frac=ns * T * 1e-6 / inner_ms,
                what=what + "; frac = bound_ms / achieved_ms")


def c2_inner_loop(hp, inp, torch, T=20000):
    """Step rate of the single-chain configuration (N=100000, d=1024, b=8) at a reduced number
    of inner steps per epoch."""
    cfg = dict(WORKLOADS["c2"])
    cfg["T"] = T
    h, X, Xq, y, st, _ = make_problem(hp, inp, torch, cfg)
    h.set_option(hp.OPT_TIMING, 1)
    for k in range(3):
        h.epoch(k)
    s = h.get_stats(0)
    out = dict(N=cfg["N"], d=cfg["d"], K=1, b=8, B=1, T=T, T_of_the_configuration=WORKLOADS["c2"]["T"],
               inner_variant=s.inner_variant, ms_inner_loop=s.ms_inner_loop,
               ms_full_gradient=s.ms_full_gradient, steps_per_s=T / (s.ms_inner_loop * 1e-3),
               feature_updates_per_s=T * cfg["d"] / (s.ms_inner_loop * 1e-3), loss=s.loss)
    h.close()
    del X, Xq, y, st
    return out


def read_ceiling(hp, torch, t, reps=5):
    """GB/s of the library's read-only yardstick kernel over tensor t (each byte read once)."""
    out = torch.empty(2048, dtype=torch.int32, device=t.device)
    for _ in range(2):
        hp.debug_read_bandwidth(t, out)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        hp.debug_read_bandwidth(t, out)
    e1.record()
    torch.cuda.synchronize()
    return t.numel() * t.element_size() / (e0.elapsed_time(e1) / reps * 1e-3) / 1e9


def c5_full_gradient(hp, inp, torch, reps=5):
    """Gradient pass alone on the binary-logistic configuration: N=1e6, d=4096, fp32 (16.4 GB)."""
    N, d = 1_000_000, 4096
    X, y, _ = inp.logistic_device(N, d, seed=0)
    st = hp.alloc_state(N, d, R=1, b=16)
    st["w"].normal_(0.0, 0.1)
    h = hp.Halp(N, d, loss=hp.LOSS_LOGISTIC, b=16, B=64, lam=1e-5)
    h.bind(X=X, y=y, **st)
    for _ in range(2):
        h.full_gradient()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
    ev[0].record()
    for k in range(reps):
        h.full_gradient()
        ev[k + 1].record()
    torch.cuda.synchronize()
    ms = [ev[k].elapsed_time(ev[k + 1]) for k in range(reps)]
    nbytes = N * (4 * d + 4 + 4)
    mean = float(np.mean(ms))
    ceiling = read_ceiling(hp, torch, X)
    out = dict(workload="binary logistic N=1e6 d=4096 fp32 (16.4 GB)", ms=mean, ms_min=float(min(ms)),
               achieved=nbytes / mean / 1e6, peak=HBM_PEAK_GBS, unit="GB/s",
               frac=nbytes / mean / 1e6 / HBM_PEAK_GBS, bytes=nbytes,
               traffic=measured_traffic("fullgrad_k1", "c5"), traffic_source=traffic_source("c5"),
               read_only_kernel_GBs=ceiling,
               frac_of_read_only_kernel=nbytes / mean / 1e6 / ceiling, loss=h.get_stats(0).loss)
    h.close()
    # the same configuration's minibatch inner loop (B=64, b=16) at a reduced step count
    T = 2000
    delta_d = float(X.abs().max().item()) / 32767.0
    Xq = torch.zeros((1, N, d), dtype=torch.int16, device="cuda")
    h = hp.Halp(N, d, loss=hp.LOSS_LOGISTIC, b=16, B=64, T=T, alpha=0.05, mu=0.01, lam=1e-5,
                delta_d=delta_d, seed=0)
    h.bind(X=X, Xq=Xq, y=y, **st)
    h.quantize_data()
    h.set_option(hp.OPT_TIMING, 1)
    for k in range(3):
        h.epoch(k)
    s = h.get_stats(0)
    out["inner_loop"] = dict(B=64, b=16, T=T, inner_variant=s.inner_variant, ms=s.ms_inner_loop,
                             steps_per_s=T / (s.ms_inner_loop * 1e-3),
                             us_per_step=s.ms_inner_loop / T * 1e3,
                             row_bytes_per_step=64 * d * 2,
                             traffic=measured_traffic("inner_batch_kernel", "c5"),
                             traffic_source=traffic_source("c5"),
                             exchange_timeouts=int(st["counters"][:, 3].sum().item()))
    h.close()
    del X, y, st, Xq
    torch.cuda.empty_cache()
    return out


def side_inner_loop(hp, inp, torch, which, T, poll_delay=-1):
    """Inner-loop step rate of the configurations beside the headline one (softmax K=10 at
    b=8/16; logistic with a minibatch of 64 at b=16), at a reduced step count; `inner_variant`
    says which kernel ran (1 general, 2 register-resident)."""
    out = {}
    if which in ("c3", "c3batch"):
        N, d, K = 60000, 784, 10
        X, y, _ = inp.softmax_sparse(N, d, K, seed=0)
        Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
        cases = [dict(b=8, B=1, loss=hp.LOSS_SOFTMAX, lam=1e-4, alpha=1e-2, mu=2.5),
                 dict(b=16, B=1, loss=hp.LOSS_SOFTMAX, lam=1e-4, alpha=1e-2, mu=2.5)]
        if which == "c3batch":  # the same data with 64 rows per step: class-wave kernel, general kernel
            cases = [dict(b=8, B=64, loss=hp.LOSS_SOFTMAX, lam=1e-4, alpha=1e-2, mu=2.5, variant=0),
                     dict(b=16, B=64, loss=hp.LOSS_SOFTMAX, lam=1e-4, alpha=1e-2, mu=2.5, variant=0),
                     dict(b=8, B=64, loss=hp.LOSS_SOFTMAX, lam=1e-4, alpha=1e-2, mu=2.5, variant=1)]
    else:
        N, d, K = 1_000_000, 4096, 1
        Xd, yd, _ = inp.logistic_device(N, d, seed=0)
        cases = [dict(b=16, B=64, loss=hp.LOSS_LOGISTIC, lam=1e-5, alpha=0.05, mu=0.01)]
    for c in cases:
        b = c["b"]
        delta_d = float(Xd.abs().max().item()) / float(2 ** (b - 1) - 1)
        st = hp.alloc_state(N, d, K=K, b=b)
        st["w"].normal_(0.0, 0.01)
        Xq = torch.zeros((1, N, d), dtype=torch.int8 if b == 8 else torch.int16, device="cuda")
        h = hp.Halp(N, d, K=K, loss=c["loss"], b=b, B=c["B"], T=T, alpha=c["alpha"], mu=c["mu"],
                    lam=c["lam"], delta_d=delta_d, seed=0)
        h.bind(X=Xd, Xq=Xq, y=yd, **st)
        h.quantize_data()
        if poll_delay >= 0:
            h.set_option(hp.OPT_EXCHANGE_POLL_DELAY, poll_delay)
        if c.get("variant"):
            h.set_option(hp.OPT_INNER_VARIANT, c["variant"])
        h.set_option(hp.OPT_TIMING, 1)
        for k in range(3):
            h.epoch(k)
        s = h.get_stats(0)
        out[f"{which}_b{b}_B{c['B']}" + ("_general" if c.get("variant") == 1 else "")] = dict(
            N=N, d=d, K=K, b=b, B=c["B"], T=T, inner_variant=s.inner_variant,
            ms_inner_loop=s.ms_inner_loop, ms_full_gradient=s.ms_full_gradient,
            steps_per_s=T / (s.ms_inner_loop * 1e-3),
            feature_updates_per_s=T * d * K / (s.ms_inner_loop * 1e-3),
            full_gradient_GBs=N * (4 * d + 4 * K + 4) / (s.ms_full_gradient * 1e-3) / 1e9,
            loss=s.loss)
        h.close()
        del Xq, st
    return out


def softmax_gradient_pass(hp, torch, rows, reps):
    """The softmax gradient pass alone on a seeded uniform matrix [rows x 784], K=10: the C3
    shape at a row count that can be raised past the last-level cache.  Timed in steady state:
    the first few launches after an idle period run faster than the ones that follow (the
    next five or so slower), so twenty untimed passes come first and at least forty are timed."""
    d, K = 784, 10
    g = torch.Generator(device="cuda")
    g.manual_seed(0)
    X = torch.rand((1, rows, d), device="cuda", generator=g)
    y = torch.randint(0, K, (1, rows), dtype=torch.int32, device="cuda", generator=g)
    st = hp.alloc_state(rows, d, K=K, b=8)
    st["w"].normal_(0.0, 0.01, generator=g)
    Xq = torch.zeros((1, rows, d), dtype=torch.int8, device="cuda")
    h = hp.Halp(rows, d, K=K, loss=hp.LOSS_SOFTMAX, b=8, T=8, alpha=1e-2, mu=2.5, lam=1e-4,
                delta_d=1.0 / 127.0, seed=0)
    h.bind(X=X, Xq=Xq, y=y, **st)
    warm, reps = 20, max(reps, 40)

    def timed():
        for _ in range(warm):
            h.full_gradient()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            h.full_gradient()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    ms = timed()
    loss = h.get_stats(0).loss
    g_halves = st["g"].clone()
    # the same pass with fp32 products, for comparison: time, and how far its gradient lies
    h.set_option(hp.OPT_GRADIENT_FP32, 1)
    ms_fp32 = timed()
    dg = float((st["g"].double() - g_halves.double()).norm() / st["g"].double().norm())
    nbytes = rows * (4 * d + 4 * K + 4)
    out = dict(workload=f"softmax gradient pass, N={rows}, d={d}, K={K}, fp32 data and accumulation, "
                        "products on pairs of halves", passes=reps, warmup_passes=warm, ms=ms, bytes=nbytes,
               achieved=nbytes / (ms * 1e-3) / 1e9, peak=HBM_PEAK_GBS, unit="GB/s",
               frac=nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, loss=loss,
               fp32_products=dict(ms=ms_fp32, frac=nbytes / (ms_fp32 * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                  rel_l2_of_gradients=dg))
    h.close()
    return out


def conditioning_sweep(hp, inp, torch, epochs, T):
    """The conditioning study (appendix "Conditioning Evaluation") as a many-chains workload:
    linear regression 1000 x 64 with Hessian spectrum 1..kappa, `epochs` epochs of T steps, SVRG
    against 16-bit and 8-bit HALP, every (kappa, step size, mu) grid point one chain of a single
    handle per algorithm.  Reports the best final gradient norm per kappa and algorithm, and
    the time of the whole sweep."""
    N, d = 1000, 64
    kappas = [1.0, 10.0, 100.0, 1e3, 1e4, 1e5]
    alphas = [10.0 ** (-k / 2.0) for k in range(3, 15)]          # 3.2e-2 .. 1e-7
    mus = [0.5, 2.0, 8.0, 32.0, 128.0, 512.0, 2000.0]
    data = [inp.linreg_conditioned(N, d, k, seed=1) for k in kappas]
    out = {"N": N, "d": d, "T": T, "epochs": epochs, "kappas": kappas,
           "grid": {"alpha": alphas, "mu": mus}, "runs": {}}
    t_all = 0.0
    for name, alg, b in [("svrg_fp32", hp.ALG_SVRG, 8), ("halp16", hp.ALG_HALP, 16), ("halp8", hp.ALG_HALP, 8)]:
        grid = [(a, m) for a in alphas for m in (mus if alg == hp.ALG_HALP else [1.0])]
        R = len(kappas) * len(grid)
        X = torch.from_numpy(np.stack([data[i][0] for i in range(len(kappas)) for _ in grid])).cuda()
        y = torch.from_numpy(np.stack([data[i][1] for i in range(len(kappas)) for _ in grid])).cuda()
        # one data scale for the handle: the largest entry over all kappas
        delta_d = float(X.abs().max().item()) / float(2 ** (b - 1) - 1)
        st = hp.alloc_state(N, d, R=R, b=b)
        Xq = torch.zeros((R, N, d), dtype=torch.int8 if b == 8 else torch.int16, device="cuda")
        h = hp.Halp(N, d, R=R, b=b, T=T, alpha=1e-3, mu=1.0, delta_d=delta_d, seed=0, algorithm=alg)
        h.bind(X=X, Xq=Xq, y=y, **st)
        h.set_chain_hyper(alpha=[a for _ in kappas for a, _ in grid], mu=[m for _ in kappas for _, m in grid])
        if alg == hp.ALG_HALP:
            h.quantize_data()
        h.full_gradient()
        torch.cuda.synchronize()
        g0 = st["g"].double().reshape(R, -1).norm(dim=1).cpu().numpy()
        t0 = time.perf_counter()
        for k in range(epochs):
            h.epoch(k)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        t_all += dt
        h.full_gradient()
        torch.cuda.synchronize()
        gn = st["g"].double().reshape(R, -1).norm(dim=1).cpu().numpy()
        gn = np.where(np.isfinite(gn), gn, np.inf).reshape(len(kappas), len(grid))
        best = gn.argmin(axis=1)
        out["runs"][name] = {
            "chains": R, "seconds": dt, "inner_variant": h.get_stats(0).inner_variant,
            "feature_updates_per_s": R * T * d * epochs / dt,
            "initial_gradient_norm": [float(g0[i * len(grid)]) for i in range(len(kappas))],
            "best_gradient_norm": [float(gn[i, best[i]]) for i in range(len(kappas))],
            "best_alpha_mu": [list(grid[best[i]]) for i in range(len(kappas))]}
        h.close()
        del X, y, Xq, st
    out["seconds_total"] = t_all
    return out


def clipping_study(hp, inp, torch, epochs):
    """The clipping study (appendix "Clipping Discussion") at the shape of the paper's synthetic
    classification set (10 classes, 10 000 features, N = 7500; seeded stand-in data): 8-bit HALP,
    and 16-bit HALP with the 8-bit run's box ("clip", same mu) or its lattice spacing ("scale",
    mu_16 (2^15-1) = mu_8 (2^7-1)); T = 2N, five seeds each as chains over shared data.  Reports
    the gradient norm before every epoch (mean over seeds).  The fp32 SVRG comparator exists for
    one-class losses only, so this table has no SVRG row; the 100 000-coordinate model runs on the
    general inner-loop kernel."""
    N, d, K, seeds = 7500, 10000, 10, 5
    alpha, mu8, lam = 2.0, 0.1, 1e-4
    X, y, _ = inp.softmax_dense(N, d, K, seed=0)
    Xd, yd = torch.from_numpy(X).cuda()[None], torch.from_numpy(y).cuda()[None]
    runs = [("halp8", 8, mu8), ("halp16_clip", 16, mu8), ("halp16_scale", 16, mu8 * 127.0 / 32767.0)]
    out = {"N": N, "d": d, "K": K, "T": 2 * N, "epochs": epochs, "alpha": alpha, "lambda": lam,
           "mu8": mu8, "seeds": seeds, "runs": {}}
    for name, b, mu in runs:
        delta_d = float(Xd.abs().max().item()) / float(2 ** (b - 1) - 1)
        st = hp.alloc_state(N, d, K=K, R=seeds, b=b)
        Xq = torch.zeros((1, N, d), dtype=torch.int8 if b == 8 else torch.int16, device="cuda")
        h = hp.Halp(N, d, K=K, R=seeds, loss=hp.LOSS_SOFTMAX, b=b, T=2 * N, alpha=alpha, mu=mu, lam=lam,
                    delta_d=delta_d, seed=100, share_data=True)
        h.bind(X=Xd, Xq=Xq, y=yd, **st)
        h.quantize_data()
        gn, loss, clamped = [], [], 0
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(epochs):
            h.epoch(k)
            gn.append(st["g"].double().reshape(seeds, -1).norm(dim=1).mean().item())
            loss.append(st["scales"][:, 6].mean().item())
            clamped += int(st["counters"][:, 0].sum().item())
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        h.full_gradient()
        gn.append(st["g"].double().reshape(seeds, -1).norm(dim=1).mean().item())
        loss.append(st["scales"][:, 6].mean().item())
        out["runs"][name] = {"b": b, "mu": mu, "seconds": dt, "inner_variant": h.get_stats(0).inner_variant,
                             "gradient_norm": gn, "loss": loss, "clamped_coordinates": clamped}
        h.close()
        del st, Xq
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="c4", choices=sorted(WORKLOADS) + ["c3", "c3batch", "c5", "c3grad", "cond", "clip"],
                    help="c4 (default), c2, c1: the headline line; c3, c5: inner-loop step rate "
                         "of the softmax and minibatch configurations; c3grad: the softmax "
                         "gradient pass; cond: the conditioning sweep (5 x --steps epochs); clip: the "
                         "clipping study (2 x --steps epochs)")
    ap.add_argument("--inner-steps", type=int, default=2000, help="T for --workload c3 / c5")
    ap.add_argument("--rows", type=int, default=960000, help="N for --workload c3grad")
    ap.add_argument("--algorithm", default="halp", choices=["halp", "lpsvrg", "svrg"],
                    help="halp (default, Algorithm 4), lpsvrg (Algorithm 2 in integers, fixed "
                         "delta = --delta) or svrg (Algorithm 1, fp32) for the c4 / c2 / c1 "
                         "workloads; the last two are side measurements and skip the oracle timing")
    ap.add_argument("--delta", type=float, default=4.0 / 127.0,
                    help="model scale of --algorithm lpsvrg (teacher weights are N(0,1))")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--no-c5", action="store_true", help="skip the 16 GB gradient-pass measurement")
    ap.add_argument("--poll-delay", type=int, default=-1,
                    help="c5 minibatch loop: 256-cycle sleeps before the first poll of a step's exchange "
                         "(-1: the library's default)")
    ap.add_argument("--no-side", action="store_true",
                    help="skip the step rates of the other configurations' inner loops")
    ap.add_argument("--cpu-chains", type=int, default=64)
    ap.add_argument("--inner-waves", type=int, default=0, help="waves per chain (0 = library's choice)")
    ap.add_argument("--inner-helpers", type=int, default=0, choices=[0, 1, 2, 3],
                    help="helper waves beside the chain waves of the register inner loop: 0 the library's "
                         "choice, 1 wherever built, 2 never")
    ap.add_argument("--chains", type=int, default=0,
                    help="override the number of chains; above the workload's R the chains share "
                         "chain 0's data and differ in their seeds only")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain device copy of X (known size) to calibrate HBM counters")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (every chain and the whole gradient "
                 "pass live on one MI355X); run with --gpus 1")

    import torch

    import halp_inputs as inp
    import paper_1803_03383_amd as hp

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    torch.cuda.set_device(0)
    if args.workload == "c3grad":
        print(json.dumps({"workload": "c3grad",
                          "softmax_gradient_pass": softmax_gradient_pass(hp, torch, args.rows, args.steps)}))
        return
    if args.workload == "clip":
        print(json.dumps({"workload": "clip", "clipping_study":
                          clipping_study(hp, inp, torch, max(args.steps, 1) * 2)}))
        return
    if args.workload == "cond":
        print(json.dumps({"workload": "cond", "conditioning_sweep":
                          conditioning_sweep(hp, inp, torch, max(args.steps, 1) * 5, 1000)}))
        return
    if args.workload in ("c3", "c3batch", "c5"):
        print(json.dumps({"workload": args.workload, "side_inner_loop":
                          side_inner_loop(hp, inp, torch, args.workload, args.inner_steps, args.poll_delay)}))
        return
    cfg = dict(WORKLOADS[args.workload])
    if args.chains > 0 and args.chains != cfg["R"]:
        cfg["share_data"] = args.chains > cfg["R"]
        cfg["R"] = args.chains
    R, N, d, T = cfg["R"], cfg["N"], cfg["d"], cfg["T"]
    if args.algorithm != "halp":
        cfg["algorithm"] = args.algorithm
        if args.algorithm == "lpsvrg":
            cfg["delta"] = args.delta
        args.no_cpu = args.no_c5 = True
    h, X, Xq, y, st, delta_d = make_problem(hp, inp, torch, cfg)
    if args.inner_waves:
        h.set_option(hp.OPT_INNER_WAVES, args.inner_waves)
    if args.inner_helpers:
        h.set_option(hp.OPT_INNER_HELPERS, args.inner_helpers)

    for k in range(args.warmup):
        h.epoch(k)
    torch.cuda.synchronize()
    loss0 = float(st["scales"][:, 6].mean().item()) if args.warmup else None
    h.set_option(hp.OPT_TIMING, 1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        h.epoch(args.warmup + k)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    stats = h.get_stats(0)
    loss1 = float(st["scales"][:, 6].mean().item())
    clamped = int(st["counters"][:, 0].sum().item())

    # counter summaries are only valid for the unmodified workload
    wl_key = args.workload if (args.chains in (0, WORKLOADS[args.workload]["R"])
                               and args.algorithm == "halp") else "none"
    ms_step = dt / args.steps * 1e3
    updates = R * T * d
    value = updates / (ms_step * 1e-3)
    inner_ms, fg_ms = stats.ms_inner_loop, stats.ms_full_gradient
    # fp32 SVRG: one FMA for the dot, one FMA and one subtraction for the update per coordinate
    laneops = 3.0 if args.algorithm == "svrg" else LANEOPS_PER_UPDATE_B8
    # at the headline shape (few chains, four waves each) the register kernel with helper waves runs
    # the library's launch rule at 8 bits, restated: one chain wave + helpers on the other SIMDs for
    # rows of 129 .. 512 coordinates up to two chains per CU (.. 1024 up to one); chain waves with a helper beside each
    # up to five chains per CU; one wave per chain beyond
    lone = (args.algorithm != "svrg" and d <= 1024 and
            (args.inner_helpers == 3 or (args.inner_helpers == 0 and args.inner_waves == 0 and 128 < d
                                         and R <= (2 if d <= 512 else 1) * 256)))
    helped = (not lone and args.algorithm != "svrg" and args.inner_helpers in (0, 1)
              and args.inner_waves in (0, 2, 4) and d <= 1024 and (R <= 5 * 256 or args.inner_helpers == 1))
    inner_kernel = "inner_svrg_kernel" if args.algorithm == "svrg" else (
        "inner_reg_lone_kernel" if lone else ("inner_reg_helped_kernel" if helped else "inner_reg_kernel"))
    alu_achieved = updates * laneops / (inner_ms * 1e-3)
    fg_bytes = (1 if cfg.get("share_data") else R) * N * (4 * d + 4 + 4) + \
        (R * N * 4 if cfg.get("share_data") else 0)
    fg_gbs = fg_bytes / (fg_ms * 1e-3) / 1e9

    out = {
        "metric": "inner-loop int8 feature-updates/sec + full-grad HBM GB/s (fraction of peak)",
        "value": value, "unit": "feature-updates/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8 (inner loop) / f32 (gradient pass)", "data": "synthetic",
        "config": {"workload": f"{args.workload}: R={R} independent linear-regression chains, N={N}, "
                               f"d={d}, b=8, T={T} inner steps per epoch, one step = one halp_epoch",
                   "algorithm": args.algorithm, "delta": cfg.get("delta"),
                   "alpha": cfg["alpha"], "mu": cfg["mu"], "inner_variant": stats.inner_variant, "inner_waves": args.inner_waves,
                   "share_data": bool(cfg.get("share_data")),
                   "timed_epochs": stats.timed_epochs},
        "roofline": {"kernel": inner_kernel, "bound": "alu", "achieved": alu_achieved / 1e12,
                     "peak": ALU_PEAK_LANEOPS / 1e12, "unit": "Tlane-op/s",
                     "frac": alu_achieved / ALU_PEAK_LANEOPS,
                     "traffic": measured_traffic(inner_kernel, wl_key),
                     "traffic_source": traffic_source(wl_key),
                     "ms": inner_ms, "feature_updates_per_s": updates / (inner_ms * 1e-3),
                     "steps_per_s_per_chain": T / (inner_ms * 1e-3)},
        "roofline_full_gradient": {"kernel": "fullgrad_k1", "bound": "hbm", "achieved": fg_gbs,
                                   "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": fg_gbs / HBM_PEAK_GBS,
                                   "traffic": measured_traffic("fullgrad_k1", wl_key),
                                   "traffic_source": traffic_source(wl_key), "ms": fg_ms, "bytes": fg_bytes},
        "ms_recenter": stats.ms_recenter,
        "loss_first_timed": loss0, "loss_last": loss1, "clamped_coordinates_last_epoch": clamped,
        "paper_context": "paper reports HALP up to 4x faster per epoch than its AVX2 fp64 SVRG on 56 "
                         "Xeon E7-4850 v3 cores (Table 3); no GPU or bandwidth figure is published",
    }
    if args.algorithm == "halp" and args.workload == "c4" and args.chains in (0, WORKLOADS["c4"]["R"]):
        out["roofline"]["latency"] = step_latency_floor(hp, torch, T, inner_ms, waves=1 if lone else 4)
    if args.algorithm == "halp":  # the same matrix through a kernel that only reads
        ceiling = read_ceiling(hp, torch, X)
        out["roofline_full_gradient"]["read_only_kernel_GBs"] = ceiling
        out["roofline_full_gradient"]["frac_of_read_only_kernel"] = fg_gbs / ceiling
    if args.copy_probe:  # read R*N*d*4 bytes, write as many: the yardstick for FETCH_SIZE / WRITE_SIZE
        Y = torch.empty_like(X)
        Y.copy_(X)
        torch.cuda.synchronize()
        out["copy_probe_bytes_each_way"] = X.numel() * 4
        del Y
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(cfg, X, Xq, y, delta_d, 0, min(args.cpu_chains, R))
    h.close()
    del h, X, Xq, y, st
    torch.cuda.empty_cache()
    if args.algorithm == "halp" and args.workload == "c4" and args.chains in (0, WORKLOADS["c4"]["R"]):
        out["roofline_chip_filled"] = chip_filled_inner_loop(hp, inp, torch, WORKLOADS["c4"])
    if not args.no_side and args.algorithm == "halp" and args.workload == "c4":
        # the other configurations' inner loops (reduced step counts) and the softmax gradient pass
        side = {"c2_b8_B1": c2_inner_loop(hp, inp, torch)}
        side.update(side_inner_loop(hp, inp, torch, "c3", 2000))
        out["side_inner_loops"] = side
        out["softmax_gradient_pass"] = softmax_gradient_pass(hp, torch, 960000, 10)
    if not args.no_c5:
        out["full_gradient_c5"] = c5_full_gradient(hp, inp, torch)
    print(json.dumps(out))


if __name__ == "__main__":
    main()

#!/usr/bin/env python3
"""Benchmark of the speculative-sampling hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c1..c5] [--stages]

A *step* is one complete pass of the sampler over the batch of the chosen workload: every chain
is initialised and taken from step 0 to step T through windows of [window-start prediction ->
draft rollout -> batched target evaluation of all drafted states -> accept / first-reject /
reflect -> advance + compaction].  All inputs (schedule, denoiser parameters, chain ids) are
resident in HBM before the timed region.  The metric is verified diffusion steps per second,
B*T*steps / time.  One JSON line is printed; it also carries

* ``roofline``      the dominant kernel of the workload: algorithmic bytes / flops per launch over
                    its mean launch duration measured with HIP events inside the timed region;
* ``cpu_baseline``  the fp64 oracle (``oracle/``) timed on the host on a bounded sample of the
                    same workload -- a reported baseline, not a target;
* ``mean_accepted_draft_length`` and the per-window counters.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

DEFAULT_WORKLOAD = "c4"

DESCRIPTIONS = {
    "c1": "c1: toy DDPM d=2, 64 chains, ring GMM posterior mean, linear beta T=100, K=4",
    "c2": "c2: GMM DDPM d=64, 4096 chains, 32-component posterior mean, cosine T=200, K=8",
    "c3": "c3: linear-Gaussian DDPM d=3072, 2048 chains, rank-256 Woodbury denoiser (fp32 MFMA), cosine T=250, K=10",
    "c4": "c4: MLP DDPM d=12288, 512 chains, 3-layer width-4096 SiLU MLP (bf16 MFMA), linear T=500, K=16",
    "c5": "c5: speculative ULA d=1000, 16384 chains, 16-component GMM score, gamma=1e-2, T=2000, K=16",
    "phi4": "phi4: speculative ULA on the phi^4 lattice energy, 8x8 periodic grid, beta=100, gamma=1e-3, 16384 chains, T=2000, K=20",
}

# HBM bytes per launch of the roofline kernel (fetched * 2.0 + written * 1.0 of the rocprofv3 FETCH_SIZE /
# WRITE_SIZE counters, the factors being what the same counters read for a plain device copy), taken from
# profiles/hbm_traffic_all_kernels_c4.md and _c3.md (mean over the launches of a pass); workloads without such a
# counter run report null
MEASURED_TRAFFIC_BYTES = {"c4": 1225.1e6, "c3": 277.8e6}

# published MI355X peaks used as roofline denominators
PEAK = {"hbm": (8000.0, "GB/s"), "mfma_bf16": (2500.0, "TFLOP/s"), "mfma_fp32": (157.3, "TFLOP/s"),
        "alu_fp64": (78.6, "TFLOP/s"), "alu_fp32": (157.3, "TFLOP/s"),
        # vector instruction issue: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-instructions per second (the fp32
        # figure is this times 2 for the FMA and 2 for the packed form)
        "alu_lane": (39.3, "T four-cycle lane-op/s")}


def roofline_plan(cfg):
    """Which kernel is reported for a workload, how it is timed and its algorithmic work.

    Returns dict(kernel, stage or den_which, bound, peak key, work(counters) -> total units)."""
    d, K = cfg.d, cfg.K
    if cfg.kind == "mlp":
        H = cfg.params.H
        # the batched evaluation of the drafted states (rows = sum Kt - chain-windows); the window-start
        # call (one row per chain, a smaller tile) is left out of this figure
        return dict(kernel="mlpgemm::kernel_pp<EPI=1,GATHER> (256x256x64 tiles, 8 waves in two alternating groups, 16x16x32 bf16 MFMA) "
                           "layer-1 GEMM of the batched target call, rows x 12288 -> 4096, A rows gathered from the bf16 image "
                           "of the drafts (largest share of the kernel time; layer 3 has the same flops)",
                    den_which=1, den_min_rows=cfg.B + 1, bound="mfma", peak="mfma_bf16", scale=1e-12,
                    work=lambda c: 2.0 * (c[4] - c[1]) * d * H)
    if cfg.kind == "lowrank":
        rpad = -(-cfg.params.U.shape[1] // 16) * 16
        return dict(kernel="lrgemm::kernel<64,128,1,4,STAGE=2,NS=2> (P' Q^T + epilogue, fp32 MFMA) of the batched target call", den_which=2,
                    den_min_rows=cfg.B + 1, bound="mfma", peak="mfma_fp32", scale=1e-12,
                    work=lambda c: 2.0 * (c[4] - c[1]) * d * rpad)
    if cfg.kind == "gmm":
        # the analytic denoiser bounds these windows (about 3/4 of the kernel time).  fp64 flops per
        # (component, coordinate) pair: variance 3, reciprocal counted as 1, x - sqrt(ab) mu 2, quadratic form 3,
        # gain 2, component mean 2, weighting and the sum over components 2
        M = cfg.params.means.shape[0]
        return dict(kernel="gmm_posterior_mean_reg_kernel (mixture posterior mean, fp64) of the batched target call", den_which=1,
                    den_min_rows=cfg.B + 1, bound="alu", peak="alu_fp64", scale=1e-12,
                    work=lambda c: 15.0 * M * d * (c[4] - c[1]))
    if cfg.kind == "langevin":
        M = cfg.params.means.shape[0]
        # fp64 flops per evaluated position: logits 3 M d, gradient 2 M d + 2 d, Delta / dots / update 12 d
        return dict(kernel="langevin_window_wave_kernel<4> (fused draft + score + verify, one wavefront per chain; with --loop fused "
                           "its run form: every chain's windows back to back in one launch)", stage="langevin_window",
                    bound="alu", peak="alu_fp64", scale=1e-12,
                    work=lambda c: float(c[0] + c[1]) * d * (5.0 * M + 14.0))
    if cfg.kind == "phi4":
        # Vector work per site and evaluated position, in units of one four-cycle wavefront instruction per lane
        # (the rate of fp64 arithmetic, conversions and 32-bit multiplies: 16 lanes per clock and SIMD; plain 32-bit
        # operations cost half a unit, v_mad_u64_u32 1.75, transcendentals 2).  Per lane and position (4 sites):
        # Philox4x32-10 55 (20 wide multiplies, 40 xor / add), Box-Muller for 4 normals 25, their conversion to
        # fp64 4, stencil gradient 36, Delta and the two dot products 18, their reduction over the chain's lanes 25,
        # update 9, accept test 8: 180 per lane, 45 per site.
        return dict(kernel="phi4_window_kernel<16> (fused draft + stencil gradient + verify, 16 lanes per chain; with --loop fused "
                           "phi4_run_kernel<16>: every chain's windows back to back in one launch)",
                    stage="langevin_window", bound="alu", peak="alu_lane", scale=1e-12,
                    work=lambda c: float(c[0] + c[1]) * d * 45.0)
    raise ValueError(cfg.kind)


def _sampler(cfg, drafter):
    import workloads as W
    from paper_2501_05370_amd.runner import make_sampler
    if drafter == "independent":
        return make_sampler(cfg, drafter="independent", draft_params=W.draft_params(cfg))
    return make_sampler(cfg, drafter=drafter)


def run_gpu(cfg, steps, warmup, stages, drafter="frozen", loop="eager", wps=1, verify_shape=0, gemm_variant=0):
    import torch
    from paper_2501_05370_amd.runner import make_sampler
    from paper_2501_05370_amd.sampler import StageTimer

    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU (the HIP library has no CPU fallback)")
    torch.cuda.set_device(0)
    smp = _sampler(cfg, drafter)
    if verify_shape:
        smp.ctx.sd_set_verify_shape(verify_shape)
    if gemm_variant:
        smp.den.sdden_mlp_select_gemm(gemm_variant)
    ids = torch.arange(cfg.B, dtype=torch.int64, device="cuda")
    plan = roofline_plan(cfg)
    run_kw = {} if loop in ("eager", "fused") else dict(windows_per_sync=wps, graph=(loop == "graph"))
    run = smp.run_fused if loop == "fused" else smp.run
    if loop == "fused":
        plan = dict(plan, stage="langevin_run")
    for w in range(warmup):
        smp.ctx.sd_set_seed(cfg.seed + 1000 + w)
        run(ids, **run_kw)
    torch.cuda.synchronize()

    den = getattr(smp, "den", None)
    events_in_loop = loop in ("eager", "fused")   # per-stage events cannot be recorded into replayed graphs
    if events_in_loop:
        if stages:
            smp.timer = StageTimer()
        elif "stage" in plan:
            smp.timer = StageTimer([plan["stage"]])
        if "den_which" in plan:
            den.sdden_profile_min_rows(plan.get("den_min_rows", 0))
            den.sdden_profile(plan["den_which"])
    smp.buf.counters.zero_()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(steps):
        smp.ctx.sd_set_seed(cfg.seed + s)
        run(ids, reset_counters=False, **run_kw)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    counters = smp.buf.counters.tolist()
    timed_note = None
    if not events_in_loop:
        # the roofline kernel (and the stage table) are timed in one more pass of the plain loop with the
        # same seed: same kernels on the same data, HIP events on the launch stream
        timed_note = "separate eager pass after the timed region (the timed passes replay HIP graphs / launch several windows per readback)"
        smp.timer = StageTimer() if stages else (StageTimer([plan["stage"]]) if "stage" in plan else smp.timer)
        if "den_which" in plan:
            den.sdden_profile_min_rows(plan.get("den_min_rows", 0))
            den.sdden_profile(plan["den_which"])
        smp.ctx.sd_set_seed(cfg.seed)
        _, counters_roof = smp.run(ids)
    else:
        counters_roof = counters
    timed = smp.timer.collect() if hasattr(smp.timer, "collect") else {}
    if "den_which" in plan:
        k_ms, k_launches = den.sdden_profile_collect()
        den.sdden_profile(0)
        den.sdden_profile_min_rows(0)
    else:
        k_ms, k_launches, _ = timed[plan["stage"]]
    cw = list(counters_roof)
    if drafter.startswith("efficient_frozen") and "den_which" in plan:
        # one call per window on the start state and all drafts but a chain's final state:
        # rows = chain-windows + sum Kt - chains finished; expressed through the counters the plan uses
        cw[4] = cw[4] + 2 * cw[1] - cfg.B * (steps if events_in_loop else 1)
    work = plan["work"](cw)
    peak, unit = PEAK[plan["peak"]]
    achieved = work * plan["scale"] / (k_ms * 1e-3) if k_ms > 0 else 0.0
    roofline = {"kernel": plan["kernel"], "bound": plan["bound"], "achieved": round(achieved, 3), "peak": peak,
                "unit": unit, "frac": round(achieved / peak, 5), "traffic": MEASURED_TRAFFIC_BYTES.get(cfg.name),
                "avg_launch_us": round(1e3 * k_ms / max(1, k_launches), 3), "launches": k_launches,
                "work_per_launch": work / max(1, k_launches)}
    if timed_note:
        roofline["timed_in"] = timed_note
    if cfg.kind == "langevin":
        # The algorithmic count prices the weighted mean over all M components (2 M d of the 5 M d); the kernel skips
        # components whose responsibility is below 1e-25, which changes nothing to fp64 rounding.  Live components
        # are counted here on the final states of the run (this well-separated mixture leaves one or two).
        M = cfg.params.means.shape[0]
        x = smp.buf.y_out[:min(cfg.B, 2048)].double()
        mu = torch.as_tensor(cfg.params.means, dtype=torch.float64, device=x.device)
        s2 = float(cfg.params.stds[0, 0]) ** 2
        logit = torch.as_tensor(cfg.params.logw, dtype=torch.float64, device=x.device)[None, :] - torch.cdist(x, mu) ** 2 / (2 * s2)
        live = float((torch.softmax(logit, dim=1) > 1e-25).sum(dim=1).double().mean().item())
        executed = (3.0 * M + 2.0 * live + 14.0) / (5.0 * M + 14.0)
        roofline["executed"] = {"live_components_of_%d" % M: round(live, 2), "achieved": round(achieved * executed, 3),
                                "frac": round(achieved * executed / peak, 5),
                                "note": "flops the kernel executes: the weighted mean runs over the live components only"}
    stage_table = {k: {"ms_total": round(v[0], 3), "launches": v[1], "us_per_launch": round(1e3 * v[0] / max(1, v[1]), 2)}
                   for k, v in timed.items()} if stages else None
    return elapsed, counters, roofline, stage_table


def run_context(cfg, drafter="frozen"):
    """Untimed extras around the headline figure: the acceptance rate per window position (one more
    sampler pass with a per-window tally), the target calls per chain step in the paper's sense (one
    call = one batched evaluation, whatever its row count) and the plain sequential chain on the same
    GPU (the same sampler with a window of one step, which accepts trivially)."""
    import torch
    import workloads as W
    from paper_2501_05370_amd.runner import make_sampler

    K, T = cfg.K, cfg.T
    smp = _sampler(cfg, drafter)
    b = smp.buf
    ids = torch.arange(cfg.B, dtype=torch.int64, device="cuda")
    smp.ctx.sd_set_seed(cfg.seed)
    B = smp.start(ids, True)
    j = torch.arange(1, K + 1, device="cuda")
    reached = torch.zeros(K, dtype=torch.int64, device="cuda")
    accepted = torch.zeros(K, dtype=torch.int64, device="cuda")
    windows = 0
    while B > 0:
        n0 = b.n[:B].clone()
        smp.window(B)
        Kt = torch.clamp(T - n0, max=K).to(torch.int64)
        nacc = (b.adv[:B].to(torch.int64) - b.rejected[:B].to(torch.int64))[:, None]   # accepted drafts
        r = (Kt[:, None] >= j) & (nacc >= j - 1)
        reached += r.sum(0)
        accepted += (r & (nacc >= j)).sum(0)
        smp.advance(B)
        B = int(b.B_active.item())
        windows += 1
    rate = (accepted.double() / reached.clamp(min=1).double()).tolist()
    calls = windows * (2 if (cfg.kind not in ("langevin", "phi4") and K > 1 and not drafter.startswith("efficient_frozen")) else 1)
    calls += 1 if drafter.startswith("efficient_frozen") else 0
    out = {"acceptance_rate_by_position": [round(x, 4) for x in rate],
           "target_calls_per_pass": calls, "chain_steps_per_target_call": round(T / calls, 3)}
    del smp
    seq_cfg = W.make_config(cfg.name, K=1)
    seq = make_sampler(seq_cfg)
    seq.ctx.sd_set_seed(cfg.seed)
    seq.run(ids)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    seq.ctx.sd_set_seed(cfg.seed + 1)
    _, c = seq.run(ids)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    out["sequential_gpu"] = {"value": round(c[0] / dt, 1), "unit": "diffusion steps/s", "ms_per_pass": round(1e3 * dt, 3),
                             "target_calls_per_pass": c[3],
                             "note": "same kernels with a window of one step: T sequential target calls per chain"}
    return out


_ORACLE = {}          # what the oracle workers need, built once in the parent (forked workers share it copy-on-write)


def _oracle_setup(cfg, drafter):
    import workloads as W
    from oracle import langevin as L
    from oracle.denoisers import GMMDenoiser, GMMScore, LowRankDenoiser, MLPDenoiser
    sched = cfg.schedule
    if cfg.kind == "gmm":
        D = GMMDenoiser(cfg.params, sched.alpha_bar_state)
    elif cfg.kind == "lowrank":
        D = LowRankDenoiser(cfg.params, sched.alpha_bar_state)
    elif cfg.kind == "mlp":
        D = MLPDenoiser(cfg.params)
    elif cfg.kind == "phi4":
        D = L.Phi4Energy(cfg.params.L, cfg.params.beta)
    else:
        D = GMMScore(cfg.params)
    kw = {}
    if drafter == "independent":
        dp = W.draft_params(cfg)
        Dd = {"gmm": lambda: GMMDenoiser(dp, sched.alpha_bar_state), "lowrank": lambda: LowRankDenoiser(dp, sched.alpha_bar_state),
              "mlp": lambda: MLPDenoiser(dp)}[cfg.kind]()
        kw = dict(drafter="independent", D_draft=Dd)
    _ORACLE.update(cfg=cfg, D=D, kw=kw, drafter=drafter)


def _oracle_share(job):
    """The oracle on chains first .. first + nchains - 1 of the workload, window by window, for budget_s seconds of
    wall time or until they finish (then again with the next seed).  One BLAS thread: the cores are used by running
    several of these at once.  Returns (verified steps, windows, passes, seconds)."""
    first, nchains, budget_s = job
    from threadpoolctl import threadpool_limits
    from oracle import langevin as L
    from oracle import philox
    from oracle import speculative as S
    cfg, D, kw, drafter = _ORACLE["cfg"], _ORACLE["D"], _ORACLE["kw"], _ORACLE["drafter"]
    sched = cfg.schedule
    ids0 = np.arange(first, first + nchains, dtype=np.int64)
    out = np.zeros((first + nchains, cfg.d))
    steps_done = windows = runs = 0
    seed = cfg.seed
    with threadpool_limits(limits=1):
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < budget_s:
            # a fresh pass over the sampled chains (small workloads finish several within the budget)
            ids = ids0
            y = philox.initial_state(seed, ids, cfg.d)
            n = np.zeros(nchains, dtype=np.int64)
            runs += 1
            Dfz = D(y, n) if drafter.startswith("efficient_frozen") else None
            while n.size and time.perf_counter() - t0 < budget_s:
                if drafter.startswith("efficient_frozen"):
                    res, _, _, _, Dnext = S.window_efficient(sched, D, y, n, ids, Dfz, cfg.K, seed,
                                                             carry="last_accepted" if drafter.endswith("last_accepted") else "draft")
                    y_out, adv = res.y_out, res.adv
                    Dfz = Dnext[n + adv < cfg.T]
                elif cfg.kind in ("langevin", "phi4"):
                    y_out, adv, _, _, _ = L.ula_window(D, y, n, ids, cfg.K, cfg.T, cfg.gamma, seed)
                else:
                    res, *_ = S.window(sched, D, y, n, ids, cfg.K, seed, **kw)
                    y_out, adv = res.y_out, res.adv
                steps_done += int(adv.sum())
                windows += 1
                y, n, ids = S.advance(cfg.T, y_out, adv, n, ids, out)
            seed += 1
        dt = time.perf_counter() - t0
    return steps_done, windows, runs, dt


def cpu_baseline(cfg, budget_s=10.0, drafter="frozen"):
    """The oracle timed on the host on a bounded sample of the workload, twice: on one core, and with the chains
    split over all the cores this process may use (one single-threaded worker process per core, at most 16).
    Must run before anything initialises the GPU: the workers are forked."""
    import multiprocessing as mp
    nchains = {"c1": 64, "c2": 256, "c3": 16, "c4": 4, "c5": 16, "phi4": 256}[cfg.name]
    nchains = min(nchains, cfg.B)
    _oracle_setup(cfg, drafter)
    s1, w1, r1, dt1 = _oracle_share((0, nchains, budget_s))
    cores = max(1, min(16, len(os.sched_getaffinity(0))))
    per = max(1, min(nchains, cfg.B // cores))
    jobs = [(c * per, per, budget_s) for c in range(cores)]
    t0 = time.perf_counter()
    with mp.get_context("fork").Pool(cores) as pool:
        parts = pool.map(_oracle_share, jobs)
    wall = time.perf_counter() - t0
    sp = sum(q[0] for q in parts)
    unit = "verified diffusion steps/s"
    return {"value": round(sp / wall, 3), "unit": unit, "cores": cores, "kind": "oracle",
            "sample": f"{cores} worker processes (one BLAS thread each) x {per} chains of {cfg.B}, "
                      f"{sum(q[1] for q in parts)} windows from step 0 ({sp} verified steps in {wall:.1f} s of wall time, "
                      f"process start-up included; numpy fp64)",
            "one_core": {"value": round(s1 / dt1, 3), "unit": unit, "cores": 1,
                         "sample": f"{nchains} of {cfg.B} chains, {w1} windows in {r1} pass(es) from step 0 "
                                   f"({s1} verified steps in {dt1:.1f} s; numpy fp64, one thread)"}}


def kernel_gemm(iters=20, rows_per_chain_masked=1, variants=None):
    """The three GEMMs of the c4 batched target call in isolation, back to back on fixed data: rows = the
    B*(K-1) drafted states a full window evaluates (the last draft of every chain is masked, as in the sampler),
    bf16 image supplied, each layer timed with HIP events on the launch stream by the library's profiling
    hooks.  One JSON line per kernel variant (sdden_mlp_select_gemm)."""
    import torch
    import workloads as W
    from paper_2501_05370_amd.runner import make_denoiser
    torch.cuda.set_device(0)
    cfg = W.make_config("c4")
    B, K, d, H = cfg.B, cfg.K, cfg.d, cfg.params.H
    R = B * K
    den = make_denoiser(cfg, R)
    g = torch.Generator(device="cuda").manual_seed(0)
    X = torch.randn(R, d, device="cuda", generator=g)
    Xb = X.to(torch.bfloat16).view(torch.int16).contiguous()
    krow = torch.randint(0, cfg.T, (B, K), device="cuda", generator=g, dtype=torch.int32)
    krow[:, K - rows_per_chain_masked:] = -1
    rows = int((krow >= 0).sum().item())
    out = torch.zeros(R + 1, d, device="cuda")
    flops = {1: 2.0 * rows * d * H, 2: 2.0 * rows * H * H, 3: 2.0 * rows * H * d}
    ref = None
    names = {0: "kernel_pp", 1: "kernel_hs", 2: "kernel_pp without fragment reads (timing only)",
             3: "kernel_pp without direct loads (timing only)", 4: "kernel_pp, MFMAs and barriers only (timing only)", 5: "kernel_pp without the B fragment reads (timing only)"}
    vs = [(v, names[v]) for v in (variants or [0, 1, 2, 3, 4, 5])]
    for variant, name in vs:
        den.sdden_mlp_select_gemm(variant)
        for _ in range(2):
            den.sdden_eval_mirror(R, X, Xb, krow.view(-1), out[1:])
        torch.cuda.synchronize()
        if ref is None:
            ref = out.clone()
        layers = {"max_abs_diff_vs_first_variant": float((out - ref).abs().max().item())}
        for which in (1, 2, 3):
            den.sdden_profile(which)
            for _ in range(iters):
                den.sdden_eval_mirror(R, X, Xb, krow.view(-1), out[1:])
            ms, n = den.sdden_profile_collect()
            den.sdden_profile(0)
            us = 1e3 * ms / max(1, n)
            layers[f"layer{which}"] = {"avg_launch_us": round(us, 2), "launches": n,
                                       "PFLOP/s": round(flops[which] / (us * 1e-6) * 1e-15, 4),
                                       "frac_of_2.5": round(flops[which] / (us * 1e-6) * 1e-15 / 2.5, 4)}
        print(json.dumps({"kernel": "mlp_gemm", "variant": name, "rows": rows, "d": d, "H": H,
                          "note": "back-to-back launches of the three layers on fixed data", **layers}), flush=True)


def kernel_verify(workload, accept, shapes, iters=20):
    """The accept / first-reject / reflect kernel alone, at the batch size of a workload, on inputs whose first
    rejection is planted: `all` = every draft accepted (prediction rows equal the window-start prediction, so
    Delta = 0), `second` = every chain rejects its second draft, `tail` = the same except that one chain in 32 accepts
    everything (the launch then lasts as long as a lone chain's dependent steps), `mixed` = the first rejection of a chain is
    geometric with per-position acceptance 0.55 (the shape the c4 sampler shows after its first windows).  Reports,
    per launch shape, the mean launch time and the rate of the bytes the method needs (rows up to the first
    rejection, the four rows of the reflection, the state written) and of the rows the group schedule streams."""
    import torch
    import workloads as W
    from paper_2501_05370_amd.runner import make_context
    torch.cuda.set_device(0)
    cfg = W.make_config(workload)
    B, K, d, T = cfg.B, cfg.K, cfg.d, cfg.T
    ctx = make_context(cfg)
    g = torch.Generator(device="cuda").manual_seed(0)
    y = torch.randn(B, d, device="cuda", generator=g)
    D0 = torch.randn(B, d, device="cuda", generator=g)
    Ytil = torch.randn(B, K, d, device="cuda", generator=g)
    Dq = D0[:, None, :].repeat(1, K, 1).contiguous()                  # Delta = 0 everywhere: accepted
    n = torch.full((B,), T // 2, dtype=torch.int32, device="cuda")
    ids = torch.arange(B, dtype=torch.int64, device="cuda")
    if accept == "all":
        jr = torch.full((B,), K, dtype=torch.int64)                    # K = no rejection
    elif accept == "second":
        jr = torch.ones(B, dtype=torch.int64)
    elif accept == "tail":
        jr = torch.ones(B, dtype=torch.int64)
        jr[::32] = K                                                   # one chain in 32 accepts every draft
    else:
        rng = np.random.default_rng(0)
        jr = torch.as_tensor(np.minimum(K, 1 + rng.geometric(0.45, size=B) - 1 + 0), dtype=torch.int64)
        jr = torch.clamp(jr, min=1)                                    # the first draft of a frozen window is exact
    rows = torch.arange(B)
    rej = jr < K
    Dq[rows[rej], jr[rej]] += 1.0e3                                    # a draft mean this far off is rejected
    y_out = torch.zeros(B, d, device="cuda")
    adv = torch.zeros(B, dtype=torch.int32, device="cuda")
    rejected = torch.zeros(B, dtype=torch.uint8, device="cuda")
    row = 4.0 * d
    jrn = jr.numpy().astype(np.float64)
    # rows the method needs: y, D0, drafts 0..jr, predictions 1..jr; then the reflection re-reads three and
    # writes one (a fully accepted window copies its last draft: one read, one write)
    need = np.where(jrn < K, (2 * jrn + 3) + 4, (2 * K + 1) + 2).sum() * row
    for shape in shapes:
        ctx.sd_set_verify_shape(shape)
        for _ in range(3):
            ctx.sd_verify(B, y, n, ids, D0, Dq, Ytil, y_out, adv, rejected)
        torch.cuda.synchronize()
        got = adv.cpu().numpy()
        assert np.array_equal(got, np.where(jrn < K, jrn + 1, K).astype(np.int32)), "planted first rejections not found"
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            ctx.sd_verify(B, y, n, ids, D0, Dq, Ytil, y_out, adv, rejected)
        e1.record()
        torch.cuda.synchronize()
        us = 1e3 * e0.elapsed_time(e1) / iters
        print(json.dumps({"kernel": "verify_kernel", "workload": workload, "accept": accept, "shape": shape,
                          "chains": B, "d": d, "K": K, "mean_advance": float(np.where(jrn < K, jrn + 1, K).mean()),
                          "avg_launch_us": round(us, 2), "needed_bytes_per_launch": need,
                          "needed_TB/s": round(need / (us * 1e-6) * 1e-12, 3),
                          "frac_of_8_TB/s": round(need / (us * 1e-6) * 1e-12 / 8.0, 4),
                          "note": "back-to-back launches on fixed data (event bracket over all launches)"}), flush=True)


def _time_launches(fn, iters, warm=3):
    """Mean duration in microseconds of `iters` back-to-back calls of fn (events on the launch stream)."""
    import torch
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return 1e3 * e0.elapsed_time(e1) / iters


def kernel_stream(iters=20):
    """What a plain hand-written streaming kernel reaches on this chip (sd_measure_stream): copy, read and fill
    of buffers the size of the c4 window arrays (403 MB) and of 1 GiB."""
    import torch
    from paper_2501_05370_amd import binding
    torch.cuda.set_device(0)
    for nbytes in (512 * 16 * 12288 * 4, 49152 * 21845):         # the c4 window arrays (403 MB); 1 GiB in whole rows
        src = torch.ones(nbytes // 4, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for mode, name, moved in ((0, "copy", 2 * nbytes), (1, "read", nbytes), (2, "fill", nbytes),
                                  (3, "copy, row per workgroup", 2 * nbytes), (4, "read, row per workgroup", nbytes),
                                  (5, "fill, row per workgroup", nbytes)):
            us = _time_launches(lambda: binding.sd_measure_stream(src, dst, nbytes, mode), iters)
            print(json.dumps({"kernel": "stream_kernel", "mode": name, "buffer_bytes": nbytes, "bytes_moved": moved,
                              "avg_launch_us": round(us, 2), "TB/s": round(moved / (us * 1e-6) * 1e-12, 3),
                              "frac_of_8_TB/s": round(moved / (us * 1e-6) * 1e-12 / 8.0, 4)}), flush=True)
        del src, dst


def kernel_mfma(iters=20):
    """What a loop of nothing but MFMAs on register operands sustains (sd_measure_mfma): the matrix cores under
    the chip's power management, with no operand traffic at all."""
    import torch
    from paper_2501_05370_amd import binding
    torch.cuda.set_device(0)
    sink = torch.zeros(4096, dtype=torch.float32, device="cuda")
    for shape, name in ((0, "v_mfma_f32_32x32x16_bf16"), (1, "v_mfma_f32_16x16x32_bf16")):
        rounds = 20000
        flops = binding.sd_measure_mfma(shape, rounds, sink)
        us = _time_launches(lambda: binding.sd_measure_mfma(shape, rounds, sink), iters)
        print(json.dumps({"kernel": "mfma_kernel", "instruction": name, "workgroups": "one of 512 threads per CU",
                          "rounds_of_16_mfma": rounds, "avg_launch_us": round(us, 2),
                          "PFLOP/s": round(flops / (us * 1e-6) * 1e-15, 4),
                          "frac_of_2.5": round(flops / (us * 1e-6) * 1e-15 / 2.5, 4)}), flush=True)


def kernel_draft(workload, iters=20):
    """The frozen draft rollout alone at the batch size of a workload (all chains mid-run, full windows): bytes
    written per launch (fp32 drafts, plus their bf16 image where the target network reads bf16) over its time."""
    import torch
    import workloads as W
    from paper_2501_05370_amd.runner import make_context
    torch.cuda.set_device(0)
    cfg = W.make_config(workload)
    B, K, d, T = cfg.B, cfg.K, cfg.d, cfg.T
    ctx = make_context(cfg)
    g = torch.Generator(device="cuda").manual_seed(0)
    y = torch.randn(B, d, device="cuda", generator=g)
    D0 = torch.randn(B, d, device="cuda", generator=g)
    n = torch.full((B,), T // 2, dtype=torch.int32, device="cuda")
    ids = torch.arange(B, dtype=torch.int64, device="cuda")
    Ytil = torch.zeros(B, K, d, device="cuda")
    krow = torch.zeros(B, K, dtype=torch.int32, device="cuda")
    mirror = torch.zeros(B, K, d, dtype=torch.int16, device="cuda") if cfg.kind == "mlp" else None
    ctx.sd_set_draft_mirror(mirror)
    us = _time_launches(lambda: ctx.sd_draft(B, y, n, ids, D0, Ytil, krow), iters)
    moved = B * K * d * (4 + (2 if mirror is not None else 0)) + 2 * B * d * 4
    print(json.dumps({"kernel": "draft_frozen_kernel", "workload": workload, "chains": B, "d": d, "K": K,
                      "bf16_image": mirror is not None, "bytes_moved": moved, "avg_launch_us": round(us, 2),
                      "TB/s": round(moved / (us * 1e-6) * 1e-12, 3),
                      "normals_per_second": round(B * K * d / (us * 1e-6), 1)}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD, choices=sorted(DESCRIPTIONS))
    ap.add_argument("--stages", action="store_true", help="time every stage (adds event overhead)")
    ap.add_argument("--drafter", default="frozen", choices=["frozen", "independent", "efficient_frozen", "efficient_frozen_last_accepted"],
                    help="frozen (default, the benchmark's drafter); independent: a cheaper network of the same "
                         "family called at every window position; efficient_frozen: frozen on the prediction "
                         "carried over from the previous window, one batched target call per window (c1-c4); "
                         "efficient_frozen_last_accepted: the same with the appendix's alternative carry rule "
                         "(after a rejection, the prediction at the last accepted state)")
    ap.add_argument("--loop", default=None, choices=["eager", "multi", "graph", "fused"],
                    help="window loop: eager = one host readback of the batch size per window; multi = batch size kept "
                         "on the device, --windows-per-sync windows per readback; graph = multi with window + advance "
                         "replayed from a HIP graph; fused (c5, phi4) = every chain's windows back to back in one launch "
                         "(sd_langevin_run: bit-identical results, no compaction needed).  Default: graph for c1, multi for "
                         "c2 and c3, fused for c5 and phi4 (whichever measured faster), eager for c4 (windows of 2 ms: no difference)")
    ap.add_argument("--windows-per-sync", type=int, default=4)
    ap.add_argument("--verify-shape", type=int, default=0,
                    help="launch shape of the accept / reflect kernel in the sampler (sd_set_verify_shape; 0 = default)")
    ap.add_argument("--gemm-variant", type=int, default=0,
                    help="MLP GEMM kernel in the sampler (sdden_mlp_select_gemm; 0 = default; the workload must use the MLP)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-context", action="store_true",
                    help="skip the untimed extras (acceptance by position, sequential chain on the GPU)")
    ap.add_argument("--accept", default="mixed", choices=["all", "second", "tail", "mixed"], help="with --kernel verify")
    ap.add_argument("--shapes", default="0", help="with --kernel verify: comma-separated sd_set_verify_shape codes")
    ap.add_argument("--kernel", default=None, choices=["gemm", "verify", "draft", "stream", "mfma"],
                    help="time one kernel family in isolation instead of the sampler (controlled runs behind the "
                         "bounds quoted for the kernels): gemm = the three MLP GEMMs of the c4 batched call; verify = the "
                         "accept / reflect kernel on planted rejections (--workload, --accept, --shapes); draft = the frozen "
                         "rollout; stream / mfma = the plain copy and MFMA-only kernels the bounds are compared with")
    ap.add_argument("--variants", default=None, help="with --kernel gemm: comma-separated sdden_mlp_select_gemm codes")
    ap.add_argument("--iters", type=int, default=20, help="launches per timed kernel with --kernel")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device copy (reference for scaling rocprof FETCH_SIZE/WRITE_SIZE)")
    args = ap.parse_args()
    if args.copy_calibration:
        import torch
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": src.numel() * 4, "copy_bytes_written": src.numel() * 4, "copies": 5}))
        return
    if args.kernel == "gemm":
        kernel_gemm(args.iters, variants=[int(v) for v in args.variants.split(",")] if args.variants else None)
        return
    if args.kernel == "stream":
        kernel_stream(args.iters)
        return
    if args.kernel == "mfma":
        kernel_mfma(args.iters)
        return
    if args.kernel == "draft":
        kernel_draft(args.workload, args.iters)
        return
    if args.kernel == "verify":
        kernel_verify(args.workload, args.accept, [int(v) for v in args.shapes.split(",")], args.iters)
        return
    if args.gpus != 1:
        raise SystemExit("bench.py: this build runs on ONE GPU only (chains are independent and would shard by "
                         "chain id with no collective on the hot path); run with --gpus 1")
    import workloads as W
    import torch
    if torch.cuda.device_count() < 1:          # counting devices does not initialise the GPU
        raise SystemExit("bench.py needs a GPU (the HIP library has no CPU fallback)")
    cfg = W.make_config(args.workload)
    steps = args.steps if args.steps is not None else {"c1": 20, "c2": 10, "c3": 3, "c4": 3, "c5": 2, "phi4": 3}[cfg.name]
    if args.drafter != "frozen" and cfg.kind in ("langevin", "phi4"):
        raise SystemExit("bench.py: the drafter variants are built for the diffusion workloads c1-c4")
    if args.loop == "fused" and cfg.kind not in ("langevin", "phi4"):
        raise SystemExit("bench.py: --loop fused is the one-launch form of the Langevin workloads (c5, phi4)")
    loop = args.loop or ({"c1": "graph", "c2": "multi", "c3": "multi", "c5": "fused", "phi4": "fused"}.get(cfg.name, "eager")
                         if args.drafter == "frozen" else "eager")
    # the oracle is timed first: its worker processes are forked, which must not happen once the GPU is initialised
    baseline = None if args.no_cpu_baseline else cpu_baseline(cfg, drafter=args.drafter)
    elapsed, counters, roofline, stage_table = run_gpu(cfg, steps, args.warmup, args.stages, args.drafter, loop,
                                                       args.windows_per_sync, args.verify_shape, args.gemm_variant)
    total_steps = counters[0]
    assert total_steps == cfg.B * cfg.T * steps, (total_steps, cfg.B, cfg.T, steps)
    line = {
        "metric": "verified diffusion steps/sec at 1 GPU",
        "value": round(total_steps / elapsed, 1),
        "unit": "verified diffusion steps/s",
        "n_gpus": 1, "steps": steps, "warmup": args.warmup,
        "ms_per_step": round(1e3 * elapsed / steps, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.kind == "mlp" else ("f64" if cfg.kind in ("langevin", "phi4") else "f32"), "data": "synthetic",
        "config": {"workload": DESCRIPTIONS[cfg.name], "chains": cfg.B, "d": cfg.d, "window_K": cfg.K,
                   "chain_steps_T": cfg.T, "drafter": args.drafter, "seed": cfg.seed, "window_loop": loop,
                   "step_definition": "one full sampler pass: all chains from step 0 to T"},
        "mean_accepted_draft_length": round(counters[0] / max(1, counters[1]), 4),
        # one launch per pass with --loop fused: a "window" is then the mean number of windows per chain
        "windows_per_step": round((counters[1] / cfg.B if loop == "fused" else counters[3]) / steps, 2),
        "ms_per_window": round(1e3 * elapsed / max(1, counters[1] / cfg.B if loop == "fused" else counters[3]), 4),
        "rejections_per_chain_window": round(counters[2] / max(1, counters[1]), 4),
        "target_rows_evaluated": counters[4],
        "roofline": roofline,
    }
    if stage_table:
        line["stages"] = stage_table
    if not args.no_context:
        line["context"] = run_context(cfg, args.drafter)
    if baseline is not None:
        line["cpu_baseline"] = baseline
    print(json.dumps(line))


if __name__ == "__main__":
    main()

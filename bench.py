#!/usr/bin/env python3
"""Benchmark of the routing-aware fused-MoE path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--model dsv3] [--no-sweep] [--no-extra]

One "step" is one pass of the whole hot path on a batch that is already resident in HBM:
expert histogram -> cost-model select (Eq. 6) -> fused MoE with the selected configuration
(align, up-projection + SwiGLU, down-projection, top-k combine).
Default workload: the largest single-GPU one, the DeepSeek-V3-shaped layer (H=7168, I=2048, E=256,
top-8) at T=8192 tokens with uniform routing.  Before the timed region the script (untimed) profiles
the configuration family at 5 batch sizes x 5 skew levels and fits the cost model, then times every
configuration at every (T, beta) point of the model's sweep to report regret against exhaustive
search, the speedup over static batch-size-only dispatch, and microseconds / TFLOP/s / GB/s /
roofline fraction per point.  After the timed region it adds the largest point of the other model
shapes (best configuration of an exhaustive pass over the large-tile configurations) and the CPU
oracle on a token sample.  Rank 0 prints ONE JSON line at the end; tables go to stderr and --out.
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

HBM_PEAK_TBS = 8.0       # MI355X HBM3E
MFMA_PEAK_PFLOPS = 2.5   # dense bf16
FP8_PEAK_PFLOPS = 5.0    # dense FP8

# HBM bytes per launch of the dominant kernel (up-projection + SwiGLU) recorded from two separate
# `rocprofv3 --pmc` runs of this script (FETCH_SIZE, then WRITE_SIZE; each scaled by what the same
# counter reads for the library's 1 GiB copy kernel).  These are RECORDED values, not measured in the
# run that prints them: each entry names the text summary under profiles/ that holds the run and its
# per-kernel table.  Keyed by (model, T, beta), one entry per tile configuration (bm, bn, bk, waves, stages) that was
# profiled; other workloads, or another dispatched configuration, report null.
RECORDED_TRAFFIC = {
    ("dsv3", 8192, "1.0"): [(16.24e9 + 286.7e6, (288, 256, 32, 8, 4), "profiles/dsv3_T8192_uniform_pingpong_288x256_272x256_256x256_trace_traffic_sq.md"),
                            (17.98e9 + 278.7e6, (272, 256, 32, 8, 4), "profiles/dsv3_T8192_uniform_pingpong_288x256_272x256_256x256_trace_traffic_sq.md")],
    ("dsv3", 2048, "0.2"): [(5.43e9 + 68.8e6, (256, 256, 32, 8, 4), "profiles/dsv3_T2048_beta02_and_mixtral_T8192_pingpong_256x256_trace_traffic_sq.md")],
    ("mixtral", 8192, "1.0"): [(16.56e9 + 471.6e6, (256, 256, 32, 8, 4), "profiles/dsv3_T2048_beta02_and_mixtral_T8192_pingpong_256x256_trace_traffic_sq.md")],
    ("qwen3", 8192, "1.0"): [(1.69e9 + 104.0e6, (272, 256, 32, 8, 4), "profiles/qwen3_T8192_and_olmoe_T4096_pingpong_trace_traffic_sq.md")],
    ("olmoe", 4096, "1.0"): [(1.14e9 + 68.1e6, (256, 256, 32, 8, 4), "profiles/qwen3_T8192_and_olmoe_T4096_pingpong_trace_traffic_sq.md")],
}

# Largest point of every other model shape, reported next to the headline.
EXTRA_ROWS = {
    "dsv3": [("dsv3", 8192, 0.1), ("mixtral", 8192, 1.0), ("qwen3", 8192, 1.0), ("olmoe", 4096, 1.0)],
}
# Points of the W8A8 FP8 variant (Sec. 4.3) reported next to them: a weight-bound decode-sized batch and the largest one.
FP8_ROWS = {
    "dsv3": [("dsv3", 64, 1.0), ("dsv3", 8192, 1.0), ("mixtral", 16, 1.0), ("mixtral", 8192, 1.0), ("olmoe", 64, 1.0)],
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def geomean(v):
    v = np.asarray(v, np.float64)
    return float(np.exp(np.log(v).mean())) if v.size else float("nan")


def kernel_name(cfg):
    fam = "moe_pingpong_kernel<1>" if cfg.mode & 0x400 else "moe_stream_kernel<1>" if cfg.mode & 0x100 else "moe_gemm_kernel<1>"
    return fam + " (up-projection + SwiGLU)"


def stage_times_us(ramp, tuner, layers, cfg, pt, iters=6):
    """Mean HIP-event time of each stage of ramp_fused_moe (align, up-projection, down-projection, combine)."""
    out = []
    for stage in (1, 2, 3, 4):
        ramp.probe_enable(stage)
        ramp.probe_read()
        tuner.time_config(layers, cfg, pt, warmup=1, iters=iters, budget_ms=100.0)
        ms, n = ramp.probe_read()
        out.append(ms / max(n, 1) * 1e3)
    ramp.probe_enable(0)
    return out


def kernel_roofline(s, T, counts, k_us):
    """Roofline of the dominant kernel (up-projection + SwiGLU): algorithmic flops / bytes of one launch."""
    P = T * s.k
    e_act = int((np.asarray(counts) > 0).sum())
    k_flops = 4.0 * P * s.H * s.I
    k_bytes = e_act * 2 * s.H * s.I * 2 + T * s.H * 2 + P * s.I * 2
    t_hbm_k, t_mfma_k = k_bytes / (HBM_PEAK_TBS * 1e12) * 1e6, k_flops / (MFMA_PEAK_PFLOPS * 1e15) * 1e6
    if t_mfma_k >= t_hbm_k:
        roof = dict(bound="mfma", achieved=k_flops / k_us * 1e-6, peak=MFMA_PEAK_PFLOPS * 1e3, unit="TFLOP/s")
    else:
        roof = dict(bound="hbm", achieved=k_bytes / k_us * 1e-3, peak=HBM_PEAK_TBS * 1e3, unit="GB/s")
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof.update(kernel_us=k_us, algorithmic_flops=k_flops, algorithmic_bytes=k_bytes)
    return roof


def mfma_ceiling(torch, ramp, dev, rounds=20000):
    """PFLOP/s of a register-resident MFMA loop (no memory traffic) on zero operands and on N(0,1) bf16 operands:
    what the matrix pipes sustain under this chip's power limit, next to the nominal 2.5 PFLOP/s."""
    sink = torch.empty(256 * 512 * 4, dtype=torch.float32, device=dev)
    out = {}
    gen = torch.Generator(device=dev)
    gen.manual_seed(99)
    for name, ops in (("zeros", torch.zeros(12 * 512, dtype=torch.bfloat16, device=dev)),
                      ("normal", torch.randn(12 * 512, generator=gen, device=dev).to(torch.bfloat16))):
        best = 0.0
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            flops = ramp.mfma_rate_probe(ops, rounds, sink)
            e1.record()
            torch.cuda.synchronize()
            best = max(best, flops / (e0.elapsed_time(e1) * 1e-3) * 1e-15)
        out[name + "_operands_pflops"] = best
    return out


def vendor_gemm_reference(torch, s, P, dev, iters=10):
    """Context only, never part of the timed path: what the vendor library's dense bf16 GEMM (torch.matmul) sustains on
    this box on N(0,1) operands, at the up-projection's dimensions with the pairs as one dense batch (no gather, no
    expert grouping, no SwiGLU): the practical ceiling of an MFMA-bound kernel under the chip's power limit."""
    try:
        M, N, K = int(min(max(P, 4096), 16384)), 2 * s.I, s.H
        gen = torch.Generator(device=dev)
        gen.manual_seed(5)
        a = torch.randn(M, K, generator=gen, device=dev).to(torch.bfloat16)
        b = torch.randn(N, K, generator=gen, device=dev).to(torch.bfloat16)
        for _ in range(3):
            c = a @ b.t()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(iters):
            c = a @ b.t()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / iters
        del a, b, c
        return dict(shape_mnk=[M, N, K], us=us, pflops=2.0 * M * N * K / us * 1e-9, operands="N(0,1) bf16",
                    what="torch.matmul (vendor GEMM library), dense, reference only")
    except Exception as exc:  # a missing or failing vendor library must not fail the benchmark
        return dict(error=str(exc)[:200])


def fp8_rows(torch, ramp, synth, tuner, rows, iters, dev, log_fn):
    """W8A8 FP8 variant: exhaustive pass over its tile family at each point (one layer set per model shape),
    against the FP8 roofline (weights one byte each, 5.0 PFLOP/s)."""
    out = []
    for name in dict.fromkeys(r[0] for r in rows):
        s = synth.SHAPES[name]
        pts = [r for r in rows if r[0] == name]
        layer_bytes = 3 * s.E * s.H * s.I
        n_layers = int(max(1, min(8, (3 << 30) // layer_bytes)))
        layers = tuner.LayerSet(s, max(r[1] for r in pts), n_layers, seed=1, device=dev, x_std=1.0, fp8=True, bf16=False)
        fam = tuner.Family.of(s, fp8=True)
        for _, T, beta in pts:
            p = tuner.Point(T, beta, seed=4242).materialise(s)
            times = [tuner.time_config(layers, c, p, warmup=3, iters=iters, budget_ms=150.0) for c in fam.cfgs]
            b = int(np.argmin(times))
            t_hbm, t_mfma, nbytes, flops = tuner.roofline_lower_bound_us(s, T, p.counts, HBM_PEAK_TBS, FP8_PEAK_PFLOPS, weight_bytes=1)
            row = dict(model=name, T=T, beta=beta, dtype="fp8_e4m3 (W8A8, power-of-two 128x128 block scales)", us=times[b],
                       config=fam.cfgs[b].key(), configs_timed=len(fam.cfgs), bound="hbm" if t_hbm >= t_mfma else "mfma",
                       roofline_frac=max(t_hbm, t_mfma) / times[b], tflops=flops / times[b] * 1e-6, gbs=nbytes / times[b] * 1e-3,
                       weight_copies_rotated=n_layers)
            out.append(row)
            log_fn(f"[bench] FP8 {name} T={T} beta={beta}: best of {len(fam.cfgs)} configurations {times[b]:.1f} us "
                   f"({100 * row['roofline_frac']:.1f}% of the FP8 {row['bound']} bound), {fam.cfgs[b]}")
        del layers
        torch.cuda.empty_cache()
    return out


def extra_row(torch, ramp, synth, tuner, name, T, beta, iters, dev):
    """Largest point of another model shape: exhaustive pass over its large-tile configurations (bm >= 128),
    stage times of the best one."""
    s = synth.SHAPES[name]
    layer_bytes = 3 * s.E * s.H * s.I * 2
    n_layers = int(max(1, min(8, (3 << 30) // layer_bytes)))
    layers = tuner.LayerSet(s, T, n_layers, seed=1, device=dev, x_std=1.0)
    fam = tuner.Family.of(s)
    p = tuner.Point(T, beta, seed=4242).materialise(s)
    cands = [c for c in fam.cfgs if c.bm >= 128]
    times = [tuner.time_config(layers, c, p, warmup=3, iters=iters, budget_ms=150.0) for c in cands]
    b = int(np.argmin(times))
    st = stage_times_us(ramp, tuner, layers, cands[b], p)
    t_hbm, t_mfma, nbytes, flops = tuner.roofline_lower_bound_us(s, T, p.counts, HBM_PEAK_TBS, MFMA_PEAK_PFLOPS)
    roof = kernel_roofline(s, T, p.counts, st[1])
    row = dict(model=name, T=T, beta=beta, us=times[b], config=cands[b].key(), configs_timed=len(cands),
               bound="hbm" if t_hbm >= t_mfma else "mfma", roofline_frac=max(t_hbm, t_mfma) / times[b],
               tflops=flops / times[b] * 1e-6, gbs=nbytes / times[b] * 1e-3,
               stage_us=dict(align=st[0], up=st[1], down=st[2], combine=st[3]),
               up_kernel=dict(bound=roof["bound"], achieved=roof["achieved"], unit=roof["unit"], frac=roof["frac"]),
               weight_copies_rotated=n_layers)
    log(f"[bench] {name} T={T} beta={beta}: best of {len(cands)} large-tile configurations {times[b]:.1f} us "
        f"({100 * row['roofline_frac']:.1f}% of the {row['bound']} bound), {cands[b]}; stages align/up/down/combine "
        + "/".join(f"{v:.1f}" for v in st) + " us")
    del layers
    torch.cuda.empty_cache()
    return row


def head_to_head_regret(tuner, layers, fam, p, chosen, times, iters):
    """The minimum over all configurations of one noisy timing each is biased low (the winner is partly the luckiest
    measurement), which inflates the regret of near-ties.  Second figure: the three fastest configurations of `times` and
    the dispatched one timed again in alternation (three rounds), regret against the fastest of those medians."""
    if chosen == int(np.argmin(times)):
        return 0.0
    cand = list(dict.fromkeys([chosen] + [int(i) for i in np.argsort(times)[:3]]))
    again = {c: [] for c in cand}
    for _ in range(3):
        for c in cand:
            again[c].append(tuner.time_config(layers, fam.cfgs[c], p, warmup=2, iters=iters, budget_ms=40.0))
    med = {c: float(np.median(v)) for c, v in again.items()}
    return med[chosen] / min(med.values()) - 1.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--model", default="dsv3", choices=["tiny", "olmoe", "qwen3", "mixtral", "dsv3"])
    ap.add_argument("--T", type=int, default=None, help="headline batch size (default: largest of the sweep)")
    ap.add_argument("--beta", default=None, help="headline skew (default 1.0)")
    ap.add_argument("--layers", type=int, default=None, help="distinct weight copies to rotate over")
    ap.add_argument("--no-sweep", action="store_true", help="skip the regret / static-dispatch sweep")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-extra", action="store_true", help="skip the largest points of the other model shapes")
    ap.add_argument("--heldout", type=int, default=0, help="extra seeded held-out histograms for regret (dsv3: 200)")
    ap.add_argument("--iters", type=int, default=50)
    ap.add_argument("--config", default=None,
                    help="bm,bn,bk,waves,stages,mode: skip profiling/fit and run the headline with this fixed "
                         "configuration (for profiler runs)")
    ap.add_argument("--save-model", default=None, help="write the fitted cost-model table of this shape (JSON) here")
    ap.add_argument("--out", default=os.path.join(ROOT, "gpurun_out"))
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is a single-GPU path (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2604_26039_amd import ramp, synth, tuner

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    ramp.lib()  # fail loudly if the HIP library is missing
    dev = "cuda:0"
    torch.cuda.set_device(0)
    t_begin = time.time()
    s = synth.SHAPES[args.model]
    sweep = synth.SWEEPS[args.model]
    T_head = args.T if args.T is not None else max(sweep["T"])
    beta_head = 1.0 if args.beta is None else (args.beta if args.beta.startswith("zipf") else float(args.beta))
    T_max = max(max(sweep["T"]), T_head)
    layer_bytes = 3 * s.E * s.H * s.I * 2
    n_layers = args.layers if args.layers else int(max(1, min(8, (3 << 30) // layer_bytes)))
    os.makedirs(args.out, exist_ok=True)

    t0 = time.time()
    layers = tuner.LayerSet(s, T_max, n_layers, seed=1, device=dev, x_std=1.0)
    fam = tuner.Family.of(s)
    n_cfg = len(fam.cfgs)
    log(f"[bench] {args.model}: H={s.H} I={s.I} E={s.E} k={s.k}; {n_cfg} configurations; {n_layers} weight copies "
        f"({layer_bytes * n_layers / 2**30:.1f} GiB); setup {time.time() - t0:.1f}s")

    fixed_cfg = None
    if args.config:
        want = tuple(int(v) for v in args.config.split(","))
        match = [i for i, c in enumerate(fam.cfgs) if c.key() == want]
        if not match:
            # an instantiated variant that the pool rule leaves out for this shape (e.g. a GROUP_M block shape): run it by name
            extra_cfg = ramp.Config(*want)
            fam = tuner.Family(fam.shape, fam.cfgs + [extra_cfg], np.append(fam.ntiles, ramp.config_ntiles(fam.shape, extra_cfg)).astype(np.int32),
                               np.append(fam.wave_cap, ramp.config_wave_capacity(extra_cfg)).astype(np.int32))
            n_cfg = len(fam.cfgs)
            match = [n_cfg - 1]
        fixed_cfg = match[0]
        args.no_sweep = True
        args.no_extra = True

    # ------------------------------------------------------------------ one-time profiling + fit (Sec. 4.2)
    fit_T = tuner.fit_batch_sizes(sweep["T"])
    fit_pts = [tuner.Point(T, b, seed=100000 + 97 * i + j) for i, T in enumerate(fit_T) for j, b in enumerate(tuner.FIT_BETAS)]
    t0 = time.time()
    if fixed_cfg is not None:
        fit_pts = fit_pts[:2]
    log(f"[bench] profiling {len(fit_pts)} fit points x {n_cfg} configs (T in {fit_T}, beta in {tuner.FIT_BETAS})")
    if fixed_cfg is None:
        g_fit, t_fit = tuner.profile(layers, fam, fit_pts, iters=min(args.iters, 20), warmup=3, budget_ms=60.0)
    else:
        for pt in fit_pts:
            pt.materialise(s)
        g_fit = np.stack([fam.grid(pt.counts) for pt in fit_pts], axis=1)
        t_fit = np.ones_like(g_fit, dtype=np.float64)
    counts_fit = [p.materialise(s).counts for p in fit_pts]
    # Eq. 6 as printed, every single departure from it, the fit-only change plus the traffic column, and the model
    # that is dispatched (all four departures)
    MODELS = {"eq6": ramp.CM_EQ6, "relative_fit": ramp.CM_RELATIVE, "distinct_tiles": ramp.CM_DISTINCT_TILES,
              "wave_floor": ramp.CM_WAVE_FLOOR, "pairs": ramp.CM_PAIRS, "rounds": ramp.CM_ROUNDS,
              "relative_fit+distinct_tiles": ramp.CM_RELATIVE | ramp.CM_DISTINCT_TILES,
              "all_but_rounds": tuner.MI355X_MODEL & ~ramp.CM_ROUNDS,
              "eq6_mi355x": tuner.MI355X_MODEL}
    thetas = {name: tuner.fit(fam, g_fit, t_fit, counts_fit, flags) for name, flags in MODELS.items()}
    DISPATCH = "eq6_mi355x"
    theta, dispatch_flags = thetas[DISPATCH], MODELS[DISPATCH]
    # term ablation of the dispatch model (Sec. 5.3): the same fit with the later columns zeroed, so their
    # coefficients come out zero (minimum-norm solution): 2 terms = a + b*w, 3 terms = + c*m, 4 terms = + d*P
    u_fit = tuner.distinct_tiles(fam, counts_fit)
    P_fit = np.array([ramp.grid(s.E, fam.cfgs, fam.ntiles, c)[2] for c in counts_fit], np.int64)
    gr_fit = tuner.grid_rounds(fam, counts_fit)
    ABLATION = {2: ramp.cost_model_fit(fam.wave_cap, g_fit, t_fit, distinct=np.zeros_like(u_fit), pairs=np.zeros_like(P_fit),
                                       flags=dispatch_flags, grid_rounds=gr_fit),
                3: ramp.cost_model_fit(fam.wave_cap, g_fit, t_fit, distinct=u_fit, pairs=np.zeros_like(P_fit),
                                       flags=dispatch_flags, grid_rounds=gr_fit),
                4: theta}
    # Sec. 5.3's fifth term (g^2) on top of Eq. 6 as printed and on top of the dispatch model
    theta5 = {name: tuner.fit5(fam, g_fit, t_fit, counts_fit, MODELS[name]) for name in ("eq6", DISPATCH)}
    if args.save_model and fixed_cfg is None:
        tuner.save_model(args.save_model, fam, theta, dispatch_flags,
                         extra=dict(model=args.model, fit_T=fit_T, fit_betas=[str(b) for b in tuner.FIT_BETAS]))

    def predictions(name, counts):
        return ramp.cost_model_select(s.E, fam.cfgs, fam.ntiles, fam.wave_cap, thetas[name], counts, want_pred=True,
                                      flags=MODELS[name], rounds=fam.rounds)[1]

    r2 = {}
    for name in ("eq6", DISPATCH):
        pred_fit = np.stack([predictions(name, c) for c in counts_fit], axis=1)
        ss_res = ((pred_fit - t_fit) ** 2).sum(axis=1)
        ss_tot = ((t_fit - t_fit.mean(axis=1, keepdims=True)) ** 2).sum(axis=1)
        r2[name] = 1.0 - ss_res / np.maximum(ss_tot, 1e-30)
    log(f"[bench] fit done in {time.time() - t0:.1f}s; R^2 (eq6) min {r2['eq6'].min():.3f} median {np.median(r2['eq6']):.3f}; "
        f"log term active in {(thetas['eq6'][:, 3] != 0).sum()}/{n_cfg} configs")

    # ------------------------------------------------------------------ sweep: exhaustive vs cost model vs static
    report = {"model": args.model, "configs": [c.key() for c in fam.cfgs],
              "theta": {k: v.tolist() for k, v in thetas.items()}, "r2": {k: v.tolist() for k, v in r2.items()},
              "ntiles": fam.ntiles.tolist(), "wave_cap": fam.wave_cap.tolist(),
              "fit": {"T": [p.T for p in fit_pts], "beta": [p.beta for p in fit_pts], "grid": g_fit.tolist(),
                      "time_us": t_fit.tolist(), "counts": [c.tolist() for c in counts_fit]},
              "points": []}
    summary = {}
    if not args.no_sweep:
        pts = [tuner.Point(T, b, seed=500 + 31 * i + j) for i, T in enumerate(sweep["T"]) for j, b in enumerate(sweep["beta"])]
        t0 = time.time()
        log(f"[bench] sweep: {len(pts)} held-out points x {n_cfg} configs")
        g_ev, t_ev = tuner.profile(layers, fam, pts, log=log, iters=args.iters, warmup=5, budget_ms=100.0)
        static_of_T = {}
        for j, p in enumerate(pts):
            if p.beta == 1.0 or p.beta == sweep["beta"][0]:
                static_of_T.setdefault(p.T, int(np.argmin(t_ev[:, j])))
        regrets = {name: [] for name in MODELS}
        regrets_h2h = []
        abl_regrets = {k: [] for k in ABLATION}
        regrets5 = {name: [] for name in theta5}
        speedups = {}
        hdr = (f"{'T':>5} {'beta':>8} {'bH':>5} {'best us':>9} {'RA us':>9} {'static us':>9} {'regret%':>8} {'eq6 reg%':>8} "
               f"{'RA/static':>9} {'bound':>5} {'roof%':>6} {'TFLOP/s':>8} {'GB/s':>7}  best / RA / static bm")
        log(hdr)
        for j, p in enumerate(pts):
            best = int(np.argmin(t_ev[:, j]))
            st = static_of_T[p.T]
            picks = {name: tuner.select(fam, thetas[name], p.counts, MODELS[name]) for name in MODELS}
            for name in MODELS:
                regrets[name].append(t_ev[picks[name], j] / t_ev[best, j] - 1.0)
            for k_terms, th_k in ABLATION.items():
                abl_regrets[k_terms].append(t_ev[tuner.select(fam, th_k, p.counts, dispatch_flags), j] / t_ev[best, j] - 1.0)
            for name, th5 in theta5.items():
                regrets5[name].append(t_ev[tuner.select5(fam, th5, p.counts, MODELS[name]), j] / t_ev[best, j] - 1.0)
            chosen = picks[DISPATCH]
            reg = regrets[DISPATCH][-1]
            reg_h2h = head_to_head_regret(tuner, layers, fam, p, chosen, t_ev[:, j], min(args.iters, 10))
            regrets_h2h.append(reg_h2h)
            hot_us = tuner.time_config(layers, fam.cfgs[chosen], p, warmup=3, iters=min(args.iters, 20), budget_ms=60.0, hot=True)
            spd = t_ev[st, j] / t_ev[chosen, j]
            speedups.setdefault(str(p.beta), []).append(spd)
            t_hbm, t_mfma, nbytes, flops = tuner.roofline_lower_bound_us(s, p.T, p.counts, HBM_PEAK_TBS, MFMA_PEAK_PFLOPS)
            bound = "hbm" if t_hbm >= t_mfma else "mfma"
            frac = max(t_hbm, t_mfma) / t_ev[chosen, j]
            row = dict(T=p.T, beta=p.beta, beta_entropy=tuner.entropy_beta(p.counts), best_us=t_ev[best, j],
                       ra_us=t_ev[chosen, j], ra_hot_us=hot_us, static_us=t_ev[st, j], regret=reg, regret_remeasured=reg_h2h,
                       regret_eq6=regrets["eq6"][-1],
                       ra_over_static=spd, bound=bound, roofline_frac=frac, roofline_frac_best=max(t_hbm, t_mfma) / t_ev[best, j],
                       tflops=flops / t_ev[chosen, j] * 1e-6, gbs=nbytes / t_ev[chosen, j] * 1e-3,
                       best_cfg=fam.cfgs[best].key(), ra_cfg=fam.cfgs[chosen].key(), static_cfg=fam.cfgs[st].key(),
                       all_us=t_ev[:, j].tolist(), grid=g_ev[:, j].tolist(), counts=p.counts.tolist())
            report["points"].append(row)
            log(f"{p.T:>5} {p.beta!s:>8} {row['beta_entropy']:5.2f} {row['best_us']:9.1f} {row['ra_us']:9.1f} "
                f"{row['static_us']:9.1f} {100 * reg:8.2f} {100 * row['regret_eq6']:8.2f} {spd:9.3f} {bound:>5} {100 * frac:6.1f} "
                f"{row['tflops']:8.1f} {row['gbs']:7.0f}  {fam.cfgs[best].bm}/{fam.cfgs[chosen].bm}/{fam.cfgs[st].bm}")
        skew = [r for r in report["points"] if str(r["beta"]) != str(sweep["beta"][0])]
        uniform = [r for r in report["points"] if str(r["beta"]) == str(sweep["beta"][0])]
        summary = dict(dispatch_model=DISPATCH,
                       mean_regret=float(np.mean(regrets[DISPATCH])), max_regret=float(np.max(regrets[DISPATCH])),
                       median_regret=float(np.median(regrets[DISPATCH])),
                       mean_regret_remeasured=float(np.mean(regrets_h2h)), max_regret_remeasured=float(np.max(regrets_h2h)),
                       mean_regret_eq6_as_printed=float(np.mean(regrets["eq6"])),
                       max_regret_eq6_as_printed=float(np.max(regrets["eq6"])),
                       model_variants={name: dict(flags=int(MODELS[name]), mean_regret=float(np.mean(v)), max_regret=float(np.max(v)))
                                       for name, v in regrets.items()},
                       term_ablation_mean_regret={str(k): float(np.mean(v)) for k, v in abl_regrets.items()},
                       five_term_mean_regret={name: float(np.mean(v)) for name, v in regrets5.items()},
                       ra_over_static_geomean={b: geomean(v) for b, v in speedups.items()},
                       ra_over_static_geomean_skewed=geomean([r["ra_over_static"] for r in skew]),
                       ra_over_static_min_uniform=float(min(r["ra_over_static"] for r in uniform)),
                       best_over_static_geomean_skewed=geomean([r["static_us"] / r["best_us"] for r in skew]),
                       paper_context=dict(mean_regret=0.0093, ra_over_static=1.22, hardware="H200 FP8"))
        log(f"[bench] sweep {time.time() - t0:.1f}s: mean regret {100 * summary['mean_regret']:.2f}% "
            f"(median {100 * summary['median_regret']:.2f}%, max {100 * summary['max_regret']:.2f}%; top three and the pick timed again: "
            f"mean {100 * summary['mean_regret_remeasured']:.2f}%, max {100 * summary['max_regret_remeasured']:.2f}%); RA/static geomean on skewed points "
            f"{summary['ra_over_static_geomean_skewed']:.3f}x (exhaustive ceiling {summary['best_over_static_geomean_skewed']:.3f}x), "
            f"worst uniform point {summary['ra_over_static_min_uniform']:.3f}x")
        log("[bench] mean / max regret by model variant: " + "; ".join(
            f"{name} {100 * v['mean_regret']:.2f}/{100 * v['max_regret']:.1f}%" for name, v in summary["model_variants"].items()))
        log("[bench] term ablation of the dispatch model 2/3/4 terms: "
            + " / ".join(f"{100 * summary['term_ablation_mean_regret'][str(k)]:.2f}%" for k in (2, 3, 4))
            + "; with a fifth term g^2: " + ", ".join(f"{n} {100 * v:.2f}%" for n, v in summary["five_term_mean_regret"].items()))

    if args.heldout > 0:
        rng = np.random.default_rng(7)
        regs, regs_eq6, regs_nr, regs_h2h, rows_h = [], [], [], [], []
        t0 = time.time()
        for h in range(args.heldout):
            T = int(rng.choice(sweep["T"][1:]))
            b = sweep["beta"][int(rng.integers(len(sweep["beta"])))]
            p = tuner.Point(T, b, seed=900000 + h).materialise(s)
            times = np.array([tuner.time_config(layers, c, p, warmup=2, iters=8, budget_ms=30.0) for c in fam.cfgs])
            chosen = tuner.select(fam, theta, p.counts, dispatch_flags)
            regs.append(times[chosen] / times.min() - 1.0)
            regs_h2h.append(head_to_head_regret(tuner, layers, fam, p, chosen, times, 8))
            rows_h.append(dict(T=T, beta=b, seed=900000 + h, regret=float(regs[-1]), regret_remeasured=float(regs_h2h[-1]),
                               best_cfg=fam.cfgs[int(np.argmin(times))].key(), ra_cfg=fam.cfgs[chosen].key()))
            regs_eq6.append(times[tuner.select(fam, thetas["eq6"], p.counts, MODELS["eq6"])] / times.min() - 1.0)
            regs_nr.append(times[tuner.select(fam, thetas["all_but_rounds"], p.counts, MODELS["all_but_rounds"])] / times.min() - 1.0)
            if h % 20 == 19:
                log(f"[bench] held-out {h + 1}/{args.heldout}: mean regret so far {100 * np.mean(regs):.2f}%")
        summary["heldout_histograms"] = dict(n=args.heldout, mean_regret=float(np.mean(regs)), max_regret=float(np.max(regs)),
                                             median_regret=float(np.median(regs)),
                                             mean_regret_remeasured=float(np.mean(regs_h2h)), max_regret_remeasured=float(np.max(regs_h2h)),
                                             histograms=rows_h,
                                             mean_regret_eq6_as_printed=float(np.mean(regs_eq6)),
                                             mean_regret_all_but_rounds=float(np.mean(regs_nr)),
                                             max_regret_all_but_rounds=float(np.max(regs_nr)))
        log(f"[bench] held-out histograms {time.time() - t0:.1f}s: mean {100 * np.mean(regs):.2f}% max {100 * np.max(regs):.2f}% "
            f"(top three and the pick timed again: mean {100 * np.mean(regs_h2h):.2f}% max {100 * np.max(regs_h2h):.2f}%) "
            f"(Eq. 6 as printed: mean {100 * np.mean(regs_eq6):.2f}%; all flags but rounds: mean {100 * np.mean(regs_nr):.2f}% max {100 * np.max(regs_nr):.2f}%)")

    # ------------------------------------------------------------------ headline: K timed steps of the whole path
    p = tuner.Point(T_head, beta_head, seed=4242).materialise(s)
    rs = layers.rs(T_head)
    d_ids = torch.from_numpy(p.ids).to(dev)
    d_w = torch.from_numpy(p.w).to(dev)
    dispatcher = tuner.Dispatcher(fam, theta, dispatch_flags, T_head, device=dev)
    ws = layers.workspace(max(ramp.fused_moe_workspace_bytes(rs, c) for c in fam.cfgs))
    X, out = layers.X[:T_head], layers.out[:T_head]
    chosen_log = []

    def step(i):
        c = dispatcher.select(d_ids)            # histogram + Eq. 6 + argmin on the device, result polled in pinned memory
        if fixed_cfg is not None:
            c = fixed_cfg
        ramp.fused_moe(rs, fam.cfgs[c], X, d_ids, d_w, layers.packed[i % layers.n_layers], out, ws)
        return c

    if fixed_cfg is not None:
        # profiler runs: a plain copy of known size (1 GiB read + 1 GiB written) to calibrate byte counters
        cal_src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        cal_dst = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        cal_src.fill_(1)
        for _ in range(3):
            ramp.copy_bytes(cal_dst, cal_src, 1 << 30)
        torch.cuda.synchronize()
        del cal_src, cal_dst

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    ramp.probe_enable(2)  # the up-projection kernel dominates (2/3 of the flops and of the weight bytes)
    ramp.probe_read()
    t_start = time.perf_counter()
    for i in range(args.steps):
        chosen_log.append(step(i))
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    probe_ms, probe_n = ramp.probe_read()
    ramp.probe_enable(0)
    ms_per_step = elapsed / args.steps * 1e3
    cfg_head = fam.cfgs[chosen_log[-1]]
    # the layer alone with the dispatched configuration (no histogram / select), HIP events per call, and its stages
    fused_us = tuner.time_config(layers, cfg_head, p, warmup=5, iters=args.iters)
    stage_us = stage_times_us(ramp, tuner, layers, cfg_head, p)
    # dispatch latency on an idle GPU, device-resident select (one enqueue, ticket polled in pinned host memory)
    # next to the host-side select (histogram kernel, E-count copy, stream synchronisation, model on the host)
    torch.cuda.synchronize()

    def idle_latency(fn):
        lat = []
        for _ in range(50):
            t0s = time.perf_counter()
            fn(d_ids)
            lat.append(time.perf_counter() - t0s)
        return float(np.median(lat)) * 1e6

    dispatch_idle_us = idle_latency(dispatcher.select)
    dispatch_host_idle_us = idle_latency(dispatcher.select_host)
    if dispatcher.select(d_ids) != dispatcher.select_host(d_ids):
        raise RuntimeError("device-resident select and host select disagree on the headline histogram")
    # the same K steps with the selection taken off the critical path: every call enqueues its selection and
    # launches with the choice of the latest finished one (the previous call's here)
    async_us = None
    if fixed_cfg is None:
        def step_async(i):
            c = dispatcher.select_async(d_ids)
            ramp.fused_moe(rs, fam.cfgs[c], X, d_ids, d_w, layers.packed[i % layers.n_layers], out, ws)
        for i in range(args.warmup):
            step_async(i)
        torch.cuda.synchronize()
        t0s = time.perf_counter()
        for i in range(args.steps):
            step_async(i)
        torch.cuda.synchronize()
        async_us = (time.perf_counter() - t0s) / args.steps * 1e6

    # the whole step as one HIP graph per weight copy: select on the device, then the layer behind the device-side
    # index over the configurations the model picks at this batch size across the sweep's skew levels
    graph_us, graph_cands = None, None
    if fixed_cfg is None:
        picked = []
        for j, b in enumerate(sweep["beta"]):
            c = tuner.select(fam, theta, tuner.Point(T_head, b, seed=900 + j).materialise(s).counts, dispatch_flags)
            if c not in picked:
                picked.append(c)
        picked = picked[:4]
        cands = [fam.cfgs[c] for c in picked]
        table = torch.from_numpy(ramp.select_table_build(cands, fam.ntiles[picked], fam.wave_cap[picked], theta[picked],
                                                         dispatch_flags, rounds=fam.rounds[picked])).to(dev)
        res_dev = torch.zeros(ramp.select_result_bytes(s.E, len(cands)), dtype=torch.uint8, device=dev)
        sel_dev = torch.zeros(1, dtype=torch.int32, device=dev)
        ws_g = layers.workspace(ramp.fused_moe_selected_workspace_bytes(rs, cands))
        graphs = []
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for li in range(layers.n_layers):
                def enqueue():
                    ramp.select_device(d_ids, T_head, s.k, s.E, len(cands), table, res_dev, 1, dispatcher.ws,
                                       best_idx_dev=sel_dev, stream=side)
                    ramp.fused_moe_selected(rs, cands, sel_dev, X, d_ids, d_w, layers.packed[li], out, ws_g, stream=side)
                enqueue()
                side.synchronize()
                gr = torch.cuda.CUDAGraph()
                with torch.cuda.graph(gr, stream=side):
                    enqueue()
                graphs.append(gr)
        torch.cuda.current_stream().wait_stream(side)
        for i in range(args.warmup):
            graphs[i % len(graphs)].replay()
        torch.cuda.synchronize()
        t0s = time.perf_counter()
        for i in range(args.steps):
            graphs[i % len(graphs)].replay()
        torch.cuda.synchronize()
        graph_us = (time.perf_counter() - t0s) / args.steps * 1e6
        graph_cands = [c.key() for c in cands]
        if cands[int(sel_dev.cpu()[0])].key() != cfg_head.key():
            log(f"[bench] note: the graph path selected {cands[int(sel_dev.cpu()[0])]} among {len(cands)} candidates")

    # roofline of the dominant kernel (up-projection + SwiGLU): algorithmic flops / bytes per launch
    k_us = probe_ms / max(probe_n, 1) * 1e3
    roof = kernel_roofline(s, T_head, p.counts, k_us)
    ceiling = mfma_ceiling(torch, ramp, dev)
    log(f"[bench] register-resident MFMA loop: {ceiling['zeros_operands_pflops']:.2f} PFLOP/s on zeros, "
        f"{ceiling['normal_operands_pflops']:.2f} PFLOP/s on N(0,1) bf16 operands (nominal peak {MFMA_PEAK_PFLOPS})")
    ceiling["vendor_gemm"] = vendor_gemm_reference(torch, s, T_head * s.k, dev)
    if "pflops" in ceiling["vendor_gemm"]:
        log(f"[bench] vendor dense GEMM {ceiling['vendor_gemm']['shape_mnk']} on N(0,1) bf16 operands: {ceiling['vendor_gemm']['pflops']:.2f} PFLOP/s (reference only)")
    rec = next((r for r in RECORDED_TRAFFIC.get((args.model, T_head, str(beta_head)), []) if tuple(cfg_head.key()[:5]) == r[1]), None)
    roof.update(traffic=rec[0] if rec else None, traffic_source=(rec[2] + " (recorded rocprofv3 --pmc value, not measured in this run)") if rec else None,
                kernel=kernel_name(cfg_head), launches=probe_n)
    t_hbm, t_mfma, nbytes, flops = tuner.roofline_lower_bound_us(s, T_head, p.counts, HBM_PEAK_TBS, MFMA_PEAK_PFLOPS)
    whole = dict(bound="hbm" if t_hbm >= t_mfma else "mfma", lower_bound_us=max(t_hbm, t_mfma),
                 frac=max(t_hbm, t_mfma) / (ms_per_step * 1e3), tflops=flops / (ms_per_step * 1e3) * 1e-6,
                 gbs=nbytes / (ms_per_step * 1e3) * 1e-3, fused_layer_us=fused_us,
                 fused_layer_frac=max(t_hbm, t_mfma) / fused_us,
                 stage_us=dict(align=stage_us[0], up=stage_us[1], down=stage_us[2], combine=stage_us[3]),
                 dispatch_idle_us=dispatch_idle_us,
                 dispatch_host_select_idle_us=dispatch_host_idle_us, async_dispatch_us_per_step=async_us,
                 graph_dispatch_us_per_step=graph_us, graph_candidates=graph_cands,
                 paper_dispatch_us_h200=38.0)
    log(f"[bench] headline {args.model} T={T_head} beta={beta_head}: {ms_per_step * 1e3:.1f} us/step (fused layer alone {fused_us:.1f} us: "
        + "/".join(f"{v:.1f}" for v in stage_us) + " us align/up/down/combine; "
        f"dispatch on an idle GPU {dispatch_idle_us:.1f} us device-resident / {dispatch_host_idle_us:.1f} us host select, "
        f"{async_us if async_us is None else round(async_us, 1)} us/step with asynchronous dispatch, "
        f"{graph_us if graph_us is None else round(graph_us, 1)} us/step as one HIP graph with device-side selection), config {cfg_head}, "
        f"dominant kernel {k_us:.1f} us = {roof['achieved']:.1f} {roof['unit']} ({100 * roof['frac']:.1f}% of peak)")

    # ------------------------------------------------------------------ CPU oracle baseline (bounded sample)
    cpu = None
    if not args.no_cpu:
        from oracle import oracle
        Wg, Wu, Wd = layers.raw0
        n0 = min(T_head, 4)
        rows = np.linspace(0, T_head - 1, n0).astype(np.int32)
        used = sorted({int(e) for t in rows for e in p.ids[t]})
        # host copies of the experts the sample touches
        hW = [{e: synth.bits(W[e]) for e in used} for W in (Wg, Wu, Wd)]
        Xb = synth.bits(layers.X[:T_head])
        tc = time.perf_counter()
        oracle.moe(Xb, p.ids, p.w, hW[0], hW[1], hW[2], E=s.E, rows=rows)
        per_tok = (time.perf_counter() - tc) / n0
        # about 15 s of CPU work, at most 256 sampled tokens (each sampled token needs host copies of its experts)
        n1 = int(min(T_head, 256, max(n0, 15.0 / max(per_tok, 1e-6))))
        if n1 > n0:
            rows = np.linspace(0, T_head - 1, n1).astype(np.int32)
            used = sorted({int(e) for t in rows for e in p.ids[t]})
            hW = [{e: synth.bits(W[e]) for e in used} for W in (Wg, Wu, Wd)]
            tc = time.perf_counter()
            oracle.moe(Xb, p.ids, p.w, hW[0], hW[1], hW[2], E=s.E, rows=rows)
            per_tok = (time.perf_counter() - tc) / n1
        del hW
        threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        # the oracle's align and select on the same input, beside the layer
        ids_flat = np.ascontiguousarray(p.ids.reshape(-1), np.int32)
        tc = time.perf_counter()
        for _ in range(5):
            oracle.align(ids_flat, T_head, s.k, s.E, cfg_head.bm)
        cpu_align_us = (time.perf_counter() - tc) / 5 * 1e6
        bms = [c.bm for c in fam.cfgs]
        tc = time.perf_counter()
        for _ in range(5):
            oracle.select(bms, fam.ntiles, fam.wave_cap, theta, p.counts, distinct_tiles=True, wave_floor=True, pairs_term=True)
        cpu_select_us = (time.perf_counter() - tc) / 5 * 1e6
        cpu = dict(value=per_tok * T_head * 1e6, unit="us/layer", cores=threads, kind="oracle",
                   oracle_align_us=cpu_align_us, oracle_select_us=cpu_select_us,
                   sample=f"{max(n0, n1)} of {T_head} tokens (evenly spaced rows), per-token time scaled to the full batch "
                          f"(extrapolated)")
        log(f"[bench] CPU oracle: {per_tok * 1e3:.2f} ms/token on {threads} threads -> {cpu['value'] / 1e6:.2f} s/layer (extrapolated)")

    # ------------------------------------------------------------------ largest points of the other model shapes
    extra, fp8 = [], []
    if not args.no_extra:
        del dispatcher, ws
        layers = None
        torch.cuda.empty_cache()
        for name, T, beta in EXTRA_ROWS.get(args.model, []):
            if time.time() - t_begin > 420:
                log(f"[bench] time budget reached, skipping {name} T={T}")
                continue
            extra.append(extra_row(torch, ramp, synth, tuner, name, T, beta, min(args.iters, 12), dev))
        if time.time() - t_begin <= 420:
            fp8 = fp8_rows(torch, ramp, synth, tuner, FP8_ROWS.get(args.model, []), min(args.iters, 12), dev, log)

    report["summary"] = summary
    report["headline"] = dict(T=T_head, beta=beta_head, us=ms_per_step * 1e3, config=cfg_head.key(), whole_path=whole)
    report["largest_points"] = extra
    report["fp8_points"] = fp8
    tag = "_fixed_config" if fixed_cfg is not None else ""
    with open(os.path.join(args.out, f"bench_{args.model}{tag}.json"), "w") as f:
        json.dump(report, f)

    line = {
        "metric": "fused-MoE us/layer (routing-aware dispatch: histogram + select + fused layer)",
        "value": ms_per_step * 1e3, "unit": "us/layer", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.model}-shaped MoE layer H={s.H} I={s.I} E={s.E} top-{s.k}, T={T_head}, beta={beta_head}",
                   "tile_config": cfg_head.key(), "weight_copies_rotated": n_layers},
        "roofline": roof, "mfma_ceiling_measured": ceiling, "whole_path": whole, "cpu_baseline": cpu, "cost_model": summary,
        "largest_points": extra, "fp8_points": fp8,
        "sweep": [dict(T=r["T"], beta=r["beta"], us=round(r["ra_us"], 1), hot_us=round(r["ra_hot_us"], 1), best_us=round(r["best_us"], 1),
                       static_us=round(r["static_us"], 1), bound=r["bound"], roofline_frac=round(r["roofline_frac"], 3),
                       regret=round(r["regret"], 4), bm=r["ra_cfg"][0]) for r in report["points"]],
        "total_s": round(time.time() - t_begin, 1),
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()

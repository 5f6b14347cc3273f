#!/usr/bin/env python3
"""Benchmark of the K-FAC hot path on one MI355X.

A "step" is one pass of the whole path over one synthetic mini-batch: factor construction
with running average for every Conv/FC layer, damped inversion of every factor (or of the
seeded stale subset in configuration 5), preconditioning of every weight gradient, and the
unit-wise BatchNorm call for all BatchNorm layers.  Inputs are resident in HBM before the
timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5] [--dtype f32|bf16]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}   # MI355X dense MFMA peaks
PEAK_HBM_GBS = 8000.0


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4, help="benchmark configuration 1..5 (default: full ResNet-50 set, batch 32)")
    ap.add_argument("--dtype", choices=["f32", "bf16"], default="f32", help="type of activations / output gradients")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-steps", type=int, default=2)
    ap.add_argument("--no-extras", action="store_true", help="skip the measurements beside the step")
    ap.add_argument("--schedule", choices=["fused", "staged"], default="fused",
                    help="fused: one kfac_step call per step (factors, inverses and preconditioning planned as one "
                         "graph); staged: kfac_stats, kfac_invert, kfac_precondition one after the other")
    ap.add_argument("--opt", action="append", default=[], metavar="FIELD=VALUE",
                    help="a kfac_options field for the context of the timed step (e.g. --opt streams=2)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives are built); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2002_06015_amd import kfac, workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    kfac.lib()
    cfg = args.config
    in_dtype = kfac.KFAC_BF16 if args.dtype == "bf16" else kfac.KFAC_F32

    class Job:
        """One layer list resident in HBM: inputs, factors, inverses, outputs, a context, and the calls of a step."""

        def __init__(self, layers, bns, seed_cfg, dtype_name, subset=None, schedule="fused", opts=None, device_inputs=False,
                     share=None):
            self.layers, self.n, self.N = layers, len(layers), layers[0].N
            self.in_dtype = kfac.KFAC_BF16 if dtype_name == "bf16" else kfac.KFAC_F32
            tdt = torch.bfloat16 if dtype_name == "bf16" else torch.float32
            self.spatial_mean = any(L.h_in > 1 for L in layers)   # the conv configurations ask for spatially averaged output gradients
            self.schedule = schedule
            self.subset = list(range(self.n)) if subset is None else list(subset)
            self.Cs = [C for C, _ in bns]
            if share is not None:      # the same tensors in another element type
                self.acts = [x.to(tdt) for x in share.acts]
                self.grads = [x.to(tdt) for x in share.grads]
                self.gws, self.bn_gg, self.bn_gb = share.gws, share.bn_gg, share.bn_gb
            elif device_inputs:
                # timing only: the same distributions drawn on the device (the seeded host arrays of the
                # parity tests take minutes to generate at batch 128)
                g = torch.Generator(device="cuda"); g.manual_seed(1000 * seed_cfg)
                self.acts = [torch.randn(L.N, L.c_in, L.h_in, L.w_in, device="cuda", generator=g).clamp_(min=0).to(tdt) for L in layers]
                self.grads = [(torch.randn(L.N, L.c_out, L.h, L.w, device="cuda", generator=g) * wl.GRAD_SIGMA).to(tdt) for L in layers]
                self.gws = [torch.randn(L.dG, L.dA, device="cuda", generator=g) * wl.GRAD_SIGMA for L in layers]
                self.bn_gg = [torch.randn(self.N, C, device="cuda", generator=g) * wl.GRAD_SIGMA for C in self.Cs]
                self.bn_gb = [torch.randn(self.N, C, device="cuda", generator=g) * wl.GRAD_SIGMA for C in self.Cs]
            else:
                self.acts, self.grads, self.gws = [], [], []
                for i, L in enumerate(layers):
                    s = wl.layer_seed(seed_cfg, i)
                    self.acts.append(torch.from_numpy(wl.make_act(L, s)).cuda().to(tdt))
                    self.grads.append(torch.from_numpy(wl.make_grad_out(L, s)).cuda().to(tdt))
                    self.gws.append(torch.from_numpy(wl.make_grad_W(L, s)).cuda())
                self.bn_gg, self.bn_gb = [], []
                for i, C in enumerate(self.Cs):
                    gg, gb = wl.make_bn_grads(self.N, C, wl.layer_seed(seed_cfg, 100 + i))
                    self.bn_gg.append(torch.from_numpy(gg).cuda())
                    self.bn_gb.append(torch.from_numpy(gb).cuda())
            self.sub_layers = [layers[i] for i in self.subset]
            self.ctx = kfac.Context(layers, self.in_dtype, extra_layer_lists=[self.sub_layers], opts=opts)
            self.A = [torch.zeros(L.dA, L.dA, device="cuda") for L in layers]
            self.G = [torch.zeros(L.dG, L.dG, device="cuda") for L in layers]
            self.Ai = [torch.zeros_like(x) for x in self.A]
            self.Gi = [torch.zeros_like(x) for x in self.G]
            self.U = [torch.zeros(L.dG, L.dA, device="cuda") for L in layers]
            self.info = torch.zeros(2 * self.n, dtype=torch.int32, device="cuda")
            self.F = [torch.zeros(C, 3, device="cuda") for C in self.Cs]
            self.og = [torch.zeros(C, device="cuda") for C in self.Cs]
            self.ob = [torch.zeros(C, device="cuda") for C in self.Cs]

        def stats(self, decay):
            kfac.kfac_stats(self.ctx, self.layers, self.in_dtype, self.acts, self.grads, decay, self.spatial_mean, self.A, self.G)

        def invert(self, idx):
            pick = lambda xs: [xs[i] for i in idx]
            kfac.kfac_invert(self.ctx, pick(self.layers), pick(self.A), pick(self.G), wl.GAMMA, pick(self.Ai), pick(self.Gi),
                             None, self.info)

        def precond(self):
            kfac.kfac_precondition(self.ctx, self.layers, self.Gi, self.Ai, self.gws, self.U)

        def bn(self, decay):
            if self.Cs:
                kfac.bn_unitwise_precondition(self.ctx, self.N, self.Cs, self.bn_gg, self.bn_gb, decay, wl.BN_LAMBDA, self.F,
                                              self.og, self.ob)

        def step(self, decay, idx):
            if self.schedule == "fused":
                mask = [False] * self.n
                for i in idx:
                    mask[i] = True
                kfac.kfac_step(self.ctx, self.layers, self.in_dtype, self.acts, self.grads, decay, self.spatial_mean, self.A,
                               self.G, mask, wl.GAMMA, self.Ai, self.Gi, None, self.info, self.gws, self.U)
            else:
                self.stats(decay)
                self.invert(idx)
                self.precond()
            self.bn(decay)

        def start(self, warmup):
            """Step 0 initialises every running average and every inverse; then the warm-up steps (all untimed)."""
            self.step(0.0, list(range(self.n)))
            torch.cuda.synchronize()
            assert int(self.info.abs().sum().item()) == 0, "a factor was not positive definite"
            for _ in range(warmup):
                self.step(wl.DECAY, self.subset)
            torch.cuda.synchronize()

        def timed(self, steps):
            """K steps between two synchronisations; events between the steps give the per-step spread."""
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
            # The interpreter's heap is collected and frozen first: a full collection over the objects of the imported
            # modules takes 30-40 ms here, and one falling into the timed region would show up as a step of 45 ms.
            # The collector stays enabled.
            import gc
            gc.collect()
            gc.freeze()
            torch.cuda.synchronize()
            ev[0].record()
            for k in range(steps):
                self.step(wl.DECAY, self.subset)
                ev[k + 1].record()
            torch.cuda.synchronize()
            gc.unfreeze()
            per = [ev[k].elapsed_time(ev[k + 1]) for k in range(steps)]
            log("per-step ms: " + " ".join("%.2f" % v for v in per))
            per.sort()
            assert int(self.info.abs().sum().item()) == 0
            return ev[0].elapsed_time(ev[steps]) / steps, per[len(per) // 2], per[0]

        def stage_times(self, reps):
            out = {"stats": 0.0, "invert": 0.0, "precondition": 0.0, "bn": 0.0}
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(5)]
            for _ in range(reps):
                ev[0].record(); self.stats(wl.DECAY)
                ev[1].record(); self.invert(self.subset)
                ev[2].record(); self.precond()
                ev[3].record(); self.bn(wl.DECAY)
                ev[4].record()
                torch.cuda.synchronize()
                for j, k in enumerate(out):
                    out[k] += ev[j].elapsed_time(ev[j + 1]) / reps
            return out

        def close(self):
            self.ctx.close()

    layers = wl.config_layers(cfg)
    N = layers[0].N
    bns = wl.resnet50_layers(N)[1] if cfg >= 4 else []
    n = len(layers)
    stale = cfg == 5

    # ---------------------------------------------------------------- inputs (seeded, host -> HBM)
    t0 = time.time()
    subset = list(wl.stale_subset(n, seed=0)) if stale else list(range(n))
    main_opts = None
    if args.opt:
        fields = {}
        for kv in args.opt:
            k, v = kv.split("=", 1)
            fields[k] = float(v) if k == "chunk_gflop" else int(v)
        main_opts = kfac.options(**fields)
    job = Job(layers, bns, cfg, args.dtype, subset, args.schedule, opts=main_opts)
    log("inputs generated and uploaded in %.1f s" % (time.time() - t0))
    acts, grads, gws, A, G, Ai, Gi, U, info = job.acts, job.grads, job.gws, job.A, job.G, job.Ai, job.Gi, job.U, job.info
    bn_gg, bn_gb, F, og, ob, Cs = job.bn_gg, job.bn_gb, job.F, job.og, job.ob, job.Cs
    sub_layers, spatial_mean, ctx = job.sub_layers, job.spatial_mean, job.ctx
    stats, invert, precond, bn, step = job.stats, job.invert, job.precond, job.bn, job.step

    def sel(xs, idx):
        return [xs[i] for i in idx]

    job.start(args.warmup)

    # ---------------------------------------------------------------- timed region
    ms_per_step, median_ms, min_ms = job.timed(args.steps)
    assert all(bool(torch.isfinite(u).all().item()) for u in U)

    # ---------------------------------------------------------------- per-stage and per-kernel times
    # (the stages one after the other, whatever the schedule of the timed region: with the fused
    # schedule they overlap and have no separate durations)
    args.profile_steps = max(1, args.profile_steps)
    stage_ms = job.stage_times(args.profile_steps)
    # per-kernel durations (HIP events around every launch, on the launch's own stream), also
    # taken with the stages one after the other and on one stream (a context of its own with
    # options.streams = 1): under the fused schedule launches of different streams wait for each
    # other's compute units and an event pair then brackets the wait too
    pjob = Job(layers, bns, cfg, args.dtype, subset, "staged", opts=kfac.options(streams=1), share=job)
    for x, y in zip(pjob.A + pjob.G + pjob.Ai + pjob.Gi, A + G + Ai + Gi):
        x.copy_(y)
    pjob.stats(wl.DECAY); pjob.invert(subset); pjob.precond(); pjob.bn(wl.DECAY)      # warm-up of the new context
    torch.cuda.synchronize()
    kfac.kfac_profile_enable(pjob.ctx, True)
    entries, stage_exec = [], {"stats": [0.0, 0.0], "invert": [0.0, 0.0], "precondition": [0.0, 0.0], "bn": [0.0, 0.0]}
    for _ in range(args.profile_steps):
        for name, call in (("stats", lambda: pjob.stats(wl.DECAY)), ("invert", lambda: pjob.invert(subset)),
                           ("precondition", pjob.precond), ("bn", lambda: pjob.bn(wl.DECAY))):
            call()
            part = kfac.kfac_profile_read(pjob.ctx, 16384)
            entries += part
            stage_exec[name][0] += sum(e["flops"] for e in part) / args.profile_steps    # flops the launches execute
            stage_exec[name][1] += sum(e["bytes"] for e in part) / args.profile_steps    # bytes of the copy-like launches
    kfac.kfac_profile_enable(pjob.ctx, False)
    pjob.close()
    del pjob
    kernels = {}
    for e in entries:
        name = e["kernel"] + ("_tile%d" % (128 if e["variant"] == 0 else 64) if e["kernel"].startswith("gemm_f") or
                              e["kernel"] == "gemm_bf16" else "")
        k = kernels.setdefault(name, {"launches": 0, "ms": 0.0, "flops": 0.0, "bytes": 0.0})
        k["launches"] += 1
        k["ms"] += e["ms"]
        k["flops"] += e["flops"]
        k["bytes"] += e["bytes"]
    for k in kernels.values():
        for f in ("launches", "ms", "flops", "bytes"):
            k[f] /= args.profile_steps
    # the dominant kernel: the one that carries most of the step's arithmetic (if none has any,
    # the one that takes most of the time)
    if any(k["flops"] > 0 for k in kernels.values()):
        dom_name = max(kernels, key=lambda q: kernels[q]["flops"])
    else:
        dom_name = max(kernels, key=lambda q: kernels[q]["ms"])
    dom = kernels[dom_name]
    # HBM traffic per launch of that kernel: measured separately with rocprofv3 --pmc (FETCH_SIZE and
    # WRITE_SIZE, scaled by what they read for the plain copy kernel of the same run) and kept with
    # the profile summaries.  The record says which kernel, how many launches per step and which
    # commit it was measured at; it is only reported if this run's dominant kernel matches it.
    traffic, traffic_source = None, None
    try:
        with open(os.path.join(ROOT, "profiles", "pmc_traffic.json")) as f:
            for rec in json.load(f)["records"]:
                if rec["config"] == cfg and rec["dtype"] == args.dtype and rec["schedule_of_profile"] == "staged":
                    if rec["kernel"] == dom_name and abs(rec["launches_per_step"] - dom["launches"]) < 0.5:
                        traffic = rec["bytes_per_launch"]
                        traffic_source = {"file": "profiles/" + rec["summary"], "measured_at_commit": rec["commit"],
                                          "kernel": rec["kernel"], "launches_per_step": rec["launches_per_step"]}
                    else:
                        traffic_source = {"refused": "the record in profiles/pmc_traffic.json is for %s with %g launches per "
                                                     "step; this run's dominant kernel is %s with %g"
                                                     % (rec["kernel"], rec["launches_per_step"], dom_name, dom["launches"])}
    except (OSError, ValueError, KeyError):
        traffic, traffic_source = None, None
    gemm_dt = "bf16" if dom_name.startswith("gemm_bf16") else "f32"
    split_mode = "split" in dom_name
    # the peak of the pipe the kernel issues on: the fp32 matrix instruction, the bf16 one, or -- fp32 products
    # formed by six bf16 instructions each -- a sixth of the bf16 peak in fp32-equivalent flops
    pipe_peak = PEAK_TFLOPS["bf16"] / 6.0 if split_mode else PEAK_TFLOPS[gemm_dt]
    if dom["flops"] > 0:
        achieved = dom["flops"] / (dom["ms"] * 1e-3) / 1e12
        roofline = {"kernel": dom_name, "bound": "mfma", "achieved": round(achieved, 3), "peak": round(pipe_peak, 1),
                    "unit": "TFLOP/s", "frac": round(achieved / pipe_peak, 4), "traffic": traffic,
                    "traffic_source": traffic_source,
                    "launches_per_step": dom["launches"], "avg_launch_ms": round(dom["ms"] / dom["launches"], 4)}
        if split_mode:
            roofline["frac_of_fp32_mfma_peak"] = round(achieved / PEAK_TFLOPS["f32"], 4)
            roofline["executed_bf16_tflops"] = round(6.0 * achieved, 1)
            roofline["note"] = ("fp32 contraction computed by six bf16 matrix instructions per product block (operands split "
                                "exactly into three bf16 planes, fp32 accumulation, fp32-level accuracy): achieved = fp32 flops "
                                "of the contraction, peak = the dense bf16 peak / 6 (the pipe the kernel issues on); a loop of "
                                "nothing but these matrix instructions on operands with random sign, exponent and mantissa "
                                "reaches about 0.7 of that peak on this GPU (the clock settles at 1.7-1.8 GHz instead of 2.4; "
                                "profiles/mfma_bf16_peak_loop.txt)")
    else:
        achieved = dom["bytes"] / (dom["ms"] * 1e-3) / 1e9
        roofline = {"kernel": dom_name, "bound": "hbm", "achieved": round(achieved, 1), "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": round(achieved / PEAK_HBM_GBS, 4), "traffic": traffic,
                    "traffic_source": traffic_source,
                    "launches_per_step": dom["launches"], "avg_launch_ms": round(dom["ms"] / dom["launches"], 4)}

    fl = {"stats_A": 0.0, "stats_G": 0.0, "inv": 0.0, "precond": 0.0}
    for L in layers:
        for k, v in wl.flops(L).items():
            if k != "inv":
                fl[k] += v
    fl["inv"] = sum(wl.flops(layers[i])["inv"] for i in subset)
    total_flops = sum(fl.values())
    fi_flops = fl["stats_A"] + fl["stats_G"] + fl["inv"]
    fi_ms = stage_ms["stats"] + stage_ms["invert"]
    # which roofline bounds each stage (stages one after the other): the three dense stages against the matrix
    # pipe they issue on (algorithmic flops = the definitions, executed = what the launches multiply out),
    # the unit-wise BatchNorm call against HBM
    mat_peak = PEAK_TFLOPS["bf16"] / 6.0 if (args.dtype == "f32" and split_mode) else PEAK_TFLOPS["f32"]
    roofline_by_stage = {}
    for name, alg in (("stats", fl["stats_A"] + fl["stats_G"]), ("invert", fl["inv"]), ("precondition", fl["precond"])):
        ms = stage_ms[name]
        roofline_by_stage[name] = {"bound": "mfma", "ms": round(ms, 4), "algorithmic_gflop": round(alg / 1e9, 2),
                                   "executed_gflop": round(stage_exec[name][0] / 1e9, 2),
                                   "tflops": round(alg / (ms * 1e-3) / 1e12, 2),
                                   "executed_tflops": round(stage_exec[name][0] / (ms * 1e-3) / 1e12, 2),
                                   "peak": round(mat_peak, 1), "unit": "TFLOP/s",
                                   "frac": round(stage_exec[name][0] / (ms * 1e-3) / 1e12 / mat_peak, 4)}
    if stage_ms["bn"] > 0 and stage_exec["bn"][1] > 0:
        gbs = stage_exec["bn"][1] / (stage_ms["bn"] * 1e-3) / 1e9
        roofline_by_stage["bn"] = {"bound": "hbm", "ms": round(stage_ms["bn"], 4), "gbytes": round(stage_exec["bn"][1] / 1e9, 4),
                                   "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(gbs / PEAK_HBM_GBS, 4),
                                   "note": "one launch of 7 MB: latency, not bandwidth"}

    # ---------------------------------------------------------------- oracle on the host cores
    cpu_baseline = None
    if not args.no_cpu_baseline:
        import oracle
        # the same step on the oracle: every layer once, with the timed step's decay on top of the running averages
        # the GPU holds.  Configurations whose oracle step would take minutes (batch 128) are bounded to the layers
        # that fit about 30 s, cheapest first, and the value is then that sample's time, not a step's.
        order = sorted(range(n), key=lambda i: sum(wl.flops(layers[i]).values()))
        budget_flops = 1.6e12 if N <= 32 else 1.0e12
        sample, acc = [], 0.0
        for i in order:
            f = sum(wl.flops(layers[i]).values())
            if acc + f > budget_flops and sample:
                break
            sample.append(i)
            acc += f
        whole = len(sample) == n
        t_cpu = 0.0
        for i in sample:
            L = layers[i]
            a, g, gw = acts[i].float().cpu().numpy(), grads[i].float().cpu().numpy(), gws[i].cpu().numpy()
            A0, G0 = A[i].cpu().numpy(), G[i].cpu().numpy()
            t1 = time.perf_counter()
            Ar, Gr = oracle.kfac_stats(tuple(L), a, g, wl.DECAY, spatial_mean, A0, G0)
            if i in subset:
                Air, Gir, _, _ = oracle.kfac_invert(Ar, Gr, wl.GAMMA)
            else:
                Air, Gir = Ai[i].cpu().numpy(), Gi[i].cpu().numpy()
            oracle.kfac_precondition(Gir, Air, gw)
            t_cpu += time.perf_counter() - t1
        if Cs and whole:
            t1 = time.perf_counter()
            for gg, gb in zip(bn_gg, bn_gb):
                oracle.bn_unitwise_precondition(gg.cpu().numpy(), gb.cpu().numpy(), wl.DECAY, wl.BN_LAMBDA)
            t_cpu += time.perf_counter() - t1
        cpu_baseline = {"value": round(t_cpu * 1e3, 1), "unit": "ms", "cores": oracle.num_threads(), "kind": "oracle",
                        "sample": ("one whole step of the float64 oracle, measured: all %d layers (factors with decay %.2f, "
                                   "inverses of the %d refreshed layers, preconditioning) and the %d BatchNorm layers; "
                                   "%.1f GFLOP algorithmic" % (n, wl.DECAY, len(subset), len(Cs), total_flops / 1e9)) if whole else
                                  ("NOT a whole step: the %d cheapest of %d layers (%.1f of %.1f GFLOP algorithmic), measured, "
                                   "no extrapolation" % (len(sample), n, acc / 1e9, total_flops / 1e9))}

    staleness = adaptive = layout_obj = packing = updating = full_bn = split_obj = other_configs = None
    extras = not args.no_extras      # the calls beside the step are left out of profiler runs of the step itself
    if extras:
        # ---------------------------------------------------------------- beside the step: staleness of the factors
        # (Sec. 4.3: what a refresh under Algorithm 1 adds -- every factor against its two predecessors)
        dims = [L.dA for L in layers] + [L.dG for L in layers]
        X = A + G
        P = [x * 1.02 for x in X]
        Q = [x * 0.95 for x in X]
        ratios = torch.zeros(2 * len(dims), dtype=torch.float64, device="cuda")
        kfac.kfac_staleness(ctx, dims, X, P, Q, ratios)
        torch.cuda.synchronize()
        s0, s1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s0.record()
        for _ in range(10):
            kfac.kfac_staleness(ctx, dims, X, P, Q, ratios)
        s1.record()
        torch.cuda.synchronize()
        stale_ms = s0.elapsed_time(s1) / 10
        stale_bytes = 12.0 * sum(d * d for d in dims)
        r = ratios.cpu().numpy().reshape(-1, 2)
        assert abs(float(r[:, 0].max()) - 0.02 / 1.02) < 1e-4 and abs(float(r[:, 1].min()) - 0.05 / 0.95) < 1e-4
        staleness = {"matrices": len(dims), "ms": round(stale_ms, 4), "gbytes": round(stale_bytes / 1e9, 3),
                     "gbs": round(stale_bytes / (stale_ms * 1e-3) / 1e9, 1),
                     "frac_of_hbm_peak": round(stale_bytes / (stale_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                     "note": "kfac_staleness over all factors of the configuration against two predecessors each "
                             "(12 bytes per element); not part of the timed step"}
        del P, Q



        # ------------------------------------------------------------ beside the step: the fp32 matrix instruction
        # (options.fp32_products = KFAC_PRODUCTS_FP32_MFMA: every product by v_mfma_f32_32x32x2_f32 instead of six bf16
        # instructions on split operands; the same step on a context of its own, its results compared with those of
        # the default mode)
        split_obj = None
        if args.dtype == "f32":
            U_ref = [u.clone() for u in U]
            A_ref = [a.clone() for a in A]
            job.ctx = kfac.Context(layers, in_dtype, extra_layer_lists=[sub_layers],
                                   opts=kfac.options(fp32_products=kfac.KFAC_PRODUCTS_FP32_MFMA))
            step(wl.DECAY, subset)
            torch.cuda.synchronize()
            s0.record()
            for _ in range(args.steps):
                step(wl.DECAY, subset)
            s1.record()
            torch.cuda.synchronize()
            split_ms = s0.elapsed_time(s1) / args.steps
            ev3 = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
            ev3[0].record(); stats(wl.DECAY)
            ev3[1].record(); invert(subset)
            ev3[2].record(); precond()
            ev3[3].record()
            torch.cuda.synchronize()
            assert int(info.abs().sum().item()) == 0
            # the running averages have moved on by a few steps of the same inputs; with decay they stay within
            # rounding of each other, so the two modes' results are comparable
            du = max(float((u - r).abs().max() / r.abs().max()) for u, r in zip(U, U_ref))
            da = max(float((a - r).abs().max() / r.abs().max()) for a, r in zip(A, A_ref))
            split_obj = {"ms_per_step": round(split_ms, 4),
                         "stage_ms": {"stats": round(ev3[0].elapsed_time(ev3[1]), 4),
                                      "invert": round(ev3[1].elapsed_time(ev3[2]), 4),
                                      "precondition": round(ev3[2].elapsed_time(ev3[3]), 4)},
                         "max_rel_diff_to_default": {"A": da, "U": du},
                         "note": "the timed step on a context with fp32_products = KFAC_PRODUCTS_FP32_MFMA (every product of "
                                 "the GEMM kernel by the fp32 matrix instruction); not the mode of the headline value"}
            job.ctx.close()
            job.ctx = ctx
            step(wl.DECAY, subset)       # the buffers back to the default mode's results
            torch.cuda.synchronize()

        # ------------------------------------------------------------ beside the step: Algorithm 1 over a run of steps
        # (Sec. 4.3: every statistic is rebuilt only when its own interval says so; a layer is re-inverted when one of
        # its factors was rebuilt; every step preconditions all gradients.  The inputs are the same in every step, so
        # the statistics are stationary: the most favourable case, refreshes at the Fibonacci steps 1 2 3 5 8 13 21 34.)
        T = 34
        actx = kfac.Context(layers, in_dtype, workspace_bytes=2 * kfac.kfac_workspace_bytes(layers, in_dtype))
        Ax = [torch.zeros_like(x) for x in A]
        Gx = [torch.zeros_like(x) for x in G]
        Xs = Ax + Gx
        P1 = [None] * (2 * n)
        P2 = [None] * (2 * n)
        states = kfac.kfac_refresh_init(2 * n)
        rat = torch.zeros(4 * n, dtype=torch.float64, device="cuda")
        refreshed_stats = 0
        refresh_steps = []
        torch.cuda.synchronize()
        t_begin = time.perf_counter()
        for t in range(1, T + 1):
            due = [i for i in range(2 * n) if kfac.kfac_refresh_due(states[i], t)]
            if due:
                dueset = set(due)
                kfac.kfac_stats(actx, layers, in_dtype, [acts[l] if l in dueset else None for l in range(n)],
                                [grads[l] if n + l in dueset else None for l in range(n)],
                                0.0 if t == 1 else wl.DECAY, spatial_mean, Ax, Gx)
                have1 = [i for i in due if P1[i] is not None]
                if have1:
                    kfac.kfac_staleness(actx, [dims[i] for i in have1], [Xs[i] for i in have1], [P1[i] for i in have1],
                                        [P2[i] for i in have1], rat)
                    r = rat[:2 * len(have1)].cpu().numpy().reshape(-1, 2)      # the host decides: one sync per refresh
                ratio = {i: (float("inf"), float("inf")) for i in due}
                for j, i in enumerate(have1):
                    ratio[i] = (float(r[j, 0]), float(r[j, 1]))
                for i in due:
                    kfac.kfac_refresh_advance(states[i], ratio[i][0], ratio[i][1], 0.1)
                    P2[i] = P1[i]                                              # X_-2 <- X_-1 <- X (copies, as Algorithm 1 keeps them)
                    P1[i] = Xs[i].clone()
                inv = sorted({i % n for i in due})
                kfac.kfac_invert(actx, sel(layers, inv), sel(Ax, inv), sel(Gx, inv), wl.GAMMA, sel(Ai, inv), sel(Gi, inv),
                                 None, None)
                refreshed_stats += len(due)
                refresh_steps.append(t)
            kfac.kfac_precondition(actx, layers, Gi, Ai, gws, U)
        torch.cuda.synchronize()
        adaptive_ms = (time.perf_counter() - t_begin) * 1e3 / T
        adaptive = {"steps": T, "ms_per_step": round(adaptive_ms, 4), "refresh_steps": refresh_steps,
                    "statistics_rebuilt_fraction": round(refreshed_stats / (2.0 * n * T), 4),
                    "note": "Algorithm 1 with alpha = 0.1 driving kfac_stats (due statistics only), kfac_staleness, "
                            "kfac_invert (layers with a rebuilt factor) and kfac_precondition (all layers) over %d steps "
                            "of identical inputs (stationary statistics, the most favourable case); wall clock including "
                            "the host's decisions and the copies of X_-1, X_-2; not part of the timed step" % T}
        del Ax, Gx, Xs, P1, P2
        actx.close()


        # ------------------------------------------------------------ beside the step: inputs that arrive in NHWC
        # (Sec. 5.2: converted to the layout the statistics kernels read; contents do not matter for the timing, so
        # the step's own tensors serve as the source)
        layout_obj = {}
        tot_ms = 0.0
        for name, which, srcs in (("activations", 0, acts), ("output_gradients", 1, grads)):
            dsts = [torch.empty_like(x) for x in srcs]
            kfac.kfac_nhwc_to_nchw(ctx, layers, which, in_dtype, srcs, dsts)
            torch.cuda.synchronize()
            s0.record()
            for _ in range(5):
                kfac.kfac_nhwc_to_nchw(ctx, layers, which, in_dtype, srcs, dsts)
            s1.record()
            torch.cuda.synchronize()
            ms = s0.elapsed_time(s1) / 5
            nbytes = 2.0 * sum(x.numel() * x.element_size() for x in srcs)
            layout_obj[name] = {"ms": round(ms, 4), "gbytes": round(nbytes / 1e9, 3), "gbs": round(nbytes / (ms * 1e-3) / 1e9, 1),
                                "frac_of_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}
            tot_ms += ms
            del dsts
        layout_obj["ms"] = round(tot_ms, 4)
        layout_obj["note"] = ("kfac_nhwc_to_nchw over all activations and all output gradients of the configuration "
                              "(every element read once and written once): what a caller with NHWC tensors pays in "
                              "front of the step when it converts everything; not part of the timed step")
        # the same tensors in NHWC order handed to kfac_stats_nhwc / kfac_step_nhwc: pointwise layers and output
        # gradients are contracted in place, the rest is converted inside the call
        a_t = [x.permute(0, 2, 3, 1).contiguous() for x in acts]
        g_t = [x.permute(0, 2, 3, 1).contiguous() for x in grads]
        mask_all = [i in subset for i in range(n)]
        in_place = {}
        for name, call_nchw, call_nhwc in (
                ("stats", lambda: kfac.kfac_stats(ctx, layers, in_dtype, acts, grads, wl.DECAY, spatial_mean, A, G),
                 lambda: kfac.kfac_stats(ctx, layers, in_dtype, a_t, g_t, wl.DECAY, spatial_mean, A, G, nhwc=True)),
                ("step", lambda: kfac.kfac_step(ctx, layers, in_dtype, acts, grads, wl.DECAY, spatial_mean, A, G, mask_all,
                                                wl.GAMMA, Ai, Gi, None, info, gws, U),
                 lambda: kfac.kfac_step(ctx, layers, in_dtype, a_t, g_t, wl.DECAY, spatial_mean, A, G, mask_all,
                                        wl.GAMMA, Ai, Gi, None, info, gws, U, nhwc=True))):
            for tag, call in (("nchw", call_nchw), ("nhwc", call_nhwc)):
                for _ in range(2):
                    call()
                torch.cuda.synchronize()
                s0.record()
                for _ in range(5):
                    call()
                s1.record()
                torch.cuda.synchronize()
                in_place["%s_ms_%s" % (name, tag)] = round(s0.elapsed_time(s1) / 5, 4)
        in_place["note"] = ("kfac_stats / kfac_step on the step's tensors in NCHW order and kfac_stats_nhwc / kfac_step_nhwc on "
                            "the same tensors in NHWC order (same results up to the order of the sums); five calls each, back "
                            "to back; not part of the timed step")
        layout_obj["in_place"] = in_place
        del a_t, g_t

        # ---------------------------------------------------------------- beside the step: packing of the factors
        # (Sec. 5.2: upper triangles of all factors into one send buffer, and back)
        total = kfac.kfac_packed_elems(dims)
        full_bytes = 4.0 * sum(d * d for d in dims)
        packing = {"matrices": len(dims), "packed_elements": total}
        for tname, ttype, tdtype, esize in (("f32", kfac.KFAC_F32, torch.float32, 4), ("bf16", kfac.KFAC_BF16, torch.bfloat16, 2)):
            buf = torch.empty(total, dtype=tdtype, device="cuda")
            back = [torch.empty_like(x) for x in X]
            for name, call, nbytes in (("pack", lambda: kfac.kfac_pack_upper(ctx, dims, X, ttype, buf), total * (4.0 + esize)),
                                       ("unpack", lambda: kfac.kfac_unpack_upper(ctx, dims, ttype, buf, back), total * esize + full_bytes)):
                call()
                torch.cuda.synchronize()
                s0.record()
                for _ in range(10):
                    call()
                s1.record()
                torch.cuda.synchronize()
                ms = s0.elapsed_time(s1) / 10
                packing["%s_%s" % (name, tname)] = {"ms": round(ms, 4), "gbytes": round(nbytes / 1e9, 3),
                                                   "gbs": round(nbytes / (ms * 1e-3) / 1e9, 1),
                                                   "frac_of_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}
            del buf, back
        packing["note"] = ("kfac_pack_upper / kfac_unpack_upper over all factors of the configuration; bytes: the triangle "
                           "read and written (pack), the triangle read and the whole matrix written (unpack); not part of "
                           "the timed step")

        # ---------------------------------------------------------------- beside the step: the parameter update
        # (Sec. 6.2, 6.3: w <- w - eta U + m v for all layers, then the rescaling to norm sqrt(2 d_out))
        n_w = sum(L.dA * L.dG for L in layers)
        Wt = [torch.randn(L.dG, L.dA, device="cuda") * (2.0 / L.dA) ** 0.5 for L in layers]
        Wp = [w.clone() for w in Wt]
        updating = {"layers": n, "weights": n_w}
        for name, resc, per_elem in (("update", False, 20.0), ("update_rescale", True, 28.0)):
            kfac.kfac_update_weights(ctx, layers, U, 1e-3, 0.9, resc, 1e-9, Wt, Wp)
            torch.cuda.synchronize()
            s0.record()
            for _ in range(10):
                kfac.kfac_update_weights(ctx, layers, U, 1e-3, 0.9, resc, 1e-9, Wt, Wp)
            s1.record()
            torch.cuda.synchronize()
            ms = s0.elapsed_time(s1) / 10
            updating[name] = {"ms": round(ms, 4), "gbytes": round(per_elem * n_w / 1e9, 3),
                              "gbs": round(per_elem * n_w / (ms * 1e-3) / 1e9, 1),
                              "frac_of_hbm_peak": round(per_elem * n_w / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}
        assert all(abs(float(w.double().norm()) - (2.0 * L.dG) ** 0.5) < 1e-4 * (2.0 * L.dG) ** 0.5 for w, L in zip(Wt, layers))
        updating["note"] = ("kfac_update_weights over all layers of the configuration with the preconditioned gradients of "
                            "the step; 20 bytes per weight for the update (U, w, w_prev read; w, w_prev written), 8 more for "
                            "the rescaling; not part of the timed step")
        del Wt, Wp

        # ---------------------------------------------------------------- beside the step: BatchNorm with the whole-layer Fisher
        # (Sec. 4.2 / Sec. 7 "fullBN": dense 2c x 2c Fisher per BatchNorm layer instead of the unit-wise 2 x 2 blocks)
        if Cs:
            bctx = kfac.Context(layers[:1], workspace_bytes=kfac.bn_full_workspace_bytes(N, Cs))
            Ff = [torch.zeros(2 * C, 2 * C, device="cuda") for C in Cs]
            Ffi = [torch.zeros(2 * C, 2 * C, device="cuda") for C in Cs]
            binfo = torch.zeros(len(Cs), dtype=torch.int32, device="cuda")
            kfac.bn_full_precondition(bctx, N, Cs, bn_gg, bn_gb, 0.0, wl.BN_LAMBDA, Ff, Ffi, og, ob, info=binfo)
            torch.cuda.synchronize()
            assert int(binfo.abs().sum().item()) == 0
            s0.record()
            for _ in range(3):
                kfac.bn_full_precondition(bctx, N, Cs, bn_gg, bn_gb, wl.DECAY, wl.BN_LAMBDA, Ff, Ffi, og, ob, info=binfo)
            s1.record()
            torch.cuda.synchronize()
            full_ms = s0.elapsed_time(s1) / 3
            kfac.kfac_profile_enable(bctx, True)
            kfac.bn_full_precondition(bctx, N, Cs, bn_gg, bn_gb, wl.DECAY, wl.BN_LAMBDA, Ff, Ffi, og, ob, info=binfo)
            torch.cuda.synchronize()
            parts = {}
            for e in kfac.kfac_profile_read(bctx, 16384):
                key = {"bn_full": "bn_full_pass%d" % e["variant"]}.get(e["kernel"], "inversion")
                parts[key] = parts.get(key, 0.0) + e["ms"]
            kfac.kfac_profile_enable(bctx, False)
            s0.record()
            for _ in range(10):
                bn(wl.DECAY)
            s1.record()
            torch.cuda.synchronize()
            unit_ms = s0.elapsed_time(s1) / 10
            inv_flops = float(sum((2.0 * C) ** 3 for C in Cs))
            full_bn = {"bn_layers": len(Cs), "ms": round(full_ms, 4), "unit_wise_ms": round(unit_ms, 4),
                       "fisher_gbytes": round(4.0 * sum((2 * C) ** 2 for C in Cs) / 1e9, 3),
                       "inverse_gflop": round(inv_flops / 1e9, 1),
                       "inverse_tflops": round(inv_flops / (full_ms * 1e-3) / 1e12, 2),
                       "serial_ms_by_part": {k: round(v, 4) for k, v in sorted(parts.items())},
                       "note": "bn_full_precondition over all BatchNorm layers of the configuration, every layer inverted; "
                               "unit_wise_ms is bn_unitwise_precondition on the same gradients; serial_ms_by_part comes from "
                               "a profiled call whose launches run one after the other; not part of the timed step"}
            del Ff, Ffi
            bctx.close()

    if extras and cfg == 4 and args.dtype == "f32":
        # ------------------------------------------------------------ beside the headline: the other configurations
        # (short runs of the same step: 2 warm-up + 5 timed, stages once; configuration 4 with bf16 inputs reuses the
        # tensors of this run rounded to bf16; batch 128 and the v1.5 layer set draw their inputs on the device)
        other_configs = {}

        def quick(name, jb, note):
            jb.start(2)
            mean, med, mn = jb.timed(5)
            st = jb.stage_times(1)
            fls = {"stats": sum(wl.flops(L)["stats_A"] + wl.flops(L)["stats_G"] for L in jb.layers),
                   "invert": sum(wl.flops(jb.layers[i])["inv"] for i in jb.subset),
                   "precondition": sum(wl.flops(L)["precond"] for L in jb.layers)}
            other_configs[name] = {"ms_per_step": round(mean, 4), "median_ms": round(med, 4), "min_ms": round(mn, 4),
                                   "stage_ms": {k: round(v, 4) for k, v in st.items()},
                                   "algorithmic_gflop": {k: round(v / 1e9, 3) for k, v in fls.items()},
                                   "step_tflops": round(sum(fls.values()) / (mean * 1e-3) / 1e12, 3),
                                   "layers": jb.n, "batch": jb.N, "inverted_layers": len(jb.subset), "note": note}
            jb.close()

        quick("config4_bf16_inputs", Job(layers, bns, 4, "bf16", None, "fused", share=job),
              "configuration 4 with bf16 activations / output gradients (statistics from bf16 operands; inversion and "
              "preconditioning in fp32)")
        for c, note in ((1, "single FC layer 64->32, batch 32: launch-latency bound"),
                        (2, "one conv3x3 64->64 at 56x56, batch 32"),
                        (3, "conv3x3 512->512 at 7x7 (A 4609x4609) plus FC 2048->1000, batch 32")):
            quick("config%d" % c, Job(wl.config_layers(c), [], c, "f32"), note)
        l15, bn15 = wl.resnet50_layers(32, "v1.5")
        quick("resnet50_v1_5_batch32", Job(l15, bn15, 6, "f32", device_inputs=True),
              "the v1.5 variant of the layer set (stride on the 3x3 of stages 3-5: three 3x3 / stride-2 layers on the patch "
              "path with contractions up to 25 088), inputs drawn on the device")
        l5 = wl.config_layers(5)
        quick("config5", Job(l5, wl.resnet50_layers(128)[1], 5, "f32", list(wl.stale_subset(len(l5), seed=0)), device_inputs=True),
              "full layer set at batch 128, inverses refreshed for the seeded 25 % subset, inputs drawn on the device")

    out = {
        "metric": "K-FAC step ms for ResNet-50 layer set; factor+inverse TFLOP/s vs MFMA peak",
        "value": round(ms_per_step, 4),
        "unit": "ms",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "median_ms": round(median_ms, 4),
        "min_ms": round(min_ms, 4),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": args.dtype,
        "data": "synthetic",
        "config": {"workload": "config %d: %s" % (cfg, {
            1: "single FC layer 64->32, batch 32",
            2: "one ResNet-50 conv3x3 64->64 at 56x56, batch 32",
            3: "largest ResNet-50 conv3x3 512->512 at 7x7 plus FC 2048->1000, batch 32",
            4: "full ResNet-50 layer set (53 conv + 1 FC + 53 BatchNorm), batch 32",
            5: "full ResNet-50 layer set, batch 128, inverses refreshed for a seeded 25% subset"}[cfg]),
            "layers": n, "bn_layers": len(Cs), "batch": N, "inverted_layers": len(subset),
            "g_spatial_mean": bool(spatial_mean), "schedule": args.schedule,
            "fp32_products": ("six bf16 matrix instructions on operands split exactly into three bf16 planes, fp32 "
                              "accumulation (fp32-level accuracy; the library's default; object fp32_instruction: the same "
                              "step with the fp32 matrix instruction)")},
        "algorithmic_gflop": {k: round(v / 1e9, 2) for k, v in fl.items()},
        "step_tflops": round(total_flops / (ms_per_step * 1e-3) / 1e12, 3),
        "factor_inverse_tflops": round(fi_flops / (fi_ms * 1e-3) / 1e12, 3),
        "factor_inverse_frac_of_fp32_mfma_peak": round(fi_flops / (fi_ms * 1e-3) / 1e12 / PEAK_TFLOPS["f32"], 4),
        "stage_ms": {k: round(v, 4) for k, v in stage_ms.items()},
        "stage_ms_note": "stages run one after the other (separate calls); the fused schedule overlaps them",
        "flops_note": "algorithmic_gflop, step_tflops and factor_inverse_tflops count the flops of the definitions "
                      "(patch Gram matrices, n^3 per inverse); kernels[..].tflops and roofline count the flops the "
                      "launches execute (3x3 layers use 13 displaced correlations instead of the patch Gram matrix)",
        "kernels": {k: {"launches": v["launches"], "ms": round(v["ms"], 4),
                        "tflops": round(v["flops"] / (v["ms"] * 1e-3) / 1e12, 3) if v["flops"] else None,
                        "gbs": round(v["bytes"] / (v["ms"] * 1e-3) / 1e9, 1) if v["bytes"] else None}
                    for k, v in sorted(kernels.items())},
        "roofline": roofline,
        "roofline_by_stage": roofline_by_stage,
        "cpu_baseline": cpu_baseline,
        "configs": other_configs,
        "staleness": staleness,
        "adaptive_refresh": adaptive,
        "nhwc_inputs": layout_obj,
        "packing": packing,
        "update": updating,
        "full_bn": full_bn,
        "fp32_instruction": split_obj,
    }
    ctx.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()

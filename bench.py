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
    layers = wl.config_layers(cfg)
    N = layers[0].N
    bns = wl.resnet50_layers(N)[1] if cfg >= 4 else []
    in_dtype = kfac.KFAC_BF16 if args.dtype == "bf16" else kfac.KFAC_F32
    tdt = torch.bfloat16 if args.dtype == "bf16" else torch.float32
    spatial_mean = cfg >= 2          # the conv configurations ask for spatially averaged output gradients
    stale = cfg == 5
    n = len(layers)

    # ---------------------------------------------------------------- inputs (seeded, host -> HBM)
    t0 = time.time()
    acts, grads, gws = [], [], []
    for i, L in enumerate(layers):
        s = wl.layer_seed(cfg, i)
        a, g = wl.make_act(L, s), wl.make_grad_out(L, s)
        acts.append(torch.from_numpy(a).cuda().to(tdt))
        grads.append(torch.from_numpy(g).cuda().to(tdt))
        gws.append(torch.from_numpy(wl.make_grad_W(L, s)).cuda())
        del a, g
    bn_gg, bn_gb = [], []
    for i, (C, _) in enumerate(bns):
        gg, gb = wl.make_bn_grads(N, C, wl.layer_seed(cfg, 100 + i))
        bn_gg.append(torch.from_numpy(gg).cuda())
        bn_gb.append(torch.from_numpy(gb).cuda())
    log("inputs generated and uploaded in %.1f s" % (time.time() - t0))

    subset = list(wl.stale_subset(n, seed=0)) if stale else list(range(n))
    sub_layers = [layers[i] for i in subset]
    ctx = kfac.Context(layers, in_dtype, extra_layer_lists=[sub_layers])
    A = [torch.zeros(L.dA, L.dA, device="cuda") for L in layers]
    G = [torch.zeros(L.dG, L.dG, device="cuda") for L in layers]
    Ai = [torch.zeros_like(x) for x in A]
    Gi = [torch.zeros_like(x) for x in G]
    U = [torch.zeros(L.dG, L.dA, device="cuda") for L in layers]
    info = torch.zeros(2 * n, dtype=torch.int32, device="cuda")
    Cs = [C for C, _ in bns]
    F = [torch.zeros(C, 3, device="cuda") for C in Cs]
    og = [torch.zeros(C, device="cuda") for C in Cs]
    ob = [torch.zeros(C, device="cuda") for C in Cs]

    def sel(xs, idx):
        return [xs[i] for i in idx]

    def stats(decay):
        kfac.kfac_stats(ctx, layers, in_dtype, acts, grads, decay, spatial_mean, A, G)

    def invert(idx):
        kfac.kfac_invert(ctx, sel(layers, idx), sel(A, idx), sel(G, idx), wl.GAMMA, sel(Ai, idx), sel(Gi, idx),
                         None, info)

    def precond():
        kfac.kfac_precondition(ctx, layers, Gi, Ai, gws, U)

    def bn(decay):
        if Cs:
            kfac.bn_unitwise_precondition(ctx, N, Cs, bn_gg, bn_gb, decay, wl.BN_LAMBDA, F, og, ob)

    def step(decay, idx):
        if args.schedule == "fused":
            mask = [False] * n
            for i in idx:
                mask[i] = True
            kfac.kfac_step(ctx, layers, in_dtype, acts, grads, decay, spatial_mean, A, G, mask, wl.GAMMA, Ai, Gi,
                           None, info, gws, U)
        else:
            stats(decay)
            invert(idx)
            precond()
        bn(decay)

    # step 0 initialises every running average and every inverse (untimed)
    step(0.0, list(range(n)))
    torch.cuda.synchronize()
    assert int(info.abs().sum().item()) == 0, "a factor was not positive definite"
    for _ in range(args.warmup):
        step(wl.DECAY, subset)
    torch.cuda.synchronize()

    # ---------------------------------------------------------------- timed region
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(args.steps):
        step(wl.DECAY, subset)
    e1.record()
    torch.cuda.synchronize()
    ms_per_step = e0.elapsed_time(e1) / args.steps
    assert int(info.abs().sum().item()) == 0
    assert all(bool(torch.isfinite(u).all().item()) for u in U)

    # ---------------------------------------------------------------- per-stage and per-kernel times
    # (the stages one after the other, whatever the schedule of the timed region: with the fused
    # schedule they overlap and have no separate durations)
    stage_ms = {"stats": 0.0, "invert": 0.0, "precondition": 0.0, "bn": 0.0}
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(5)]
    args.profile_steps = max(1, args.profile_steps)
    for _ in range(args.profile_steps):
        ev[0].record(); stats(wl.DECAY)
        ev[1].record(); invert(subset)
        ev[2].record(); precond()
        ev[3].record(); bn(wl.DECAY)
        ev[4].record()
        torch.cuda.synchronize()
        for j, k in enumerate(stage_ms):
            stage_ms[k] += ev[j].elapsed_time(ev[j + 1]) / args.profile_steps
    # per-kernel durations (HIP events around every launch, on the launch's own stream), also
    # taken with the stages one after the other: under the fused schedule launches of different
    # streams wait for each other's compute units and an event pair then brackets the wait too
    # ... and on one stream (a context of its own, created with KFAC_INV_STREAMS=1): launches of
    # concurrent inversion chains would otherwise stretch each other's event pairs
    prev = os.environ.get("KFAC_INV_STREAMS")
    os.environ["KFAC_INV_STREAMS"] = "1"
    main_ctx, ctx = ctx, kfac.Context(layers, in_dtype, extra_layer_lists=[sub_layers])
    if prev is None:
        del os.environ["KFAC_INV_STREAMS"]
    else:
        os.environ["KFAC_INV_STREAMS"] = prev
    stats(wl.DECAY); invert(subset); precond(); bn(wl.DECAY)      # warm-up of the new context
    torch.cuda.synchronize()
    kfac.kfac_profile_enable(ctx, True)
    for _ in range(args.profile_steps):
        stats(wl.DECAY)
        invert(subset)
        precond()
        bn(wl.DECAY)
    entries = kfac.kfac_profile_read(ctx, 16384)
    kfac.kfac_profile_enable(ctx, False)
    ctx.close()
    ctx = main_ctx
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
    # HBM traffic per launch of that kernel: measured separately with rocprofv3 --pmc (FETCH_SIZE
    # and WRITE_SIZE, scaled by what they read for the plain copy kernel of the same run) and
    # kept with the profile summaries; null if no measurement covers this configuration
    traffic = None
    try:
        with open(os.path.join(ROOT, "profiles", "pmc_traffic.json")) as f:
            for rec in json.load(f)["records"]:
                if rec["config"] == cfg and rec["dtype"] == args.dtype and rec["kernel"] == dom_name:
                    traffic = rec["bytes_per_launch"]
    except (OSError, ValueError, KeyError):
        traffic = None
    gemm_dt = "bf16" if dom_name.startswith("gemm_bf16") else "f32"
    if dom["flops"] > 0:
        achieved = dom["flops"] / (dom["ms"] * 1e-3) / 1e12
        roofline = {"kernel": dom_name, "bound": "mfma", "achieved": round(achieved, 3), "peak": PEAK_TFLOPS[gemm_dt],
                    "unit": "TFLOP/s", "frac": round(achieved / PEAK_TFLOPS[gemm_dt], 4), "traffic": traffic,
                    "launches_per_step": dom["launches"], "avg_launch_ms": round(dom["ms"] / dom["launches"], 4)}
        if "split" in dom_name:
            # fp32 operands, every product formed from three bf16 planes per operand by six bf16 matrix
            # instructions: achieved counts the fp32 flops of the contraction and is set against the fp32 peak
            # (it can exceed it); the instructions executed are six times that, set against the bf16 peak
            roofline["executed_bf16_tflops"] = round(6.0 * achieved, 1)
            roofline["frac_of_bf16_peak_executed"] = round(6.0 * achieved / PEAK_TFLOPS["bf16"], 4)
            roofline["note"] = ("fp32 contraction computed by six bf16 matrix instructions per product block (operands "
                                "split exactly into three bf16 planes, fp32 accumulation, fp32-level accuracy): achieved "
                                "= fp32 flops of the contraction, peak = the fp32 MFMA peak; KFAC_SPLIT=0 selects the "
                                "fp32 instruction (object fp32_instruction)")
    else:
        achieved = dom["bytes"] / (dom["ms"] * 1e-3) / 1e9
        roofline = {"kernel": dom_name, "bound": "hbm", "achieved": round(achieved, 1), "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": round(achieved / PEAK_HBM_GBS, 4), "traffic": traffic,
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

    # ---------------------------------------------------------------- oracle on the host cores (bounded sample)
    cpu_baseline = None
    if not args.no_cpu_baseline:
        import oracle
        # a sample of layers whose oracle time stays within tens of seconds
        budget_flops = 500e9
        order = sorted(range(n), key=lambda i: sum(wl.flops(layers[i]).values()))
        sample, acc = [], 0.0
        for i in order:
            f = sum(wl.flops(layers[i]).values())
            if acc + f > budget_flops and sample:
                break
            sample.append(i)
            acc += f
        t_cpu = 0.0
        worst = 0.0
        for i in sample:
            L = layers[i]
            s = wl.layer_seed(cfg, i)
            a, g, gw = acts[i].float().cpu().numpy(), grads[i].float().cpu().numpy(), gws[i].cpu().numpy()
            t1 = time.perf_counter()
            Ar, Gr = oracle.kfac_stats(tuple(L), a, g, 0.0, spatial_mean, None, None)
            Air, Gir, _, _ = oracle.kfac_invert(Ar, Gr, wl.GAMMA)
            oracle.kfac_precondition(Gir, Air, gw)
            t_cpu += time.perf_counter() - t1
        est_ms = t_cpu * 1e3 * total_flops / acc
        cpu_baseline = {"value": round(est_ms, 1), "unit": "ms", "cores": oracle.num_threads(), "kind": "oracle",
                        "sample": "float64 oracle on the %d cheapest layers of the set (%.1f GFLOP algorithmic, "
                                  "%.2f s measured), scaled to the whole step by algorithmic flops (x%.1f)"
                                  % (len(sample), acc / 1e9, t_cpu, total_flops / acc)}

    staleness = adaptive = layout_obj = packing = updating = full_bn = split_obj = None
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
        # (KFAC_SPLIT=0: every product by v_mfma_f32_32x32x2_f32 instead of six bf16 instructions on split operands;
        # the same step on a context of its own, its results compared with those of the default mode)
        split_obj = None
        if args.dtype == "f32":
            U_ref = [u.clone() for u in U]
            A_ref = [a.clone() for a in A]
            prev_split = os.environ.get("KFAC_SPLIT")
            os.environ["KFAC_SPLIT"] = "0"
            main_ctx2, ctx = ctx, kfac.Context(layers, in_dtype, extra_layer_lists=[sub_layers])
            if prev_split is None:
                del os.environ["KFAC_SPLIT"]
            else:
                os.environ["KFAC_SPLIT"] = prev_split
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
                         "note": "the timed step with KFAC_SPLIT=0 (every product of the GEMM kernel by the fp32 matrix "
                                 "instruction); not the mode of the headline value"}
            ctx.close()
            ctx = main_ctx2
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
                              "front of the step; not part of the timed step")

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

    out = {
        "metric": "K-FAC step ms for ResNet-50 layer set; factor+inverse TFLOP/s vs MFMA peak",
        "value": round(ms_per_step, 4),
        "unit": "ms",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
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
            "fp32_products": ("fp32 matrix instruction" if os.environ.get("KFAC_SPLIT", "1") == "0" else
                              "six bf16 matrix instructions on operands split exactly into three bf16 planes, fp32 "
                              "accumulation (fp32-level accuracy; KFAC_SPLIT=0 selects the fp32 matrix instruction)")},
        "algorithmic_gflop": {k: round(v / 1e9, 2) for k, v in fl.items()},
        "step_tflops": round(total_flops / (ms_per_step * 1e-3) / 1e12, 3),
        "factor_inverse_tflops": round(fi_flops / (fi_ms * 1e-3) / 1e12, 3),
        "factor_inverse_frac_of_mfma_peak": round(fi_flops / (fi_ms * 1e-3) / 1e12 / PEAK_TFLOPS[args.dtype if args.dtype == "f32" else "f32"], 4),
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
        "cpu_baseline": cpu_baseline,
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

#!/usr/bin/env python3
"""Benchmark of the full K-FAC second-order update on one MI355X.

A "step" is one pass of the whole hot path over all layers of the workload:
factor construction (im2col + SYRK + running average), damped inversion of
every A and G, and two-sided preconditioning of every layer gradient, through
the batched C-ABI entry points.  Inputs are synthetic, resident in HBM before
the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config NAME]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "ms per full K-FAC update (factors+inverse+precondition); KF-GEMM MFMA util %"
PEAK_FP32_MFMA_TFLOPS = 157.3
PEAK_HBM_GBPS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="resnet110_cifar")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--tune", action="append", default=[], help="development knob key=value")
    ap.add_argument("--seed", type=int, default=2000)
    ap.add_argument("--variant", choices=["inverse", "eigen"], default="inverse",
                    help="inverse: damped inverses + G_inv grad A_inv (the headline path); "
                         "eigen: eigen-decompositions + the Eq. 13 preconditioner")
    ap.add_argument("--traffic", type=float, default=None,
                    help="HBM bytes per launch of the dominant kernel, from the rocprofv3 --pmc runs "
                         "(FETCH_SIZE + WRITE_SIZE, scaled by the calibration copy); default: the figure "
                         "stored in profiles/hbm_traffic_<workload>.txt if that file exists")
    return ap.parse_args()


def make_inputs(layers, batch, hp, seed, torch, dev):
    """Synthetic device tensors with the workload's shapes and value distributions
    (ReLU'd or plain N(0,1) activations, N(0, var) output gradients, N(0,1) layer gradients)."""
    g = torch.Generator(device=dev)
    g.manual_seed(seed)
    bf = hp["dtype"] == "bf16"
    std = hp["gout_var"] ** 0.5
    acts, gouts, grads = [], [], []
    for l in layers:
        if l.kind == "conv":
            ashape = (batch, l.c_in, l.h_in, l.w)
            gshape = (batch, l.c_out, l.h_out, l.w_out)
        else:
            ashape = (l.rows, l.c_in)
            gshape = (l.rows, l.c_out)
        a = torch.randn(ashape, generator=g, device=dev)
        if hp["act"] == "relu_normal":
            a = torch.relu_(a)
        go = torch.randn(gshape, generator=g, device=dev) * std
        if bf:
            a, go = a.to(torch.bfloat16), go.to(torch.bfloat16)
        acts.append(a.contiguous())
        gouts.append(go.contiguous())
        grads.append(torch.randn((l.d_G, l.d_A), generator=g, device=dev))
    return acts, gouts, grads


def im2col_leg(kf, torch, step_update, ws_bytes_fn, work, steps):
    """The patch extractor in its batched launch configuration.  The full update above builds
    3x3/stride-1 fp32 factors straight from the NCHW input, so on such layers the extractor never
    runs; here the factor update is repeated with that fusion switched off and the extractor's
    launches are timed with HIP events (inputs differ per layer, so nothing is reused across launches)."""
    total = work["im2col_read"] + work["im2col_write"]
    if not total:
        return None
    kf.kfac_tune("fuse_conv3", 0)
    try:
        ws = torch.empty(ws_bytes_fn(), dtype=torch.uint8, device="cuda:0")
        step_update(ws)
        torch.cuda.synchronize()
        kf.kfac_timing_enable(True)
        reps = max(1, steps // 4)
        for _ in range(reps):
            step_update(ws)
        torch.cuda.synchronize()
        ms, n, _ = kf.kfac_timing_collect()["im2col"]
        kf.kfac_timing_enable(False)
    finally:
        kf.kfac_tune("fuse_conv3", 1)
    gbs = total * reps / (ms * 1e-3) / 1e9
    return dict(bound="hbm", kernel="im2col_kernel", achieved=round(gbs, 1), peak=8000.0, unit="GB/s",
                frac=round(gbs / 8000.0, 4), ms_per_step=round(ms / reps, 4), launches_per_step=n // reps,
                avg_launch_ms=round(ms / n, 5), algorithmic_bytes_per_step=total,
                note="factor update repeated with the fused 3x3 path off so that every k>1 conv layer "
                     "goes through the extractor (grouped launches of up to 40 layers)")


def cpu_baseline(config, layers, hp, variant="inverse"):
    """The CPU oracle, as it stands, timed on a bounded sample of layers of each distinct shape; the
    whole-update figure is the sum over shapes of (mean time x number of layers of that shape)."""
    from collections import Counter
    from oracle import kfac_oracle as orc
    from workloads import rng, shapes
    import numpy as np
    counts = Counter(layers)
    shapes_l = list(counts.items())
    times = {i: [] for i in range(len(shapes_l))}
    t_all = time.time()
    rep = 0
    # one layer of every distinct shape, then further layers of each (new seeds) until ~12 s of oracle work are
    # sampled; 40 s is the hard cap for the first pass over very large shapes
    while True:
        for i, (l, cnt) in enumerate(shapes_l):
            if rep >= cnt:
                continue
            spent = time.time() - t_all
            if (rep == 0 and spent > 40.0 and any(times.values())) or (rep > 0 and spent > 12.0):
                continue
            act, gout, grad = rng.layer_inputs(l, hp["batch"], 9000 + 97 * rep + i, hp["act"], hp["gout_var"] ** 0.5,
                                               hp["dtype"])
            sA, sG = shapes.layer_scales(l, hp["batch"])
            t0 = time.time()
            A, G = orc.update_factors_layer(l, act, gout, sA, sG, hp["decay"], np.eye(l.d_A), np.eye(l.d_G))
            if variant == "eigen":
                orc.precondition_eigen_layer(A, G, grad, hp["damping"])
            else:
                Ai, Gi = orc.invert_layer(A, G, hp["damping"], hp["damping"])
                orc.precondition_layer(Ai, Gi, grad)
            times[i].append((time.time() - t0) * 1e3)
        rep += 1
        if time.time() - t_all > 12.0 or rep >= max(counts.values()):
            break
    total_ms, sampled, timed = 0.0, 0, 0
    for i, (l, cnt) in enumerate(shapes_l):
        if times[i]:
            total_ms += cnt * sum(times[i]) / len(times[i])
            sampled += cnt
            timed += len(times[i])
    if sampled < len(layers):   # time cap hit: extrapolate by layer count, and say so
        total_ms *= len(layers) / sampled
    return dict(value=round(total_ms, 1), unit="ms", cores=orc.num_threads(), kind="oracle",
                sample=f"{timed} layers timed over the {len(counts)} distinct shapes ({sampled}/{len(layers)} layers "
                       f"covered; {time.time() - t_all:.0f} s of oracle work), mean per shape scaled by the number of "
                       f"layers of that shape")



def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no collective or multi-GPU path exists); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2206_15143_amd as kf
    from workloads import shapes
    if not os.path.exists(kf.lib_path()):   # the library that is built is the one that runs; compile only if there is none
        from paper_2206_15143_amd import build as hip_build
        hip_build.build()

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    for kv in args.tune:
        k, v = kv.split("=")
        kf.kfac_tune(k, int(v))

    hp = shapes.config_hparams(args.config)
    layers = shapes.config_layers(args.config)
    batch = hp["batch"]
    bf = hp["dtype"] == "bf16"
    descs = [kf.LayerDesc.from_spec(l, kf.KFAC_BF16 if bf else kf.KFAC_F32) for l in layers]
    b = [batch if l.kind == "conv" else l.rows for l in layers]
    h = [l.h_in if l.kind == "conv" else 1 for l in layers]
    w = [l.w if l.kind == "conv" else 1 for l in layers]
    sc = [shapes.layer_scales(l, batch) for l in layers]
    sA, sG = [s[0] for s in sc], [s[1] for s in sc]

    acts, gouts, grads = make_inputs(layers, batch, hp, args.seed, torch, dev)
    A_run = [torch.eye(l.d_A, device=dev) for l in layers]
    G_run = [torch.eye(l.d_G, device=dev) for l in layers]
    A_inv = [torch.empty((l.d_A, l.d_A), device=dev) for l in layers]
    G_inv = [torch.empty((l.d_G, l.d_G), device=dev) for l in layers]
    outs = [torch.empty((l.d_G, l.d_A), device=dev) for l in layers]
    info = torch.zeros(2 * len(layers), dtype=torch.int32, device=dev)
    ws = torch.empty(kf.kfac_workspace_bytes_batched(descs, b, h, w), dtype=torch.uint8, device=dev)
    lam = hp["damping"]

    eigen = args.variant == "eigen"
    if eigen:   # A_inv / G_inv hold Q_A / Q_G
        v_A = [torch.empty((l.d_A,), device=dev) for l in layers]
        v_G = [torch.empty((l.d_G,), device=dev) for l in layers]

    # descriptors, addresses and per-layer scalars converted to the C arrays once: none of them changes
    # between steps, and the conversion is host work outside the path
    m = dict(descs=kf.marshal_descs(descs), acts=kf.marshal_ptrs(acts), gouts=kf.marshal_ptrs(gouts),
             grads=kf.marshal_ptrs(grads), outs=kf.marshal_ptrs(outs), A_run=kf.marshal_ptrs(A_run),
             G_run=kf.marshal_ptrs(G_run), A_inv=kf.marshal_ptrs(A_inv), G_inv=kf.marshal_ptrs(G_inv),
             b=kf.marshal_ints(b), h=kf.marshal_ints(h), w=kf.marshal_ints(w),
             sA=kf.marshal_floats(sA), sG=kf.marshal_floats(sG))
    if eigen:
        m.update(v_A=kf.marshal_ptrs(v_A), v_G=kf.marshal_ptrs(v_G))

    def first_stage():
        kf.kfac_update_factors_batched(m["descs"], m["acts"], m["gouts"], m["b"], m["h"], m["w"], m["sA"], m["sG"],
                                       hp["decay"], m["A_run"], m["G_run"], ws)

    def second_stage():
        if eigen:
            kf.kfac_eigen_batched(m["descs"], m["A_run"], m["G_run"], m["A_inv"], m["v_A"], m["G_inv"], m["v_G"],
                                  info, ws)
        else:
            kf.kfac_invert_batched(m["descs"], m["A_run"], m["G_run"], lam, lam, m["A_inv"], m["G_inv"], info, ws)

    def third_stage():
        if eigen:
            kf.kfac_precondition_eigen_batched(m["descs"], m["A_inv"], m["v_A"], m["G_inv"], m["v_G"], lam,
                                               m["grads"], m["outs"], ws)
        else:
            kf.kfac_precondition_batched(m["descs"], m["A_inv"], m["G_inv"], m["grads"], m["outs"], ws)

    def step():
        first_stage()
        second_stage()
        third_stage()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    assert int(info.abs().sum().item()) == 0, "a factor was flagged (not positive definite / eigen sweep budget)"

    # the three calls timed one by one, for the stale-factor schedule of the paper's last experiment
    # (factors refreshed every F_freq iterations, inverses every K_freq, preconditioning every iteration)
    def timed(fn):
        fn()
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) * 1e3 / args.steps
    t_upd = timed(first_stage)
    t_inv = timed(second_stage)
    t_pre = timed(third_stage)
    F_FREQ, K_FREQ = 50, 500
    schedule = dict(update_factors_ms=round(t_upd, 4), **{"eigen_ms" if eigen else "invert_ms": round(t_inv, 4)},
                    precondition_ms=round(t_pre, 4),
                    F_freq=F_FREQ, K_freq=K_FREQ,
                    amortised_ms_per_iteration=round(t_pre + t_upd / F_FREQ + t_inv / K_FREQ, 4))

    # per-kernel-class durations: the same steps again with a HIP-event pair around every launch
    kf.kfac_timing_enable(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    cls = kf.kfac_timing_collect()
    kf.kfac_timing_enable(False)
    stages = {k: round(v[0] / args.steps, 4) for k, v in cls.items()}
    launches = {k: v[1] // args.steps for k, v in cls.items()}
    in_bytes = 2 if bf else 4
    work = shapes.algorithmic_work(layers, batch, in_bytes)
    peak = PEAK_FP32_MFMA_TFLOPS   # every factor kernel runs on fp32 MFMA (bf16 inputs are widened on load)
    # KF-GEMM kernels: per kernel, algorithmic triangle flops (counted by the library per launch) over
    # the HIP-event time of its launches; the roofline object is the one with the largest share of time
    names = {"syrk_partial": "syrk_partial_kernel", "syrk_wave": "syrk_wave_kernel",
             "syrk_conv3": "syrk_conv3_kernel", "syrk_small": "syrk_small_nchw_kernel",
             "syrk_bf16": "syrk_bf16_kernel", "syrk_corr3": "corr3_main_kernel"}
    per_kernel = {}
    for k, kname in names.items():
        ms, n, flops = cls[k]
        if n == 0:
            continue
        tf = flops / (ms * 1e-3) / 1e12
        per_kernel[kname] = dict(achieved=round(tf, 2), frac=round(tf / peak, 4), ms_per_step=round(ms / args.steps, 4),
                                 launches_per_step=n // args.steps,
                                 avg_launch_ms=round(ms / n, 5), algorithmic_flops_per_step=flops / args.steps)
    if "corr3_main_kernel" in per_kernel:
        # The autocorrelation route computes the same factors with fewer products than the definition (13 lag
        # tiles instead of 45 per channel-tile pair and k-step): `achieved` stays the ALGORITHMIC figure of the
        # definition, R*d*(d+1) flops per factor, so it can exceed the MFMA peak; the flops the units really
        # execute, 26*C^2*B*H*W per layer, are given beside it.
        ex = sum(26.0 * l.c_in ** 2 * batch * l.h_in * l.w for l in layers
                 if l.kind == "conv" and l.k == 3 and l.kw == 3 and l.stride == 1 and l.pad == 1 and not bf
                 and l.c_in in (16, 32, 64) and l.w % 4 == 0 and l.w <= 64 and l.h_in <= 64)
        pk = per_kernel["corr3_main_kernel"]
        pk["executed_flops_per_step"] = ex
        pk["executed_tflops"] = round(ex / (pk["ms_per_step"] * 1e-3) / 1e12, 2)
        pk["executed_frac"] = round(pk["executed_tflops"] / peak, 4)
    dom = max(per_kernel, key=lambda k: per_kernel[k]["ms_per_step"])
    d = per_kernel[dom]
    traffic = args.traffic
    tfile = os.path.join(ROOT, "profiles", f"hbm_traffic_{args.config}.txt")
    if traffic is None and os.path.exists(tfile):   # comment lines, then one JSON object {kernel: {...}}
        with open(tfile) as fh:
            body = "".join(line for line in fh if not line.startswith("#"))
        traffic = json.loads(body).get(dom, {}).get("hbm_bytes_per_launch")
    # counter-based MFMA busy fraction of the same kernel (rocprofv3 --pmc run, see profiles/), if recorded
    mfma_busy = None
    mfile = os.path.join(ROOT, "profiles", f"mfma_util_bench_{args.config}.txt")
    if os.path.exists(mfile):
        with open(mfile) as fh:
            for line in fh:
                if line.startswith(dom):
                    mfma_busy = float(line.split()[-3])
                    break
    roofline = dict(bound="mfma", kernel=dom, achieved=d["achieved"], peak=peak, unit="TFLOP/s", frac=d["frac"],
                    traffic=traffic, mfma_busy_counter=mfma_busy, launches_per_step=d["launches_per_step"], avg_launch_ms=d["avg_launch_ms"],
                    algorithmic_flops_per_launch=d["algorithmic_flops_per_step"] / d["launches_per_step"])
    if "executed_flops_per_step" in d:
        roofline.update(executed_flops_per_launch=d["executed_flops_per_step"] / d["launches_per_step"],
                        executed_achieved=d["executed_tflops"], executed_frac=d["executed_frac"],
                        note="factors from input autocorrelations: 'achieved' counts the flops of the definition "
                             "(R*d*(d+1) per factor), 'executed_*' the 26*C^2*B*H*W flops the MFMA units really do")
    syrk_flops = work["syrk_A"] + work["syrk_G"]
    assert abs(sum(v["algorithmic_flops_per_step"] for v in per_kernel.values()) - syrk_flops) <= 1e-6 * syrk_flops
    syrk_ms = sum(v["ms_per_step"] for v in per_kernel.values())
    achieved = syrk_flops / (syrk_ms * 1e-3) / 1e12
    extra = dict(kf_gemm_kernels=per_kernel, stale_schedule=schedule)
    # running-average update = the epilogue of the split reduction: the library counts, per reduce launch, the
    # split slices and the old factor read (one triangle) and the factor written (both triangles)
    r_ms, r_n, r_bytes = cls["syrk_reduce"]
    if r_n:
        extra["running_average"] = dict(bound="hbm", kernel="syrk_reduce_kernel", achieved=round(r_bytes / (r_ms * 1e-3) / 1e9, 1),
                                        peak=PEAK_HBM_GBPS, unit="GB/s", frac=round(r_bytes / (r_ms * 1e-3) / 1e9 / PEAK_HBM_GBPS, 4),
                                        ms_per_step=round(r_ms / args.steps, 4), launches_per_step=r_n // args.steps,
                                        algorithmic_bytes_per_step=r_bytes / args.steps)
    im2 = im2col_leg(kf, torch,
                     lambda w_: kf.kfac_update_factors_batched(descs, acts, gouts, b, h, w, sA, sG, hp["decay"],
                                                               A_run, G_run, w_),
                     lambda: kf.kfac_workspace_bytes_batched(descs, b, h, w), work, args.steps)
    if im2:
        extra["im2col"] = im2

    out = dict(metric=METRIC, value=round(ms_per_step, 4), unit="ms", n_gpus=1, steps=args.steps,
               warmup=args.warmup, ms_per_step=round(ms_per_step, 4), higher_is_better=False, scaling="weak",
               vs_baseline=None, dtype="f32" if not bf else "bf16 in, f32 accumulate", data="synthetic",
               config=dict(workload=args.config, variant=args.variant, layers=len(layers), batch=batch, damping=lam,
                           decay=hp["decay"],
                           in_dtype=hp["dtype"]),
               kf_gemm_mfma_util_pct=round(100 * achieved / peak, 2),
               stage_ms=stages, launches_per_step=launches, roofline=roofline, **extra)
    # one plain copy of known size: the launch the byte counters of a rocprofv3 --pmc run are scaled by
    csrc = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
    cdst = torch.empty_like(csrc)
    kf.kfac_profile_copy(cdst, csrc, csrc.numel())
    torch.cuda.synchronize()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.config, layers, hp, args.variant)
    print(json.dumps(out))


if __name__ == "__main__":
    main()

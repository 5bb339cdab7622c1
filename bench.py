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


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="resnet110_cifar")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--tune", action="append", default=[], help="development knob key=value")
    ap.add_argument("--seed", type=int, default=2000)
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
            ashape = (batch, l.c_in, l.h_in, l.h_in)
            gshape = (batch, l.c_out, l.h_out, l.h_out)
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


def cpu_baseline(config, layers, hp):
    """The CPU oracle, as it stands, timed on one layer of each distinct shape;
    the whole-update figure is the sum over shapes of (time x number of layers of that shape)."""
    from collections import Counter
    from oracle import kfac_oracle as orc
    from workloads import rng, shapes
    import numpy as np
    counts = Counter(layers)
    total_ms, sampled = 0.0, 0
    t_all = time.time()
    for i, (l, cnt) in enumerate(counts.items()):
        if time.time() - t_all > 40.0 and sampled > 0:
            break
        act, gout, grad = rng.layer_inputs(l, hp["batch"], 9000 + i, hp["act"], hp["gout_var"] ** 0.5, hp["dtype"])
        sA, sG = shapes.layer_scales(l, hp["batch"])
        t0 = time.time()
        A, G = orc.update_factors_layer(l, act, gout, sA, sG, hp["decay"], np.eye(l.d_A), np.eye(l.d_G))
        Ai, Gi = orc.invert_layer(A, G, hp["damping"], hp["damping"])
        orc.precondition_layer(Ai, Gi, grad)
        dt = (time.time() - t0) * 1e3
        total_ms += dt * cnt
        sampled += cnt
    if sampled < len(layers):   # time cap hit: extrapolate by layer count, and say so
        total_ms *= len(layers) / sampled
    return dict(value=round(total_ms, 1), unit="ms", cores=orc.num_threads(), kind="oracle",
                sample=f"one layer of each distinct shape timed ({len(counts)} shapes, {sampled}/{len(layers)} "
                       f"layers covered), scaled by the number of layers of that shape")


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no collective or multi-GPU path exists); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2206_15143_amd as kf
    from workloads import shapes

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
    sc = [shapes.layer_scales(l, batch) for l in layers]
    sA, sG = [s[0] for s in sc], [s[1] for s in sc]

    acts, gouts, grads = make_inputs(layers, batch, hp, args.seed, torch, dev)
    A_run = [torch.eye(l.d_A, device=dev) for l in layers]
    G_run = [torch.eye(l.d_G, device=dev) for l in layers]
    A_inv = [torch.empty((l.d_A, l.d_A), device=dev) for l in layers]
    G_inv = [torch.empty((l.d_G, l.d_G), device=dev) for l in layers]
    outs = [torch.empty((l.d_G, l.d_A), device=dev) for l in layers]
    info = torch.zeros(2 * len(layers), dtype=torch.int32, device=dev)
    ws = torch.empty(kf.kfac_workspace_bytes_batched(descs, b, h, h), dtype=torch.uint8, device=dev)
    lam = hp["damping"]

    def step():
        kf.kfac_update_factors_batched(descs, acts, gouts, b, h, h, sA, sG, hp["decay"], A_run, G_run, ws)
        kf.kfac_invert_batched(descs, A_run, G_run, lam, lam, A_inv, G_inv, info, ws)
        kf.kfac_precondition_batched(descs, A_inv, G_inv, grads, outs, ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    assert int(info.abs().sum().item()) == 0, "a factor was flagged not positive definite"

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
    syrk_flops = work["syrk_A"] + work["syrk_G"]
    syrk_ms, syrk_launches = cls["syrk_partial"][0] / args.steps, launches["syrk_partial"]
    achieved = syrk_flops / (syrk_ms * 1e-3) / 1e12
    peak = PEAK_FP32_MFMA_TFLOPS   # the factor kernel runs on fp32 MFMA (bf16 inputs are widened on load)
    roofline = dict(bound="mfma", kernel="syrk_partial_kernel", achieved=round(achieved, 2), peak=peak,
                    unit="TFLOP/s", frac=round(achieved / peak, 4), traffic=None,
                    launches_per_step=syrk_launches, avg_launch_ms=round(syrk_ms / max(syrk_launches, 1), 5),
                    algorithmic_flops_per_step=syrk_flops)
    im2col_bytes = work["im2col_read"] + work["im2col_write"]
    extra = {}
    if im2col_bytes and stages["im2col"] > 0:
        gbs = im2col_bytes / (stages["im2col"] * 1e-3) / 1e9
        extra["im2col"] = dict(bound="hbm", achieved=round(gbs, 1), peak=8000.0, unit="GB/s",
                               frac=round(gbs / 8000.0, 4), algorithmic_bytes_per_step=im2col_bytes)

    out = dict(metric=METRIC, value=round(ms_per_step, 4), unit="ms", n_gpus=1, steps=args.steps,
               warmup=args.warmup, ms_per_step=round(ms_per_step, 4), higher_is_better=False, scaling="weak",
               vs_baseline=None, dtype="f32" if not bf else "bf16 in, f32 accumulate", data="synthetic",
               config=dict(workload=args.config, layers=len(layers), batch=batch, damping=lam, decay=hp["decay"],
                           in_dtype=hp["dtype"]),
               kf_gemm_mfma_util_pct=round(100 * achieved / peak, 2),
               stage_ms=stages, launches_per_step=launches, roofline=roofline, **extra)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.config, layers, hp)
    print(json.dumps(out))


if __name__ == "__main__":
    main()

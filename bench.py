#!/usr/bin/env python3
"""Benchmark of the full K-FAC second-order update on one MI355X.

A "step" is one pass of the whole hot path over all layers of a workload:
factor construction (im2col + SYRK + running average), damped inversion of
every A and G, and two-sided preconditioning of every layer gradient, through
the batched C-ABI entry points.  Inputs are synthetic, resident in HBM before
the timed region.  Prints ONE JSON line: the headline workload (ResNet-50-shaped,
fp32, the paper's precision) at the top level, the other configurations as
sub-objects of `other_configs`.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config NAME] [--only-headline]
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "ms per full K-FAC update (factors+inverse+precondition); KF-GEMM MFMA util %"
PEAK = {"f32": 157.3, "bf16": 2500.0}     # dense MFMA TFLOP/s of MI355X
PEAK_HBM_GBPS = 8000.0
HEADLINE = "resnet50_imagenet"
OTHERS = ["resnet110_cifar", "resnet50_imagenet_bf16", "transformer_encoder_bf16"]

# timing class of the library -> (kernel, what bounds it, dtype of the MFMA units it runs on, part of the KF-GEMM)
CLASSES = {
    "syrk_partial": ("syrk_partial_kernel", "mfma", "f32", True),
    "syrk_wave": ("syrk_wave_kernel", "mfma", "f32", True),
    "syrk_conv3": ("syrk_conv3_kernel", "mfma", "f32", True),
    "syrk_small": ("syrk_small_nchw_kernel", "hbm", "f32", True),
    "syrk_bf16": ("syrk_bf16_kernel", "mfma", "bf16", True),
    "syrk_corr3": ("corr3_main_kernel", "mfma", "f32", True),
    "syrk_split": ("syrk_split_kernel", "mfma", "bf16", True),
    "gemm_tn": ("gemm_tn_kernel", "mfma", "f32", False),
    "gemm_wave": ("gemm_wave_kernel", "mfma", "f32", False),
    "gemm_split": ("gemm_split_kernel", "mfma", "bf16", False),
    "inv_step": ("fsweep_step_kernel", "mfma", "f32", False),
}
# launches without which a factor is not complete: counted in the KF-GEMM time
KF_GEMM_EXTRA = ("syrk_reduce", "corr3_assemble")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default=HEADLINE, help="headline workload (default: the ResNet-50-shaped fp32 set)")
    ap.add_argument("--only-headline", action="store_true", help="skip the other configurations")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--tune", action="append", default=[], help="development knob key=value")
    ap.add_argument("--seed", type=int, default=2000)
    ap.add_argument("--variant", choices=["inverse", "eigen"], default="inverse",
                    help="inverse: damped inverses + G_inv grad A_inv (the headline path); "
                         "eigen: eigen-decompositions + the Eq. 13 preconditioner")
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


def cpu_baseline(layers, hp, variant, budget_s, first_pass_cap_s):
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
    # one layer of every distinct shape (smallest first, so that a time cap cuts the few largest), then further
    # layers of each (new seeds) until the budget of oracle work is sampled
    order = sorted(range(len(shapes_l)), key=lambda i: shapes_l[i][0].d_A ** 3 + shapes_l[i][0].d_G ** 3
                   + shapes_l[i][0].n_rows(hp["batch"]) * shapes_l[i][0].d_A ** 2)
    while True:
        for i in order:
            l, cnt = shapes_l[i]
            if rep >= cnt:
                continue
            spent = time.time() - t_all
            if (rep == 0 and spent > first_pass_cap_s and any(times.values())) or (rep > 0 and spent > budget_s):
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
        if time.time() - t_all > budget_s or rep >= max(counts.values()):
            break
    total_ms, sampled, timed = 0.0, 0, 0
    for i, (l, cnt) in enumerate(shapes_l):
        if times[i]:
            total_ms += cnt * sum(times[i]) / len(times[i])
            sampled += cnt
            timed += len(times[i])
    whole = timed == len(layers)
    if sampled < len(layers):   # time cap hit: extrapolate by the definition's flop count, and say so
        def cost(l):
            return l.n_rows(hp["batch"]) * (l.d_A ** 2 + l.d_G ** 2) + l.d_A ** 3 + l.d_G ** 3
        done = sum(cost(l) * cnt for i, (l, cnt) in enumerate(shapes_l) if times[i])
        total_ms *= sum(cost(l) * cnt for l, cnt in shapes_l) / done
    note = ("every layer timed once (the whole update)" if whole else
            f"{timed} layers timed over the {len(counts)} distinct shapes ({sampled}/{len(layers)} layers covered"
            + ("" if sampled == len(layers) else "; the rest extrapolated by flop count") +
            "), mean per shape scaled by the number of layers of that shape")
    return dict(value=round(total_ms, 1), unit="ms", cores=orc.num_threads(), kind="oracle",
                sample=f"{note}; {time.time() - t_all:.0f} s of oracle work")


def read_profile_json(path):
    """profiles/*.txt: comment lines, then one JSON object."""
    if not os.path.exists(path):
        return {}
    with open(path) as fh:
        body = "".join(line for line in fh if not line.startswith("#"))
    try:
        return json.loads(body)
    except ValueError:
        return {}


def run_config(name, args, kf, torch, steps, warmup, cpu_budget):
    from workloads import shapes
    dev = "cuda:0"
    hp = shapes.config_hparams(name)
    layers = shapes.config_layers(name)
    batch = hp["batch"]
    bf = hp["dtype"] == "bf16"
    descs = [kf.LayerDesc.from_spec(l, kf.KFAC_BF16 if bf else kf.KFAC_F32) for l in layers]
    b = [batch if l.kind == "conv" else l.rows for l in layers]
    h = [l.h_in if l.kind == "conv" else 1 for l in layers]
    w = [l.w if l.kind == "conv" else 1 for l in layers]
    sc = [shapes.layer_scales(l, batch) for l in layers]
    sA, sG = [s[0] for s in sc], [s[1] for s in sc]
    eigen = args.variant == "eigen"

    # two sets of inputs: the "cold" leg alternates between them, so that no step finds its inputs where the
    # step before left them (each set alone is already far larger than the 256 MB last-level cache)
    sets = [make_inputs(layers, batch, hp, args.seed + k, torch, dev) for k in range(2)]
    in_bytes = sum(t.numel() * t.element_size() for part in sets[0] for t in part)
    A_run = [torch.eye(l.d_A, device=dev) for l in layers]
    G_run = [torch.eye(l.d_G, device=dev) for l in layers]
    A_inv = [torch.empty((l.d_A, l.d_A), device=dev) for l in layers]
    G_inv = [torch.empty((l.d_G, l.d_G), device=dev) for l in layers]
    outs = [torch.empty((l.d_G, l.d_A), device=dev) for l in layers]
    info = torch.zeros(2 * len(layers), dtype=torch.int32, device=dev)
    ws = torch.empty(kf.kfac_workspace_bytes_batched(descs, b, h, w), dtype=torch.uint8, device=dev)
    lam = hp["damping"]
    if eigen:   # A_inv / G_inv hold Q_A / Q_G
        v_A = [torch.empty((l.d_A,), device=dev) for l in layers]
        v_G = [torch.empty((l.d_G,), device=dev) for l in layers]

    # descriptors, addresses and per-layer scalars converted to the C arrays once: none of them changes
    # between steps, and the conversion is host work outside the path
    m = dict(descs=kf.marshal_descs(descs), outs=kf.marshal_ptrs(outs), A_run=kf.marshal_ptrs(A_run),
             G_run=kf.marshal_ptrs(G_run), A_inv=kf.marshal_ptrs(A_inv), G_inv=kf.marshal_ptrs(G_inv),
             b=kf.marshal_ints(b), h=kf.marshal_ints(h), w=kf.marshal_ints(w),
             sA=kf.marshal_floats(sA), sG=kf.marshal_floats(sG))
    ins = [dict(acts=kf.marshal_ptrs(s[0]), gouts=kf.marshal_ptrs(s[1]), grads=kf.marshal_ptrs(s[2])) for s in sets]
    if eigen:
        m.update(v_A=kf.marshal_ptrs(v_A), v_G=kf.marshal_ptrs(v_G))

    def first_stage(k=0):
        kf.kfac_update_factors_batched(m["descs"], ins[k]["acts"], ins[k]["gouts"], m["b"], m["h"], m["w"], m["sA"],
                                       m["sG"], hp["decay"], m["A_run"], m["G_run"], ws)

    def second_stage(k=0):
        if eigen:
            kf.kfac_eigen_batched(m["descs"], m["A_run"], m["G_run"], m["A_inv"], m["v_A"], m["G_inv"], m["v_G"],
                                  info, ws)
        else:
            kf.kfac_invert_batched(m["descs"], m["A_run"], m["G_run"], lam, lam, m["A_inv"], m["G_inv"], info, ws)

    def third_stage(k=0):
        if eigen:
            kf.kfac_precondition_eigen_batched(m["descs"], m["A_inv"], m["v_A"], m["G_inv"], m["v_G"], lam,
                                               ins[k]["grads"], m["outs"], ws)
        else:
            kf.kfac_precondition_batched(m["descs"], m["A_inv"], m["G_inv"], ins[k]["grads"], m["outs"], ws)

    def step(k=0):
        first_stage(k)
        second_stage(k)
        third_stage(k)

    # ---- the timed region: warm (the same input set every step), then cold (alternating sets) ----
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    assert int(info.abs().sum().item()) == 0, "a factor was flagged (not positive definite / eigen sweep budget)"
    step(1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i & 1)
    torch.cuda.synchronize()
    cold_ms = (time.perf_counter() - t0) * 1e3 / steps

    # the three calls timed one by one, for the stale-factor schedule of the paper's last experiment
    # (factors refreshed every F_freq iterations, inverses every K_freq, preconditioning every iteration)
    def timed(fn):
        fn()
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) * 1e3 / steps
    t_upd, t_inv, t_pre = timed(first_stage), timed(second_stage), timed(third_stage)
    F_FREQ, K_FREQ = 50, 500
    schedule = dict(update_factors_ms=round(t_upd, 4), **{"eigen_ms" if eigen else "invert_ms": round(t_inv, 4)},
                    precondition_ms=round(t_pre, 4), F_freq=F_FREQ, K_freq=K_FREQ,
                    amortised_ms_per_iteration=round(t_pre + t_upd / F_FREQ + t_inv / K_FREQ, 4))

    # per-kernel-class durations: the same steps again with a HIP-event pair around every launch, on the
    # stream the launch goes to (launches that overlap on the library's second stream are each timed in full,
    # so the classes of the inversion can add up to more than its wall time)
    kf.kfac_timing_enable(True)
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    cls = kf.kfac_timing_collect_ex()
    kf.kfac_timing_enable(False)
    stages = {k: round(v[0] / steps, 4) for k, v in cls.items() if v[1]}
    launches = {k: v[1] // steps for k, v in cls.items() if v[1]}
    work = shapes.algorithmic_work(layers, batch, 2 if bf else 4)

    # every kernel class that does arithmetic on the MFMA units: the flops it EXECUTES by its own method per
    # launch over the mean HIP-event duration of its launches, against the dense peak of the unit it runs on;
    # the flops of the definition (R d (d+1) per factor, n^3 per inverse, 2 M N K per product) beside it
    kernels = {}
    for k, (kname, bound, dt, _) in CLASSES.items():
        ms, n, wk, ex = cls[k]
        if n == 0:
            continue
        ent = dict(bound=bound, mfma_dtype=dt, ms_per_step=round(ms / steps, 4), launches_per_step=n // steps,
                   avg_launch_ms=round(ms / n, 5), executed_flops_per_launch=ex / n,
                   achieved=round(ex / (ms * 1e-3) / 1e12, 2), peak=PEAK[dt], unit="TFLOP/s",
                   frac=round(ex / (ms * 1e-3) / 1e12 / PEAK[dt], 4),
                   definition_equiv_tflops=round(wk / (ms * 1e-3) / 1e12, 2))
        if bound == "hbm":
            ent["note"] = "HBM-bound by its operand reads (narrow factors): the MFMA fraction is not its roofline"
        kernels[kname] = ent
    kf_time = sum(cls[k][0] for k, c in CLASSES.items() if c[3]) + sum(cls[k][0] for k in KF_GEMM_EXTRA)
    kf_peak_time = sum(cls[k][3] / (PEAK[c[2]] * 1e12) * 1e3 for k, c in CLASSES.items() if c[3])
    kf_def = sum(cls[k][2] for k, c in CLASSES.items() if c[3])
    syrk_flops = work["syrk_A"] + work["syrk_G"]
    assert abs(kf_def / steps - syrk_flops) <= 1e-6 * syrk_flops
    kf_gemm = dict(mfma_util_pct=round(100 * kf_peak_time / kf_time, 2) if kf_time else None,
                   ms_per_step=round(kf_time / steps, 4),
                   definition_equiv_tflops=round(kf_def / (kf_time * 1e-3) / 1e12, 2) if kf_time else None,
                   note="time at peak of the flops each KF-GEMM kernel executes (fp32 kernels against 157.3, bf16 "
                        "against 2500 TFLOP/s) over the time of all launches a factor needs (partial products, "
                        "split reduction + running average, border and assembly launches)")

    # the kernel with the largest share of the step
    dom = max(kernels, key=lambda k: kernels[k]["ms_per_step"])
    d = kernels[dom]
    prof = read_profile_json(os.path.join(ROOT, "profiles", f"hbm_traffic_{name}.txt")).get(dom, {})
    traffic = prof.get("hbm_bytes_per_launch")
    traffic_note = None
    if traffic is not None and prof.get("avg_launch_ms"):
        # the counters come from a separate rocprofv3 run of this same command: only quoted while that run's
        # kernel still behaves like the one timed here
        if abs(prof["avg_launch_ms"] - d["avg_launch_ms"]) > 0.25 * d["avg_launch_ms"]:
            traffic, traffic_note = None, "stored counter run no longer matches this kernel's duration"
    roofline = dict(bound=d["bound"] if d["bound"] != "hbm" else "mfma", kernel=dom, achieved=d["achieved"],
                    peak=d["peak"], unit="TFLOP/s", frac=d["frac"], traffic=traffic, mfma_dtype=d["mfma_dtype"],
                    launches_per_step=d["launches_per_step"], avg_launch_ms=d["avg_launch_ms"],
                    executed_flops_per_launch=d["executed_flops_per_launch"],
                    definition_equiv_tflops=d["definition_equiv_tflops"],
                    share_of_step=round(d["ms_per_step"] / ms_per_step, 3))
    if traffic_note:
        roofline["traffic_note"] = traffic_note
    if dom == "gemm_split_kernel":
        roofline["note"] = ("fp32 products as six bf16 MFMA products of the operands' bf16 pieces: 'achieved' counts the "
                            "bf16 flops executed (6 x 2 M N K) against the bf16 peak; definition_equiv_tflops counts "
                            "2 M N K, for comparison with the fp32 MFMA peak of 157.3")

    out = dict(ms_per_step=round(ms_per_step, 4), cold_ms_per_step=round(cold_ms, 4),
               cold_note=f"steps alternate between two input sets of {in_bytes / 1e9:.2f} GB each; the warm figure "
                         "re-reads one set, which is itself far beyond the 256 MB last-level cache",
               config=dict(workload=name, variant=args.variant, layers=len(layers), batch=batch, damping=lam,
                           decay=hp["decay"], in_dtype=hp["dtype"], gout_sigma=round(hp["gout_var"] ** 0.5, 5)),
               dtype="f32" if not bf else "bf16 in, f32 accumulate",
               stage_ms=stages, launches_per_step=launches, roofline=roofline, kernels=kernels, kf_gemm=kf_gemm,
               algorithmic_work=work, stale_schedule=schedule)

    # running-average update = the epilogue of the split reduction.  Algorithmic bytes: one triangle of every
    # factor read and written (8 bytes per entry of the triangle); the launches also read the split slices
    r_ms, r_n, r_bytes, _ = cls["syrk_reduce"]
    if r_n:
        out["running_average"] = dict(bound="hbm", kernel="syrk_reduce_kernel",
                                      achieved=round(work["ema_bytes"] * steps / (r_ms * 1e-3) / 1e9, 1),
                                      peak=PEAK_HBM_GBPS, unit="GB/s",
                                      frac=round(work["ema_bytes"] * steps / (r_ms * 1e-3) / 1e9 / PEAK_HBM_GBPS, 4),
                                      ms_per_step=round(r_ms / steps, 4), launches_per_step=r_n // steps,
                                      algorithmic_bytes_per_step=work["ema_bytes"],
                                      moved_gbps=round(r_bytes / (r_ms * 1e-3) / 1e9, 1),
                                      note="algorithmic bytes = the factor triangles read and written; moved_gbps also "
                                           "counts the split slices the fused reduction reads and the mirrored triangle")

    # the patch extractor in its batched launch configuration.  The full update builds 3x3/stride-1 fp32 factors
    # straight from the NCHW input, so on such layers the extractor never runs; here the factor update is
    # repeated with that fusion switched off and the extractor's launches are timed with HIP events
    total_i2c = work["im2col_read"] + work["im2col_write"]
    if total_i2c and not eigen:
        kf.kfac_tune("fuse_conv3", 0)
        try:
            ws2 = torch.empty(kf.kfac_workspace_bytes_batched(descs, b, h, w), dtype=torch.uint8, device=dev)
            upd = lambda: kf.kfac_update_factors_batched(m["descs"], ins[0]["acts"], ins[0]["gouts"], m["b"], m["h"],
                                                         m["w"], m["sA"], m["sG"], hp["decay"], m["A_run"], m["G_run"],
                                                         ws2)
            upd()
            torch.cuda.synchronize()
            kf.kfac_timing_enable(True)
            reps = max(1, steps // 4)
            for _ in range(reps):
                upd()
            torch.cuda.synchronize()
            i_ms, i_n, _, _ = kf.kfac_timing_collect_ex()["im2col"]
            kf.kfac_timing_enable(False)
            del ws2
        finally:
            kf.kfac_tune("fuse_conv3", 1)
        gbs = total_i2c * reps / (i_ms * 1e-3) / 1e9
        iprof = read_profile_json(os.path.join(ROOT, "profiles", f"hbm_traffic_{name}.txt")).get("im2col_kernel", {})
        out["im2col"] = dict(bound="hbm", kernel="im2col_kernel", achieved=round(gbs, 1), peak=PEAK_HBM_GBPS,
                             unit="GB/s", frac=round(gbs / PEAK_HBM_GBPS, 4), ms_per_step=round(i_ms / reps, 4),
                             launches_per_step=i_n // reps, avg_launch_ms=round(i_ms / i_n, 5),
                             algorithmic_bytes_per_step=total_i2c,
                             counter_bytes_per_launch=iprof.get("hbm_bytes_per_launch"),
                             note="factor update repeated with the fused 3x3 path off so that every k>1 conv layer "
                                  "goes through the extractor (grouped launches of up to 40 layers)")

    if cpu_budget and not args.no_cpu_baseline:
        # free the device tensors first: the oracle needs host memory, not the GPU
        out["cpu_baseline"] = cpu_baseline(layers, hp, args.variant, cpu_budget[0], cpu_budget[1])
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no collective or multi-GPU path exists); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2206_15143_amd as kf
    if not os.path.exists(kf.lib_path()):   # the library that is built is the one that runs; compile only if there is none
        from paper_2206_15143_amd import build as hip_build
        hip_build.build()

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    for kv in args.tune:
        k, v = kv.split("=")
        kf.kfac_tune(k, int(v))

    # (budget of oracle work in seconds, cap on the first pass over the distinct shapes)
    head = run_config(args.config, args, kf, torch, args.steps, args.warmup,
                      (25.0, 25.0) if args.config == "resnet110_cifar" else (12.0, 30.0))
    out = dict(metric=METRIC, value=head["ms_per_step"], unit="ms", n_gpus=1, steps=args.steps, warmup=args.warmup,
               ms_per_step=head["ms_per_step"], higher_is_better=False, scaling="weak", vs_baseline=None,
               dtype=head["dtype"], data="synthetic", config=head["config"],
               kf_gemm_mfma_util_pct=head["kf_gemm"]["mfma_util_pct"])
    out.update({k: v for k, v in head.items() if k not in ("ms_per_step", "dtype", "config")})
    out["paper_context"] = dict(computation="1.55-1.65x", communication="2.79-3.15x", hw="64x RTX2080Ti",
                                note="per-update reductions of DP-KFAC over the compared distributed K-FAC systems as the "
                                     "paper's abstract states them, measured on its own cluster: context, not a target "
                                     "of this one-GPU measurement")
    if not args.only_headline:
        others = {}
        for name in OTHERS:
            if name == args.config:
                continue
            gc.collect()
            torch.cuda.empty_cache()
            sub_steps = max(3, min(args.steps, 5 if name == "transformer_encoder_bf16" else 10))
            others[name] = run_config(name, args, kf, torch, sub_steps, 2,
                                      (22.0, 22.0) if name == "resnet110_cifar" else (6.0, 15.0))
            others[name]["steps"] = sub_steps
        out["other_configs"] = others
    # one plain copy of known size: the launch the byte counters of a rocprofv3 --pmc run are scaled by
    csrc = torch.empty(256 << 20, dtype=torch.uint8, device="cuda:0")
    cdst = torch.empty_like(csrc)
    kf.kfac_profile_copy(cdst, csrc, csrc.numel())
    torch.cuda.synchronize()
    print(json.dumps(out))


if __name__ == "__main__":
    main()

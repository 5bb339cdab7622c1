"""Helpers shared by the GPU parity tests: run one layer (or a set) through the
C-ABI binding and through the CPU oracle on the same seeded inputs."""
from __future__ import annotations

import numpy as np
import torch

import paper_2206_15143_amd as kf
from oracle import kfac_oracle as orc
from workloads import rng, shapes

DEV = "cuda:0"


def rel_fro(got, ref) -> float:
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))


def to_dev(x: np.ndarray, bf16: bool = False) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(x))
    if bf16:
        t = t.to(torch.bfloat16)          # exact: the values are already bf16-representable
    return t.to(DEV)


def workspace(nbytes: int) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=DEV)


def batch_args(layers, batch):
    b = [batch if l.kind == "conv" else l.rows for l in layers]
    h = [l.h_in if l.kind == "conv" else 1 for l in layers]
    w = [l.w if l.kind == "conv" else 1 for l in layers]
    return b, h, w


class GpuLayerResult:
    pass


def run_layers_gpu(layers, batch, inputs, scales, decay, damping, dtype="f32", batched=True, A0=None, G0=None,
                   marshalled=False):
    """inputs: list of (act, gout, grad) numpy arrays.  Returns per-layer dict of numpy results.
    marshalled: the batched calls get C arrays built beforehand instead of Python lists."""
    n = len(layers)
    bf = dtype == "bf16"
    descs = [kf.LayerDesc.from_spec(l, kf.KFAC_BF16 if bf else kf.KFAC_F32) for l in layers]
    b, h, w = batch_args(layers, batch)
    acts = [to_dev(i[0], bf) for i in inputs]
    gouts = [to_dev(i[1], bf) for i in inputs]
    grads = [to_dev(i[2]) for i in inputs]
    dA = [kf.kfac_dim_A(d) for d in descs]
    dG = [kf.kfac_dim_G(d) for d in descs]
    A_run = [torch.eye(a, device=DEV) if A0 is None else to_dev(A0[i].astype(np.float32)) for i, a in enumerate(dA)]
    G_run = [torch.eye(g, device=DEV) if G0 is None else to_dev(G0[i].astype(np.float32)) for i, g in enumerate(dG)]
    A_inv = [torch.full((a, a), float("nan"), device=DEV) for a in dA]
    G_inv = [torch.full((g, g), float("nan"), device=DEV) for g in dG]
    outs = [torch.full((g, a), float("nan"), device=DEV) for a, g in zip(dA, dG)]
    info = torch.full((2 * n,), -1, dtype=torch.int32, device=DEV)
    sA = [s[0] for s in scales]
    sG = [s[1] for s in scales]
    if batched:
        ws = workspace(kf.kfac_workspace_bytes_batched(descs, b, h, w))
        if marshalled:
            P = kf.marshal_ptrs
            md, mb, mh, mw = kf.marshal_descs(descs), kf.marshal_ints(b), kf.marshal_ints(h), kf.marshal_ints(w)
            mAr, mGr, mAi, mGi = P(A_run), P(G_run), P(A_inv), P(G_inv)
            kf.kfac_update_factors_batched(md, P(acts), P(gouts), mb, mh, mw, kf.marshal_floats(sA),
                                           kf.marshal_floats(sG), decay, mAr, mGr, ws)
            kf.kfac_invert_batched(md, mAr, mGr, damping, damping, mAi, mGi, info, ws)
            kf.kfac_precondition_batched(md, mAi, mGi, P(grads), P(outs), ws)
        else:
            kf.kfac_update_factors_batched(descs, acts, gouts, b, h, w, sA, sG, decay, A_run, G_run, ws)
            kf.kfac_invert_batched(descs, A_run, G_run, damping, damping, A_inv, G_inv, info, ws)
            kf.kfac_precondition_batched(descs, A_inv, G_inv, grads, outs, ws)
    else:
        for i in range(n):
            ws = workspace(kf.kfac_workspace_bytes(descs[i], b[i], h[i], w[i]))
            kf.kfac_update_factors(descs[i], acts[i], gouts[i], b[i], h[i], w[i], sA[i], sG[i], decay, A_run[i],
                                   G_run[i], ws)
            kf.kfac_invert(descs[i], A_run[i], G_run[i], damping, damping, A_inv[i], G_inv[i], info[2 * i:], ws)
            kf.kfac_precondition(descs[i], A_inv[i], G_inv[i], grads[i], outs[i], ws)
    torch.cuda.synchronize()
    res = []
    inf = info.cpu().numpy()
    for i in range(n):
        res.append(dict(A=A_run[i].cpu().numpy(), G=G_run[i].cpu().numpy(), A_inv=A_inv[i].cpu().numpy(),
                        G_inv=G_inv[i].cpu().numpy(), P=outs[i].cpu().numpy(), info=inf[2 * i:2 * i + 2]))
    return res


def run_layer_oracle(layer, inp, scale, decay, damping, A0=None, G0=None):
    act, gout, grad = inp
    A0 = np.eye(layer.d_A) if A0 is None else A0
    G0 = np.eye(layer.d_G) if G0 is None else G0
    A, G = orc.update_factors_layer(layer, act, gout, scale[0], scale[1], decay, A0, G0)
    Ai, Gi = orc.invert_layer(A, G, damping, damping)
    P = orc.precondition_layer(Ai, Gi, grad)
    return dict(A=A, G=G, A_inv=Ai, G_inv=Gi, P=P)


def check_layer(gpu, ref, tol_factor=1e-4, tol_inv=1e-4, tol_p=1e-3, tag=""):
    errs = {k: rel_fro(gpu[k], ref[k]) for k in ("A", "G", "A_inv", "G_inv", "P")}
    assert list(gpu["info"]) == [0, 0], f"{tag}: info {gpu['info']}"
    assert errs["A"] < tol_factor and errs["G"] < tol_factor, f"{tag}: factor error {errs}"
    assert errs["A_inv"] < tol_inv and errs["G_inv"] < tol_inv, f"{tag}: inverse error {errs}"
    assert errs["P"] < tol_p, f"{tag}: preconditioned gradient error {errs}"
    for k in ("A", "G", "A_inv", "G_inv"):
        assert np.array_equal(gpu[k], gpu[k].T), f"{tag}: {k} not bitwise symmetric"
    return errs


def draw_inputs(layers, batch, seed0, act_kind, gout_std, dtype="f32"):
    return [rng.layer_inputs(l, batch, seed0 + i, act_kind, gout_std, dtype) for i, l in enumerate(layers)]


def scales_for(layers, batch):
    return [shapes.layer_scales(l, batch) for l in layers]

"""GPU parity of the eigen-decomposition variant (Eq. 13): kfac_eigen and kfac_precondition_eigen
through the C ABI against the CPU oracle.

Eigenvectors are unique only up to sign (and up to rotations inside a repeated eigenvalue), so the
decomposition is compared through what is unique -- the sorted eigenvalues, and the preconditioned
gradient built from it -- and checked for validity: Q orthogonal, M Q = Q diag(v).

Tolerances (fp32 working precision eps = 6e-8 on the device, fp64 oracle): eigenvalues carry an absolute
error of a modest multiple of eps * ||M||_2 (2e-6 * lambda_max asserted, ~1e-7 measured); each of the
few hundred 32-row transforms applied to a row of V adds an eps-sized orthogonality defect
(||Q^T Q - I||_F / sqrt(n) < 1e-4 asserted, up to 1.4e-5 measured at n = 577); the residual
||M Q - Q diag(v)||_F / ||M||_F < 2e-5 (4e-6 measured); the preconditioned gradient keeps the 1e-3
relative Frobenius bound of the inverse variant.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2206_15143_amd as kf
from oracle import kfac_oracle as orc
from workloads import rng, shapes
from workloads.shapes import LayerSpec

import gpu_util as gu


def _factor_like(seed, n, rows=None, relu=True, scale=1.0):
    rows = rows or 3 * n + 5
    X = rng.draw_relu_normal(seed, 0, (rows, n)) if relu else rng.draw_normal(seed, 0, (rows, n))
    X = X.astype(np.float64)
    return (0.95 * np.eye(n) + 0.05 * scale * X.T @ X).astype(np.float32)


def _gpu_eigen(desc, A, G):
    dA, dG = A.shape[0], G.shape[0]
    QA = torch.full((dA, dA), float("nan"), device=gu.DEV)
    QG = torch.full((dG, dG), float("nan"), device=gu.DEV)
    vA = torch.full((dA,), float("nan"), device=gu.DEV)
    vG = torch.full((dG,), float("nan"), device=gu.DEV)
    info = torch.full((2,), -1, dtype=torch.int32, device=gu.DEV)
    ws = gu.workspace(kf.kfac_workspace_bytes(desc, 8))
    kf.kfac_eigen(desc, gu.to_dev(A), gu.to_dev(G), QA, vA, QG, vG, info, ws)
    torch.cuda.synchronize()
    return QA.cpu().numpy(), vA.cpu().numpy(), QG.cpu().numpy(), vG.cpu().numpy(), info.cpu().numpy()


def _check_decomposition(M, Q, v, tag):
    n = M.shape[0]
    Md, Qd, vd = M.astype(np.float64), Q.astype(np.float64), v.astype(np.float64)
    ref_v, _ = orc.eigh(Md)
    lam_max = max(abs(ref_v[0]), abs(ref_v[-1]))
    e_val = np.abs(np.sort(vd) - ref_v).max() / lam_max
    e_orth = np.linalg.norm(Qd.T @ Qd - np.eye(n)) / np.sqrt(n)
    e_res = np.linalg.norm(Md @ Qd - Qd * vd) / np.linalg.norm(Md)
    print(f"{tag}: eigenvalues {e_val:.2e} orthogonality {e_orth:.2e} residual {e_res:.2e}", flush=True)
    assert e_val <= 2e-6, tag
    assert e_orth < 1e-4, tag
    assert e_res < 2e-5, tag


@pytest.mark.parametrize("n", [1, 2, 5, 16, 17, 33, 64, 100, 145, 289])
def test_eigen_decomposition_sizes(n):
    A = _factor_like(300 + n, n, scale=0.5)
    G = _factor_like(400 + n, 7, relu=False)
    desc = kf.LayerDesc.linear(n, 7, has_bias=False)
    QA, vA, QG, vG, info = _gpu_eigen(desc, A, G)
    assert list(info) == [0, 0]
    _check_decomposition(A, QA, vA, f"A n={n}")
    _check_decomposition(G, QG, vG, "G n=7")


def test_eigen_special_matrices():
    desc = kf.LayerDesc.linear(40, 24, has_bias=False)
    # identity: nothing to rotate, Q = I exactly; diagonal with a repeated entry
    A = np.eye(40, dtype=np.float32)
    G = np.diag(np.r_[np.full(12, 2.0), np.arange(1, 13)]).astype(np.float32)
    QA, vA, QG, vG, info = _gpu_eigen(desc, A, G)
    assert list(info) == [0, 0]
    assert np.array_equal(QA, np.eye(40)) and np.array_equal(vA, np.ones(40))
    assert np.array_equal(QG, np.eye(24)) and np.array_equal(vG, np.diag(G))
    # c I + u u^T: one eigenvalue c + |u|^2, the others c (a 39-fold repeated eigenvalue)
    u = rng.draw_normal(61, 0, (40,)).astype(np.float64)
    A = (0.7 * np.eye(40) + np.outer(u, u)).astype(np.float32)
    # only the lower triangle is read
    Gl = _factor_like(62, 24)
    Gin = np.tril(Gl) + np.triu(np.full((24, 24), 7.0, dtype=np.float32), 1)
    QA, vA, QG, vG, info = _gpu_eigen(desc, A, Gin)
    assert list(info) == [0, 0]
    sv = np.sort(vA.astype(np.float64))
    assert np.allclose(sv[:-1], 0.7, atol=2e-6 * sv[-1]) and abs(sv[-1] - (0.7 + u @ u)) < 2e-6 * sv[-1]
    _check_decomposition(A, QA, vA, "rank one plus identity")
    _check_decomposition(Gl, QG, vG, "lower triangle")


def test_eigen_sweep_budget_is_reported():
    # one sweep cannot diagonalise a dense 100 x 100 factor: info says so and nothing else goes wrong
    A = _factor_like(70, 100)
    G = np.eye(3, dtype=np.float32)
    desc = kf.LayerDesc.linear(100, 3, has_bias=False)
    kf.kfac_tune("eigen_max_sweeps", 1)
    try:
        QA, vA, QG, vG, info = _gpu_eigen(desc, A, G)
    finally:
        kf.kfac_tune("eigen_max_sweeps", 20)
    assert list(info) == [1, 0]
    Qd = QA.astype(np.float64)
    assert np.linalg.norm(Qd.T @ Qd - np.eye(100)) / 10 < 1e-3       # still an orthogonal iterate


@pytest.mark.parametrize("dA,dG,gamma", [(1, 1, 0.5), (20, 7, 0.03), (65, 32, 0.03), (145, 16, 0.001), (300, 150, 0.01)])
def test_precondition_eigen_given_oracle_decomposition(dA, dG, gamma):
    # the four products and the division alone: Q, v from the oracle (rounded to fp32, and the oracle
    # then works from those same bits)
    A = _factor_like(500 + dA, dA).astype(np.float64)
    G = _factor_like(600 + dG, dG, relu=False).astype(np.float64)
    vA, QA = orc.eigh(A)
    vG, QG = orc.eigh(G)
    QA, vA, QG, vG = (x.astype(np.float32) for x in (QA, vA, QG, vG))
    grad = rng.draw_normal(700 + dA, 2, (dG, dA)).astype(np.float32)
    desc = kf.LayerDesc.linear(dA, dG, has_bias=False)
    out = torch.full((dG, dA), float("nan"), device=gu.DEV)
    ws = gu.workspace(kf.kfac_workspace_bytes(desc, 8))
    kf.kfac_precondition_eigen(desc, gu.to_dev(QA), gu.to_dev(vA), gu.to_dev(QG), gu.to_dev(vG), gamma,
                               gu.to_dev(grad), out, ws)
    torch.cuda.synchronize()
    ref = orc.precondition_eigen(QG, vG, QA, vA, grad, gamma)
    assert gu.rel_fro(out.cpu().numpy(), ref) < 1e-5


def _eigen_path_gpu(layers, batch, inputs, scales, decay, gamma, batched):
    n = len(layers)
    descs = [kf.LayerDesc.from_spec(l) for l in layers]
    b, h, w = gu.batch_args(layers, batch)
    acts = [gu.to_dev(i[0]) for i in inputs]
    gouts = [gu.to_dev(i[1]) for i in inputs]
    grads = [gu.to_dev(i[2]) for i in inputs]
    dA = [kf.kfac_dim_A(d) for d in descs]
    dG = [kf.kfac_dim_G(d) for d in descs]
    A_run = [torch.eye(a, device=gu.DEV) for a in dA]
    G_run = [torch.eye(g, device=gu.DEV) for g in dG]
    QA = [torch.full((a, a), float("nan"), device=gu.DEV) for a in dA]
    QG = [torch.full((g, g), float("nan"), device=gu.DEV) for g in dG]
    vA = [torch.full((a,), float("nan"), device=gu.DEV) for a in dA]
    vG = [torch.full((g,), float("nan"), device=gu.DEV) for g in dG]
    outs = [torch.full((g, a), float("nan"), device=gu.DEV) for a, g in zip(dA, dG)]
    info = torch.full((2 * n,), -1, dtype=torch.int32, device=gu.DEV)
    sA = [s[0] for s in scales]
    sG = [s[1] for s in scales]
    if batched:
        ws = gu.workspace(kf.kfac_workspace_bytes_batched(descs, b, h, w))
        kf.kfac_update_factors_batched(descs, acts, gouts, b, h, w, sA, sG, decay, A_run, G_run, ws)
        kf.kfac_eigen_batched(descs, A_run, G_run, QA, vA, QG, vG, info, ws)
        kf.kfac_precondition_eigen_batched(descs, QA, vA, QG, vG, gamma, grads, outs, ws)
    else:
        for i in range(n):
            ws = gu.workspace(kf.kfac_workspace_bytes(descs[i], b[i], h[i], w[i]))
            kf.kfac_update_factors(descs[i], acts[i], gouts[i], b[i], h[i], w[i], sA[i], sG[i], decay, A_run[i],
                                   G_run[i], ws)
            kf.kfac_eigen(descs[i], A_run[i], G_run[i], QA[i], vA[i], QG[i], vG[i], info[2 * i:], ws)
            kf.kfac_precondition_eigen(descs[i], QA[i], vA[i], QG[i], vG[i], gamma, grads[i], outs[i], ws)
    torch.cuda.synchronize()
    return [dict(A=A_run[i].cpu().numpy(), G=G_run[i].cpu().numpy(), QA=QA[i].cpu().numpy(), vA=vA[i].cpu().numpy(),
                 QG=QG[i].cpu().numpy(), vG=vG[i].cpu().numpy(), P=outs[i].cpu().numpy()) for i in range(n)], \
        info.cpu().numpy()


@pytest.mark.parametrize("batched", [True, False])
def test_eigen_variant_end_to_end_mixed_layers(batched):
    # factors -> eigen-decompositions -> Eq. 13, several layer kinds and orders in one grouped call
    layers = [LayerSpec("linear", 64, 32, rows=32), LayerSpec("conv", 16, 16, 3, 1, 1, 8),
              LayerSpec("conv", 8, 24, 1, 1, 0, 6), LayerSpec("linear", 150, 40, rows=257, has_bias=False),
              LayerSpec("conv", 16, 16, 3, 1, 1, 8), LayerSpec("conv", 3, 10, 5, 2, 2, 13)]
    batch, decay, gamma = 4, 0.95, 0.01
    inputs = gu.draw_inputs(layers, batch, 8800, "relu_normal", 0.0316)
    scales = gu.scales_for(layers, batch)
    res, info = _eigen_path_gpu(layers, batch, inputs, scales, decay, gamma, batched)
    assert not info.any()
    for i, l in enumerate(layers):
        print(f"layer {i}: {l}", flush=True)
        A, G = orc.update_factors_layer(l, inputs[i][0], inputs[i][1], scales[i][0], scales[i][1], decay,
                                        np.eye(l.d_A), np.eye(l.d_G))
        ref = orc.precondition_eigen_layer(A, G, inputs[i][2], gamma)
        g = res[i]
        _check_decomposition(g["A"], g["QA"], g["vA"], f"layer {i} A")
        _check_decomposition(g["G"], g["QG"], g["vG"], f"layer {i} G")
        e_p = gu.rel_fro(g["P"], ref)
        print(f"layer {i}: preconditioned gradient {e_p:.2e}", flush=True)
        assert e_p < 1e-3, i


def test_eigen_variant_resnet110_shapes_full_size():
    # the three conv shapes, the stem and the classifier of the ResNet-110-shaped workload at full size
    name = "resnet110_cifar"
    hp = shapes.config_hparams(name)
    allz = shapes.config_layers(name)
    layers = [allz[0], allz[1], allz[37], allz[73], allz[109]]
    batch = hp["batch"]
    inputs = gu.draw_inputs(layers, batch, 8900, hp["act"], hp["gout_var"] ** 0.5)
    scales = gu.scales_for(layers, batch)
    res, info = _eigen_path_gpu(layers, batch, inputs, scales, hp["decay"], hp["damping"], True)
    assert not info.any()
    for i, l in enumerate(layers):
        print(f"layer {i}: {l}", flush=True)
        A, G = orc.update_factors_layer(l, inputs[i][0], inputs[i][1], scales[i][0], scales[i][1], hp["decay"],
                                        np.eye(l.d_A), np.eye(l.d_G))
        ref = orc.precondition_eigen_layer(A, G, inputs[i][2], hp["damping"])
        g = res[i]
        _check_decomposition(g["A"], g["QA"], g["vA"], f"layer {i} A")
        e_p = gu.rel_fro(g["P"], ref)
        print(f"layer {i}: preconditioned gradient {e_p:.2e}", flush=True)
        assert e_p < 1e-3, i


def test_eigen_variant_order_1153_full_size():
    """A ResNet-50-shaped 3x3 layer at full size (d_A = 1153, d_G = 128, 25 088 patch rows).  The oracle's cyclic
    Jacobi iteration would take minutes at this order, so the decomposition is checked through what defines it --
    Q orthogonal and M Q = Q diag(v), which together bound every eigenvalue's error by the residual -- and the
    preconditioned gradient through the equation Eq. 13 solves exactly, (A (x) G + gamma I) vec(P) = vec(grad),
    i.e. G P A + gamma P = grad, with the oracle's own factors A and G (fp64, from the same inputs)."""
    hp = shapes.config_hparams("resnet50_imagenet")
    l = LayerSpec("conv", 128, 128, 3, 1, 1, 28)
    batch, decay, gamma = hp["batch"], hp["decay"], 0.01
    inputs = gu.draw_inputs([l], batch, 8950, hp["act"], hp["gout_var"] ** 0.5)
    scales = gu.scales_for([l], batch)
    res, info = _eigen_path_gpu([l], batch, inputs, scales, decay, gamma, True)
    assert not info.any()
    g = res[0]
    A, G = orc.update_factors_layer(l, inputs[0][0], inputs[0][1], scales[0][0], scales[0][1], decay,
                                    np.eye(l.d_A), np.eye(l.d_G))
    assert gu.rel_fro(g["A"], A) < 1e-4 and gu.rel_fro(g["G"], G) < 1e-4
    for M, Q, v, tag in ((g["A"], g["QA"], g["vA"], "A"), (g["G"], g["QG"], g["vG"], "G")):
        n = M.shape[0]
        Md, Qd, vd = M.astype(np.float64), Q.astype(np.float64), v.astype(np.float64)
        e_orth = np.linalg.norm(Qd.T @ Qd - np.eye(n)) / np.sqrt(n)
        e_res = np.linalg.norm(Md @ Qd - Qd * vd) / np.linalg.norm(Md)
        e_tr = abs(vd.sum() - np.trace(Md)) / np.trace(Md)
        print(f"{tag} n={n}: orthogonality {e_orth:.2e} residual {e_res:.2e} trace {e_tr:.2e}", flush=True)
        assert e_orth < 1e-4 and e_res < 2e-5 and e_tr < 1e-5, tag
        assert vd.min() > 0.9 * decay           # a running average started at the identity: M >= decay I
    P = g["P"].astype(np.float64)
    grad = inputs[0][2].astype(np.float64)
    resid = G @ P @ A + gamma * P - grad
    # ||P - P*||_F <= ||resid||_F / (lambda_min(A) lambda_min(G) + gamma), lambda_min >= decay
    bound = np.linalg.norm(resid) / (decay * decay + gamma) / np.linalg.norm(P)
    print(f"preconditioned gradient: residual bound {bound:.2e}", flush=True)
    assert bound < 1e-3

"""GPU parity at the full sizes of the workload configs, in the launch
configuration bench.py times (batched entry points over the whole layer set).

Where the oracle can produce the whole result in seconds it is compared
element by element; for the largest matrices the factors are compared on
sampled entries the oracle computes one by one, and the inverse and the
preconditioned gradient through properties that hold at any size (the residual
||M X - I||_F bounds the relative error of X, and the oracle's own two-sided
product of the GPU inverses isolates the last stage).
"""
from collections import Counter

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2206_15143_amd as kf
from oracle import kfac_oracle as orc
from workloads import rng, shapes

import gpu_util as gu


def _residual(M, X, lam):
    """||(M + lam I) X - I||_F in fp64 (upper bound of the relative Frobenius error of X)."""
    Md = torch.from_numpy(M).to(gu.DEV, torch.float64)
    Md = Md + lam * torch.eye(Md.shape[0], device=gu.DEV, dtype=torch.float64)
    Xd = torch.from_numpy(X).to(gu.DEV, torch.float64)
    R = Md @ Xd - torch.eye(Md.shape[0], device=gu.DEV, dtype=torch.float64)
    return float(torch.linalg.norm(R))


def test_resnet110_config_batched_full_size():
    name = "resnet110_cifar"
    hp = shapes.config_hparams(name)
    layers = shapes.config_layers(name)
    batch = hp["batch"]
    std = hp["gout_var"] ** 0.5
    print("drawing inputs", flush=True)
    inputs = gu.draw_inputs(layers, batch, 1000 * hp["index"], hp["act"], std)
    scales = gu.scales_for(layers, batch)
    print("gpu run", flush=True)
    gpu = gu.run_layers_gpu(layers, batch, inputs, scales, hp["decay"], hp["damping"], batched=True)
    worst = {}
    for i in range(len(layers)):      # every layer against the oracle's whole chain
        ref = gu.run_layer_oracle(layers[i], inputs[i], scales[i], hp["decay"], hp["damping"])
        errs = gu.check_layer(gpu[i], ref, tag=f"{name} layer {i}")
        for k, v in errs.items():
            worst[k] = max(worst.get(k, 0.0), v)
        if i % 10 == 9:
            print(f"{i + 1} layers compared with the oracle", flush=True)
    print("worst relative Frobenius errors over the 110 layers:", {k: f"{v:.2e}" for k, v in worst.items()}, flush=True)
    lam = hp["damping"]
    for i, l in enumerate(layers):
        g = gpu[i]
        assert list(g["info"]) == [0, 0]
        for k in ("A", "G", "A_inv", "G_inv"):
            assert np.array_equal(g[k], g[k].T), (i, k)
        assert _residual(g["A"], g["A_inv"], lam) < 1e-4, i
        assert _residual(g["G"], g["G_inv"], lam) < 1e-4, i
        # bias corner of A: 0.95 + 0.05 * (rows / batch)
        corner = orc.running_average(np.eye(1), np.array([[scales[i][0] * l.n_rows(batch)]]), hp["decay"])[0, 0]
        assert abs(g["A"][-1, -1] - corner) <= 1e-6 * corner


FULL_SIZE_CONFIGS = [("resnet50_imagenet", 24), ("resnet50_imagenet_bf16", 24), ("transformer_encoder_bf16", 3),
                     ("vgg16_cifar", 11), ("inception_nonsquare", 7), ("bert_base_small_batch", 3)]


def _distinct(name):
    return list(Counter(shapes.config_layers(name)).keys())


def _shape_cases():
    cases = []
    for name, n in FULL_SIZE_CONFIGS:
        d = _distinct(name)
        assert len(d) == n, (name, len(d))
        cases += [pytest.param(name, i, id=f"{name}-{i}") for i in range(n)]
    return cases


@pytest.mark.parametrize("name,i", _shape_cases())
def test_distinct_shapes_full_size(name, i):
    """Every distinct layer shape of the ResNet-50-shaped (fp32 B=32, bf16 B=64), transformer-shaped
    (bf16, 4096 token rows), VGG-16-shaped, non-square-kernel and small-batch BERT-shaped layer sets at
    full size, through the batched entry points."""
    hp = shapes.config_hparams(name)
    batch = hp["batch"]
    lam = hp["damping"]
    std = hp["gout_var"] ** 0.5
    dtype = hp["dtype"]
    l = _distinct(name)[i]
    gen = np.random.default_rng(3 + i)
    print(f"{name} shape {i}: {l}", flush=True)
    inp = rng.layer_inputs(l, batch, 1000 * hp["index"] + 500 + i, hp["act"], std, dtype)
    sc = shapes.layer_scales(l, batch)
    g = gu.run_layers_gpu([l], batch, [inp], [sc], hp["decay"], lam, dtype=dtype, batched=True)[0]
    assert list(g["info"]) == [0, 0]
    abar, grow = orc.layer_rows(l, inp[0], inp[1])
    if l.d_A <= 300 or (l.d_A <= 600 and l.n_rows(batch) <= 110000):
        ref = gu.run_layer_oracle(l, inp, sc, hp["decay"], lam)
        errs = gu.check_layer(g, ref, tag=str(l))
        print({k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
        return
    # sampled entries of both factors, straight from the definition
    for F, X, s, d in ((g["A"], abar, sc[0], l.d_A), (g["G"], grow, sc[1], l.d_G)):
        us = np.concatenate([gen.integers(0, d, 40), [d - 1, d - 1, 0]])
        vs = np.concatenate([gen.integers(0, d, 40), [d - 1, 0, 0]])
        ref = np.array([orc.running_average(np.array([[1.0 if u == v else 0.0]]),
                                            np.array([[orc.factor_entry(X, s, int(u), int(v))]]),
                                            hp["decay"])[0, 0] for u, v in zip(us, vs)])
        got = F[us, vs].astype(np.float64)
        assert np.linalg.norm(got - ref) / np.linalg.norm(ref) < 1e-4
        assert np.array_equal(F, F.T)
    # Freivalds check of both factors: F z against decay z + (1 - decay) s X^T (X z) for random +-1 vectors, from
    # the oracle's rows in fp64: a wrong tile anywhere in the factor shows, which sampled entries would miss
    for F, X, s, d in ((g["A"], abar, sc[0], l.d_A), (g["G"], grow, sc[1], l.d_G)):
        z = gen.integers(0, 2, size=(d, 4)).astype(np.float64) * 2.0 - 1.0
        want = hp["decay"] * z + (1.0 - hp["decay"]) * s * (X.T @ (X @ z))
        got = (torch.from_numpy(F).to(gu.DEV, torch.float64) @ torch.from_numpy(z).to(gu.DEV)).cpu().numpy()
        assert np.linalg.norm(got - want) / np.linalg.norm(want) < 1e-4
    # trace of the new A factor = scale * ||abar||_F^2 (cheap at any size)
    tr_new = (np.trace(g["A"].astype(np.float64)) - hp["decay"] * l.d_A) / (1 - hp["decay"])
    assert abs(tr_new - sc[0] * (abar ** 2).sum()) <= 1e-4 * tr_new
    del abar, grow
    for F, X in ((g["A"], g["A_inv"]), (g["G"], g["G_inv"])):
        assert np.array_equal(X, X.T)
        if F.shape[0] <= 1600:
            assert gu.rel_fro(X, orc.inverse(F.astype(np.float64), lam)) < 1e-4
        else:
            # X - M^-1 = M^-1 (M X - I) and M >= (decay + lam) I for a running average started at
            # the identity, so ||X - M^-1||_F <= ||M X - I||_F / (decay + lam)
            bound = _residual(F, X, lam) / (hp["decay"] + lam)
            assert bound / np.linalg.norm(X.astype(np.float64)) < 1e-4
    Pref = orc.precondition(g["G_inv"].astype(np.float64), inp[2].astype(np.float64),
                            g["A_inv"].astype(np.float64))
    assert gu.rel_fro(g["P"], Pref) < 1e-3

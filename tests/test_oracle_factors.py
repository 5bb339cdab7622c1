"""Pins for the oracle's patch extraction, factor construction and running average.

Nothing here re-types the oracle's own formula: each check is a closed form,
an invariant, or an independent library route (torch.conv2d, numpy matmul,
eigvalsh, matrix_rank).
"""
import numpy as np
import pytest
import torch

from oracle import kfac_oracle as orc
from workloads import rng, shapes


def _x(seed, shape):
    return rng.draw_normal(seed, 0, shape)


@pytest.mark.parametrize("C,H,W", [(3, 5, 4), (8, 7, 7)])
def test_patches_1x1_is_the_nchw_to_rows_permutation(C, H, W):
    x = _x(1, (2, C, H, W))
    p = orc.patches(x, 1, 1, 1, 0, has_bias=False)
    ref = np.transpose(x, (0, 2, 3, 1)).reshape(-1, C)
    assert np.array_equal(p, ref.astype(np.float64))
    assert np.array_equal(orc.rows_from_nchw(x), ref.astype(np.float64))


@pytest.mark.parametrize("k,stride,pad,H,W", [(3, 1, 1, 6, 5), (3, 2, 1, 8, 8), (7, 2, 3, 14, 14),
                                                (1, 2, 0, 8, 6), (3, 1, 0, 5, 5), (5, 3, 2, 11, 9)])
def test_patches_times_flat_weight_is_a_convolution(k, stride, pad, H, W):
    # pins column order (c, i, j), row order (n, oh, ow), zero padding, stride
    B, C, Co = 2, 3, 4
    x = _x(2, (B, C, H, W))
    w = rng.draw_normal(3, 1, (Co, C, k, k))
    bias = rng.draw_normal(3, 2, (Co,))
    p = orc.patches(x, k, k, stride, pad, has_bias=True)
    wflat = np.concatenate([w.reshape(Co, -1), bias[:, None]], axis=1).astype(np.float64)
    got = p @ wflat.T                                                     # [R, Co]
    ref = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                     torch.from_numpy(bias).double(), stride=stride, padding=pad)
    Ho, Wo = ref.shape[2], ref.shape[3]
    assert p.shape[0] == B * Ho * Wo
    ref = ref.permute(0, 2, 3, 1).reshape(-1, Co).numpy()
    assert np.allclose(got, ref, rtol=1e-12, atol=1e-12)
    assert np.all(p[:, -1] == 1.0)


@pytest.mark.parametrize("kh,kw,stride,ph,pw,H,W", [(1, 7, 1, 0, 3, 9, 10), (7, 1, 1, 3, 0, 9, 10), (1, 3, 1, 0, 1, 5, 7),
                                                     (3, 1, 1, 1, 0, 5, 7), (3, 5, 2, 0, 2, 9, 11), (3, 3, 1, 2, 0, 6, 6)])
def test_patches_with_different_row_and_column_padding_is_a_convolution(kh, kw, stride, ph, pw, H, W):
    # the padding of the rows and of the columns are separate arguments: swapping them, or using one for both,
    # changes either the shape or the zero pattern of the patches and fails here
    B, C, Co = 2, 3, 4
    x = _x(12, (B, C, H, W))
    w = rng.draw_normal(13, 1, (Co, C, kh, kw))
    p = orc.patches(x, kh, kw, stride, ph, has_bias=False, pad_w=pw)
    got = p @ w.reshape(Co, -1).astype(np.float64).T
    ref = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(), None,
                                     stride=stride, padding=(ph, pw))
    assert p.shape == (B * ref.shape[2] * ref.shape[3], C * kh * kw)
    assert np.allclose(got, ref.permute(0, 2, 3, 1).reshape(-1, Co).numpy(), rtol=1e-12, atol=1e-12)


def test_patches_one_sided_padding_zero_count_closed_form():
    # all-ones input, 1 x 7 kernel padded by 3 columns only: output H x W, and of the 7 taps of output column ow
    # min(ow, 3) + min(W - 1 - ow, 3) ... fall outside: in-bounds taps per row of the map = 7 W - 12 (W >= 4);
    # no row of the map is padded, so a 7 x 1 kernel with the same arguments swapped gives 7 H - 12 per column
    B, C, H, W = 2, 3, 5, 9
    ones = np.ones((B, C, H, W), np.float32)
    p = orc.patches(ones, 1, 7, 1, 0, has_bias=False, pad_w=3)
    assert p.shape == (B * H * W, 7 * C) and p.sum() == B * C * H * (7 * W - 12)
    q = orc.patches(ones, 7, 1, 1, 3, has_bias=False, pad_w=0)
    assert q.shape == (B * H * W, 7 * C) and q.sum() == B * C * W * (7 * H - 12)
    # pad_w left out: the same padding in both directions, as before
    assert np.array_equal(orc.patches(ones, 3, 3, 1, 1, has_bias=False), orc.patches(ones, 3, 3, 1, 1, False, pad_w=1))


def test_patches_padding_zero_count_closed_form():
    # all-ones input: every zero comes from padding.  For 3x3, stride 1, pad 1
    # on HxW the number of in-bounds taps is (3H-2)(3W-2) per channel and image.
    B, C, H, W = 2, 3, 6, 9
    p = orc.patches(np.ones((B, C, H, W), np.float32), 3, 3, 1, 1, has_bias=False)
    assert p.shape == (B * H * W, 27)
    assert p.sum() == B * C * (3 * H - 2) * (3 * W - 2)
    assert (p == 0).sum() == B * C * (9 * H * W - (3 * H - 2) * (3 * W - 2))


def test_factor_closed_forms():
    R, d, s = 37, 6, 0.25
    assert np.array_equal(orc.factor(np.ones((R, d)), s), np.full((d, d), s * R))
    idx = np.array([0, 2, 2, 5, 5, 5, 1])
    onehot = np.eye(d)[idx]
    assert np.array_equal(orc.factor(onehot, 1.0), np.diag(np.bincount(idx, minlength=d).astype(float)))


def test_factor_invariants_and_library_route():
    R, d = 50, 9
    X = _x(5, (R, d)).astype(np.float64)
    F = orc.factor(X, 1.0 / R)
    assert np.array_equal(F, F.T)                                       # exact symmetry
    assert np.allclose(F, X.T @ X / R, rtol=1e-13, atol=1e-13)          # numpy route
    assert np.isclose(np.trace(F), (X ** 2).sum() / R, rtol=1e-13)
    assert np.linalg.eigvalsh(F).min() >= -1e-12 * np.linalg.norm(F)
    assert np.allclose(orc.factor(X, 3.0 / R), 3.0 * F, rtol=1e-14)     # linear in scale
    perm = np.random.default_rng(0).permutation(R)
    assert np.allclose(orc.factor(X[perm], 1.0 / R), F, rtol=1e-12, atol=1e-14)
    # a non-symmetric probe: entry (u, v) pairs column u with column v
    assert np.isclose(orc.factor_entry(X, 1.0 / R, 2, 7), (X[:, 2] * X[:, 7]).sum() / R, rtol=1e-13)


@pytest.mark.parametrize("R,d", [(3, 8), (5, 12), (1, 4)])
def test_unaveraged_factor_has_rank_at_most_R(R, d):
    X = _x(6, (R, d)).astype(np.float64)
    F = orc.factor(X, 1.0)
    assert np.linalg.matrix_rank(F, tol=1e-9) == min(R, d)
    w = np.linalg.eigvalsh(F)
    assert (w > 1e-9).sum() == R and w.min() > -1e-10


def test_bias_column_border_of_A():
    # with the homogeneous column last: A[-1,-1] = s*R and A[:, -1] = s * column sums
    layer = shapes.LayerSpec("conv", 3, 4, 3, 1, 1, 6)
    act = rng.draw_relu_normal(9, 0, (2, 3, 6, 6))
    abar = orc.patches(act, 3, 3, 1, 1, True)
    A = orc.factor(abar, 0.5)
    R = abar.shape[0]
    assert A[-1, -1] == 0.5 * R
    assert np.allclose(A[:-1, -1], 0.5 * abar[:, :-1].sum(axis=0), rtol=1e-13)
    # centre tap (i=j=1) of channel c sees every pixel exactly once
    for c in range(3):
        assert np.isclose(A[c * 9 + 4, -1], 0.5 * act[:, c].astype(np.float64).sum(), rtol=1e-12)
    assert layer.d_A == A.shape[0]


def test_G_from_nchw_equals_einsum_over_positions():
    g = rng.draw_normal(4, 1, (3, 5, 4, 6), std=0.1)
    G = orc.factor(orc.rows_from_nchw(g), 1.0 / 3)
    ref = np.einsum("nchw,ndhw->cd", g.astype(np.float64), g.astype(np.float64)) / 3
    assert np.allclose(G, ref, rtol=1e-12, atol=1e-15)


def test_running_average_ends_and_closed_form():
    d = 5
    F0 = np.eye(d)
    gen = np.random.default_rng(1)
    news = [(lambda M: M @ M.T)(gen.standard_normal((d, d))) for _ in range(6)]
    assert np.array_equal(orc.running_average(F0, news[0], 0.0), news[0])   # decay 0 -> new factor
    assert np.array_equal(orc.running_average(F0, news[0], 1.0), F0)        # decay 1 -> unchanged
    decay = 0.95
    F = F0
    for Fn in news:
        F = orc.running_average(F, Fn, decay)
    T = len(news)
    closed = decay ** T * F0 + (1 - decay) * sum(decay ** (T - 1 - k) * news[k] for k in range(T))
    assert np.allclose(F, closed, rtol=1e-13, atol=1e-14)
    # the weight on the OLD factor is `decay` (0.95 in section 6.1): one step from identity
    one = orc.running_average(np.eye(2), np.array([[3.0, 1.0], [1.0, 2.0]]), 0.95)
    assert np.allclose(one, [[0.95 + 0.15, 0.05], [0.05, 0.95 + 0.10]], rtol=1e-14)

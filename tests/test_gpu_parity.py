"""GPU parity: the HIP library (through the C-ABI binding) against the CPU oracle,
element by element on the same seeded inputs.

Tolerances (relative Frobenius error, from the benchmark spec): 1e-4 for the
fp32 factors, 1e-4 for the inverses, 1e-3 for the preconditioned gradient.
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


def _run_and_check(layers, batch, seed, act_kind="relu_normal", gout_std=0.0316, decay=0.95, damping=0.03,
                   dtype="f32", batched=True, tols=(1e-4, 1e-4, 1e-3)):
    inputs = gu.draw_inputs(layers, batch, seed, act_kind, gout_std, dtype)
    scales = gu.scales_for(layers, batch)
    gpu = gu.run_layers_gpu(layers, batch, inputs, scales, decay, damping, dtype, batched)
    out = []
    for i, l in enumerate(layers):
        print(f"layer {i}: {l}", flush=True)
        ref = gu.run_layer_oracle(l, inputs[i], scales[i], decay, damping)
        out.append(gu.check_layer(gpu[i], ref, *tols, tag=f"layer {i} {l.kind} dA={l.d_A} dG={l.d_G}"))
    return out


def test_config1_fc_tiny_end_to_end():
    layers = shapes.config_layers("fc_tiny")
    hp = shapes.config_hparams("fc_tiny")
    errs = _run_and_check(layers, hp["batch"], 1000, hp["act"], hp["gout_var"] ** 0.5, hp["decay"], hp["damping"],
                          batched=False)
    print(errs)


@pytest.mark.parametrize("d_in,d_out,rows,bias", [
    (20, 7, 50, True),        # one 32-tile, ragged everything
    (64, 32, 33, True),       # 64 + bias
    (144, 16, 300, True),     # the 144 tile config
    (150, 40, 257, False),    # just over 144, no bias, rows not a multiple of 16
    (300, 130, 100, True),    # several tiles per side, R < d (rank deficient before the average)
    (100, 40, 3000, True),    # two 64-tiles per side (diagonal and off-diagonal blocks), many K stages and splits: the
                              # prefetch ring of the small row-major tiles, aligned loads (ld = 100), long bias sums
    (45, 33, 777, False),     # odd row pitch (scalar loads), K = 48 stages + 9 rows, no bias
    (27, 16, 8200, True),     # the stem's shape class: 28-column factor, one 32-tile, hundreds of splits
])
def test_linear_layers(d_in, d_out, rows, bias):
    layer = LayerSpec("linear", d_in, d_out, rows=rows, has_bias=bias)
    _run_and_check([layer], rows, 2000 + d_in, act_kind="normal", gout_std=0.1, batched=False)


@pytest.mark.parametrize("cin,cout,k,stride,pad,h,batch", [
    (4, 6, 3, 1, 1, 8, 3),
    (16, 16, 3, 1, 1, 12, 2),
    (3, 8, 7, 2, 3, 20, 2),     # stem-like: odd C*k*k (147 -> padded ld)
    (8, 12, 1, 1, 0, 6, 3),     # 1x1 stride 1: NCHW read directly, HW % 4 == 0
    (8, 12, 1, 1, 0, 7, 3),     # 1x1 with HW = 49 (unaligned scalar path)
    (8, 16, 1, 2, 0, 8, 2),     # strided 1x1 projection
    (5, 4, 3, 2, 1, 9, 2),      # odd channels, stride 2
])
def test_conv_layers(cin, cout, k, stride, pad, h, batch):
    layer = LayerSpec("conv", cin, cout, k, stride, pad, h)
    _run_and_check([layer], batch, 3000 + cin * 10 + k, batched=False)


@pytest.mark.parametrize("cin,h,batch,bias", [
    (16, 32, 3, True),     # one macro tile, 4 output rows per stage (the 16-channel CIFAR shape)
    (16, 16, 5, False),    # no bias
    (32, 16, 3, True),     # two macro tiles: diagonal block with four different units
    (48, 8, 5, True),      # three macro tiles: full + single diagonal blocks and a row block
    (64, 8, 7, True),      # four macro tiles, whole image per stage
    (16, 28, 2, True),     # W = 28 (ImageNet stage 3 width)
])
def test_fused_3x3_conv_factor(cin, h, batch, bias):
    # 3x3 / stride 1 / pad 1 with C_in a multiple of 16: A is built straight from the NCHW input
    layer = LayerSpec("conv", cin, 8, 3, 1, 1, h, has_bias=bias)
    _run_and_check([layer], batch, 7000 + cin + h, batched=True)
    # same answer as the path through the materialised patch matrix
    inputs = gu.draw_inputs([layer], batch, 7100, "relu_normal", 0.05)
    scales = gu.scales_for([layer], batch)
    fused = gu.run_layers_gpu([layer], batch, inputs, scales, 0.95, 0.03)[0]
    kf.kfac_tune("fuse_conv3", 0)
    try:
        plain = gu.run_layers_gpu([layer], batch, inputs, scales, 0.95, 0.03)[0]
    finally:
        kf.kfac_tune("fuse_conv3", 1)
    assert gu.rel_fro(fused["A"], plain["A"]) < 1e-5


@pytest.mark.parametrize("cout,h,batch", [
    (16, 8, 5),      # one 16-tile, HW = 64
    (32, 6, 7),      # HW = 36: a multiple of 4 but not of 16 (ragged last k-group of every image)
    (48, 10, 3),     # three tiles (d between the 32 and 64 instances), HW = 100
    (64, 8, 9),      # four tiles
    (40, 4, 6),      # d not a multiple of 16, HW = 16
    (24, 7, 4),      # HW = 49 is not a multiple of 4: the block-tile kernel takes it
    (8, 12, 5),      # d = 8: the second load of the tile (channels 8..15) reads nothing; HW = 144 = 4.5 groups
    (16, 32, 3),     # HW = 1024, the map of config 2's first stage: 32 groups per image
])
def test_narrow_nchw_output_gradient_factor(cout, h, batch):
    # G of a conv layer with few output channels: read from NCHW by the direct (no-LDS) kernel
    layer = LayerSpec("conv", 4, cout, 3, 1, 1, h)
    _run_and_check([layer], batch, 7500 + cout + h, batched=True)
    inputs = gu.draw_inputs([layer], batch, 7600, "relu_normal", 0.05)
    scales = gu.scales_for([layer], batch)
    direct = gu.run_layers_gpu([layer], batch, inputs, scales, 0.95, 0.03)[0]
    kf.kfac_tune("use_small_kernel", 0)
    try:
        tiled = gu.run_layers_gpu([layer], batch, inputs, scales, 0.95, 0.03)[0]
    finally:
        kf.kfac_tune("use_small_kernel", 1)
    assert gu.rel_fro(direct["G"], tiled["G"]) < 1e-5


@pytest.mark.parametrize("cin,cout,h,batch,bias", [
    (144, 8, 6, 3, True),      # A of a 1x1 conv from NCHW: one macro tile, HW = 36 (4-position tail), bias border
    (136, 8, 13, 4, False),    # HW = 169 (odd: 4-byte aligned channel rows, 9-position tail), ragged last tile
    (8, 300, 8, 2, True),      # G with 300 channels: three macro tiles, HW = 64 (no tail)
    (288, 160, 12, 2, True),   # A two macro tiles, G two macro tiles (d = 160: 10 tiles), HW = 144
    (144, 8, 7, 3, True),      # HW = 49 would pad K by a quarter: the block-tile kernel takes it
    (2048 // 8, 130, 4, 2, True),   # d_A = 256 (2^n: padded by a quarter), HW = 16: one K tile per image
])
def test_wide_nchw_fp32_factors(cin, cout, h, batch, bias):
    # fp32 NCHW operands wider than 128 channels take the wave-unit kernel that stages [channel][position]
    layer = LayerSpec("conv", cin, cout, 1, 1, 0, h, has_bias=bias)
    _run_and_check([layer], batch, 7700 + cin + h, batched=True)
    inputs = gu.draw_inputs([layer], batch, 7800, "relu_normal", 0.05)
    scales = gu.scales_for([layer], batch)
    wave = gu.run_layers_gpu([layer], batch, inputs, scales, 0.95, 0.03)[0]
    kf.kfac_tune("use_wave_kernel", 0)
    try:
        tiled = gu.run_layers_gpu([layer], batch, inputs, scales, 0.95, 0.03)[0]
    finally:
        kf.kfac_tune("use_wave_kernel", 1)
    assert gu.rel_fro(wave["A"], tiled["A"]) < 1e-5
    assert gu.rel_fro(wave["G"], tiled["G"]) < 1e-5


def test_im2col_alone_is_bit_exact():
    for (cin, k, stride, pad, h, batch) in [(16, 3, 1, 1, 32, 2), (3, 7, 2, 3, 30, 2), (64, 3, 1, 1, 8, 3),
                                            (12, 1, 2, 0, 10, 2), (200, 3, 1, 1, 7, 1), (5, 3, 1, 1, 70, 1),
                                            (6, 5, 2, 2, 33, 2), (2, 3, 1, 0, 9, 3)]:
        print("im2col", cin, k, stride, pad, h, batch, flush=True)
        x = rng.draw_relu_normal(77, 0, (batch, cin, h, h))
        desc = kf.LayerDesc.conv2d(cin, 4, k, stride, pad)
        ld = kf.kfac_patch_ld(desc)
        ho = (h + 2 * pad - k) // stride + 1
        out = torch.full((batch * ho * ho, ld), float("nan"), device=gu.DEV)
        kf.kfac_im2col(desc, gu.to_dev(x), batch, h, h, out)
        torch.cuda.synchronize()
        ref = orc.patches(x, k, k, stride, pad, has_bias=False)
        got = out.cpu().numpy()
        assert np.array_equal(got[:, :ref.shape[1]].astype(np.float64), ref)
        assert np.all(got[:, ref.shape[1]:] == 0)


def test_im2col_nonsquare_kernels_and_maps_bit_exact():
    for (cin, kh, kw, stride, pad, h, w, batch) in [(8, 1, 7, 1, 0, 17, 17, 2), (8, 7, 1, 1, 0, 17, 23, 2),
                                                    (5, 1, 3, 1, 1, 8, 12, 3), (6, 3, 5, 2, 2, 21, 30, 2),
                                                    (4, 5, 2, 1, 0, 9, 40, 1), (16, 3, 3, 1, 1, 6, 50, 2)]:
        print("im2col", cin, kh, kw, stride, pad, h, w, batch, flush=True)
        x = rng.draw_relu_normal(78, 0, (batch, cin, h, w))
        desc = kf.LayerDesc.conv2d(cin, 4, kh, stride, pad, kw=kw)
        ld = kf.kfac_patch_ld(desc)
        ho = (h + 2 * pad - kh) // stride + 1
        wo = (w + 2 * pad - kw) // stride + 1
        out = torch.full((batch * ho * wo, ld), float("nan"), device=gu.DEV)
        kf.kfac_im2col(desc, gu.to_dev(x), batch, h, w, out)
        torch.cuda.synchronize()
        ref = orc.patches(x, kh, kw, stride, pad, has_bias=False)
        got = out.cpu().numpy()
        assert np.array_equal(got[:, :ref.shape[1]].astype(np.float64), ref)
        assert np.all(got[:, ref.shape[1]:] == 0)


def test_im2col_with_different_row_and_column_padding_bit_exact():
    for (cin, kh, kw, stride, ph, pw, h, w, batch) in [(8, 1, 7, 1, 0, 3, 17, 17, 2), (8, 7, 1, 1, 3, 0, 17, 17, 2),
                                                       (12, 1, 3, 1, 0, 1, 8, 8, 3), (12, 3, 1, 1, 1, 0, 8, 12, 3),
                                                       (6, 3, 5, 2, 0, 2, 21, 30, 2), (5, 3, 3, 1, 2, 0, 9, 11, 1),
                                                       (16, 3, 3, 1, 1, 2, 10, 10, 2), (4, 1, 1, 1, 0, 2, 6, 7, 2)]:
        print("im2col", cin, kh, kw, stride, ph, pw, h, w, batch, flush=True)
        x = rng.draw_relu_normal(79, 0, (batch, cin, h, w))
        desc = kf.LayerDesc.conv2d(cin, 4, kh, stride, ph, kw=kw, pad_w=pw)
        assert desc.pad + desc.pad_h == ph and desc.pad + desc.pad_w == pw
        ld = kf.kfac_patch_ld(desc)
        ho = (h + 2 * ph - kh) // stride + 1
        wo = (w + 2 * pw - kw) // stride + 1
        out = torch.full((batch * ho * wo, ld), float("nan"), device=gu.DEV)
        kf.kfac_im2col(desc, gu.to_dev(x), batch, h, w, out)
        torch.cuda.synchronize()
        ref = orc.patches(x, kh, kw, stride, ph, has_bias=False, pad_w=pw)
        got = out.cpu().numpy()
        assert np.array_equal(got[:, :ref.shape[1]].astype(np.float64), ref)
        assert np.all(got[:, ref.shape[1]:] == 0)


@pytest.mark.parametrize("cin,kh,kw,h,w,ph,pw,bias", [(24, 1, 7, 17, 17, 0, 3, True), (24, 7, 1, 9, 14, 3, 0, True),
                                                       (24, 1, 3, 8, 8, 0, 1, False), (32, 3, 1, 8, 12, 1, 0, True),
                                                       (16, 3, 3, 10, 12, 1, 0, True)])
def test_layer_with_different_row_and_column_padding_end_to_end(cin, kh, kw, h, w, ph, pw, bias):
    # "same"-padded 1 x 7 / 7 x 1 / 1 x 3 / 3 x 1 kernels through all three calls; the last is a 3 x 3 kernel padded
    # in one direction only, which must NOT take the kernels written for 3 x 3 / pad 1
    layer = LayerSpec("conv", cin, 20, kh, 1, ph, h, has_bias=bias, k_w=kw, w_in=w, pad_w=pw)
    _run_and_check([layer], 6, 9300 + 10 * kh + kw, batched=True)
    _run_and_check([layer], 6, 9400 + 10 * kh + kw, batched=False)


@pytest.mark.parametrize("cin,kh,kw,h,w,pad,bias", [(24, 1, 7, 17, 17, 0, True), (24, 7, 1, 9, 14, 0, True),
                                                    (24, 3, 1, 8, 12, 1, False), (32, 3, 3, 10, 16, 1, True),
                                                    (16, 3, 3, 12, 8, 1, True)])
def test_nonsquare_layer_end_to_end(cin, kh, kw, h, w, pad, bias):
    # kernel height != width and map height != width through all three calls (3 x 3 with a multiple of
    # 16 channels takes the fused convolution kernel, here on non-square maps)
    layer = LayerSpec("conv", cin, 20, kh, 1, pad, h, has_bias=bias, k_w=kw, w_in=w)
    _run_and_check([layer], 6, 9100 + 10 * kh + kw, batched=True)
    _run_and_check([layer], 6, 9200 + 10 * kh + kw, batched=False)


@pytest.mark.parametrize("cin,h,w,batch,bias", [
    (16, 32, 32, 3, True),      # one strip pair per image, four wavefronts splitting the pixel groups
    (16, 8, 8, 7, False),       # batch not a multiple of the image chunks of the border kernel
    (32, 16, 16, 2, True),
    (32, 6, 8, 1, True),        # a single image; strips of 2 rows
    (64, 8, 8, 7, True),        # two workgroups per range of units
    (64, 4, 12, 3, False),
    (16, 2, 16, 4, True),       # two rows: the first and the last image row are neighbours
    (16, 12, 8, 9, True),
    (32, 64, 4, 2, True),       # tall and narrow
    (16, 3, 64, 2, True),       # odd height, widest map
    (32, 2, 8, 3, True),        # small map, two rows: border terms from whole images
    (64, 3, 16, 6, True),       # small map, odd height
])
def test_conv3_factor_from_autocorrelations(cin, h, w, batch, bias):
    # 3x3 / stride 1 / pad 1 layers with 16, 32 or 64 input channels build A from 13 autocorrelation lag
    # matrices plus border corrections: against the oracle, and against the direct kernel on the same inputs
    layer = LayerSpec("conv", cin, 8, 3, 1, 1, h, has_bias=bias, w_in=w)
    _run_and_check([layer], batch, 7300 + cin + h + w, batched=True)
    inputs = gu.draw_inputs([layer], batch, 7400 + cin, "relu_normal", 0.05)
    scales = gu.scales_for([layer], batch)
    corr = gu.run_layers_gpu([layer], batch, inputs, scales, 0.95, 0.03)[0]
    kf.kfac_tune("use_corr3", 0)
    try:
        direct = gu.run_layers_gpu([layer], batch, inputs, scales, 0.95, 0.03)[0]
    finally:
        kf.kfac_tune("use_corr3", 1)
    assert gu.rel_fro(corr["A"], direct["A"]) < 1e-5
    assert np.array_equal(corr["A"], corr["A"].T)


@pytest.mark.parametrize("cin,h,w,batch", [(48, 64, 4, 2), (48, 32, 4, 3), (48, 64, 8, 2), (80, 16, 4, 2), (48, 8, 4, 2),
                                            (48, 20, 12, 2)])
def test_fused_conv3_kernel_on_tall_narrow_maps(cin, h, w, batch):
    # the direct fused kernel (channel counts the autocorrelation path does not take) on maps much taller than
    # wide: the strip height is bounded by what the bias-border summation of a workgroup covers (256 slab rows)
    layer = LayerSpec("conv", cin, 8, 3, 1, 1, h, has_bias=True, w_in=w)
    _run_and_check([layer], batch, 7500 + cin + h + w, batched=True)


@pytest.mark.parametrize("n", [1, 5, 64, 65, 130, 257, 400])
def test_inverse_sizes(n):
    gen = np.random.default_rng(n)
    X = gen.standard_normal((2 * n + 3, n))
    M = (X.T @ X / (2 * n + 3)).astype(np.float32)
    lam = 0.03
    desc = kf.LayerDesc.linear(n, 3, has_bias=False)
    G = np.eye(3, dtype=np.float32)
    A_inv = torch.full((n, n), float("nan"), device=gu.DEV)
    G_inv = torch.full((3, 3), float("nan"), device=gu.DEV)
    info = torch.full((2,), -1, dtype=torch.int32, device=gu.DEV)
    ws = gu.workspace(kf.kfac_workspace_bytes(desc, 8))
    kf.kfac_invert(desc, gu.to_dev(M), gu.to_dev(G), lam, lam, A_inv, G_inv, info, ws)
    torch.cuda.synchronize()
    ref = orc.inverse(M.astype(np.float64), lam)
    got = A_inv.cpu().numpy()
    assert list(info.cpu().numpy()) == [0, 0]
    assert gu.rel_fro(got, ref) < 1e-4
    assert np.array_equal(got, got.T)
    assert np.allclose(G_inv.cpu().numpy(), np.eye(3) / (1 + lam), rtol=1e-6)


@pytest.mark.parametrize("n", [130, 288, 289, 400, 577, 700, 1000])
def test_inverse_two_level_blocked_path(n):
    # orders above the knob take the two-level blocked sweep (256-row outer blocks, nested pivot inversions, panel
    # products, rank-256 updates); lowering the knob exercises it at sizes the oracle inverts in a moment
    gen = np.random.default_rng(100 + n)
    X = gen.standard_normal((n + 7, n))
    M = (X.T @ X / (n + 7)).astype(np.float32)
    lam = 0.05
    desc = kf.LayerDesc.linear(n, 70, has_bias=False)
    H = gen.standard_normal((90, 70))
    G = (H.T @ H / 90).astype(np.float32)
    A_inv = torch.full((n, n), float("nan"), device=gu.DEV)
    G_inv = torch.full((70, 70), float("nan"), device=gu.DEV)
    info = torch.full((2,), -1, dtype=torch.int32, device=gu.DEV)
    kf.kfac_tune("invert_fused_max_n", 100)
    try:
        ws = gu.workspace(kf.kfac_workspace_bytes(desc, 8))
        kf.kfac_invert(desc, gu.to_dev(M), gu.to_dev(G), lam, lam, A_inv, G_inv, info, ws)
        torch.cuda.synchronize()
    finally:
        kf.kfac_tune("invert_fused_max_n", 1280)
    assert list(info.cpu().numpy()) == [0, 0]
    got = A_inv.cpu().numpy()
    assert gu.rel_fro(got, orc.inverse(M.astype(np.float64), lam)) < 1e-4
    assert np.array_equal(got, got.T)
    assert gu.rel_fro(G_inv.cpu().numpy(), orc.inverse(G.astype(np.float64), lam)) < 1e-4


def test_inverse_on_the_library_streams_is_reproducible_and_agrees_with_the_one_stream_run():
    """The blocked sweep spreads a call over the caller's stream and three of its own (nested inversions, the rest of
    each step's chain, the smaller factors), ordered by events.  A missing dependency between the streams would
    make the result depend on timing: the call is repeated and must return the same bits every time.  The one-stream
    schedule applies the same updates through differently shaped products (no separate band products), so it
    agrees to rounding, not to the bit.  Mixed batch: orders on both paths, a last block of one row, a bordered
    order, an ill-conditioned factor whose refinement gates open."""
    gen = np.random.default_rng(11)
    orders = [1301, 2049, 1536, 700, 577, 1793, 64, 2304]
    mats = []
    for k, n in enumerate(orders):
        X = np.maximum(gen.standard_normal((n // 2 + 9, n)), 0.0) if k % 2 == 0 else gen.standard_normal((n + 9, n))
        M = (X.T @ X / X.shape[0]).astype(np.float32)
        if k == 1:
            M *= np.float32(40.0)           # condition number of a few 1e4 with the damping below
        mats.append(gu.to_dev(M))
    descs = [kf.LayerDesc.linear(n, 8, has_bias=False) for n in orders]
    G = [torch.eye(8, device=gu.DEV) for _ in orders]
    ws = gu.workspace(kf.kfac_workspace_bytes_batched(descs, [8] * len(orders), [1] * len(orders), [1] * len(orders)))

    def run():
        A_inv = [torch.full((n, n), float("nan"), device=gu.DEV) for n in orders]
        G_inv = [torch.empty((8, 8), device=gu.DEV) for _ in orders]
        info = torch.full((2 * len(orders),), -1, dtype=torch.int32, device=gu.DEV)
        kf.kfac_invert_batched(descs, mats, G, 0.02, 0.02, A_inv, G_inv, info, ws)
        torch.cuda.synchronize()
        flags = info.cpu().numpy()
        assert not flags.any(), f"flagged: {flags.reshape(-1, 2)[:, 0].tolist()} for orders {orders}"
        return A_inv

    kf.kfac_tune("invert_two_streams", 0)
    try:
        serial = run()
    finally:
        kf.kfac_tune("invert_two_streams", 1)
    first = run()
    for rep in range(6):
        again = run()
        for n, a, b in zip(orders, first, again):
            assert torch.equal(a, b), f"order {n}, repetition {rep}: the result depends on the run"
    for n, a, b in zip(orders, serial, first):
        diff = float(torch.linalg.norm(a.double() - b.double()) / torch.linalg.norm(a.double()))
        # (each is within rounding x condition number of the exact inverse: 3.6e-5 apart on the ill-conditioned one)
        assert diff < 1e-4, f"order {n}: pipelined and one-stream runs differ by {diff:.2e}"
    # and the one-stream result is right
    for n, M, X in zip(orders[:3], mats[:3], serial[:3]):
        Md = M.double() + 0.02 * torch.eye(n, device=gu.DEV, dtype=torch.float64)
        res = float(torch.linalg.norm(Md @ X.double() - torch.eye(n, device=gu.DEV, dtype=torch.float64))) / n ** 0.5
        assert res < 1e-3, (n, res)


def test_not_positive_definite_in_a_late_block_is_flagged_by_the_blocked_path():
    n = 700
    gen = np.random.default_rng(5)
    X = gen.standard_normal((n + 9, n))
    M = (X.T @ X / (n + 9)).astype(np.float32)
    M[650, 650] = -5.0          # makes a pivot in the third outer block negative
    desc = kf.LayerDesc.linear(n, 3, has_bias=False)
    A_inv = torch.empty((n, n), device=gu.DEV)
    G_inv = torch.empty((3, 3), device=gu.DEV)
    info = torch.full((2,), -1, dtype=torch.int32, device=gu.DEV)
    kf.kfac_tune("invert_fused_max_n", 100)
    try:
        ws = gu.workspace(kf.kfac_workspace_bytes(desc, 8))
        kf.kfac_invert(desc, gu.to_dev(M), gu.to_dev(np.eye(3, dtype=np.float32)), 0.01, 0.01, A_inv, G_inv, info, ws)
        torch.cuda.synchronize()
    finally:
        kf.kfac_tune("invert_fused_max_n", 1280)
    flags = info.cpu().numpy()
    assert flags[1] == 0
    # the pivots of the sweep are those of the LDL^T factorisation: the oracle names the first bad one
    assert flags[0] == orc.inverse_info(M.astype(np.float64), 0.01)


@pytest.mark.parametrize("n", [65, 129, 577, 1153])
def test_inverse_of_order_64k_plus_1_by_bordering(n):
    # orders 64 k + 1 (a bias column after a multiple of 64 columns): the sweep inverts the leading block, the
    # last row and column follow by bordering; same result as the plain sweep (knob off) and as the oracle
    gen = np.random.default_rng(300 + n)
    X = gen.standard_normal((n + 11, n))
    M = (X.T @ X / (n + 11)).astype(np.float32)
    lam = 0.04
    desc = kf.LayerDesc.linear(n - 1, 3, has_bias=True)
    G = np.eye(3, dtype=np.float32)
    ws = gu.workspace(kf.kfac_workspace_bytes(desc, 8))
    got = {}
    for border in (1, 0):
        A_inv = torch.full((n, n), float("nan"), device=gu.DEV)
        G_inv = torch.full((3, 3), float("nan"), device=gu.DEV)
        info = torch.full((2,), -1, dtype=torch.int32, device=gu.DEV)
        kf.kfac_tune("invert_border", border)
        try:
            kf.kfac_invert(desc, gu.to_dev(M), gu.to_dev(G), lam, lam, A_inv, G_inv, info, ws)
            torch.cuda.synchronize()
        finally:
            kf.kfac_tune("invert_border", 1)
        assert list(info.cpu().numpy()) == [0, 0]
        got[border] = A_inv.cpu().numpy()
    ref = orc.inverse(M.astype(np.float64), lam)
    assert gu.rel_fro(got[1], ref) < 1e-4
    assert gu.rel_fro(got[0], ref) < 1e-4
    assert gu.rel_fro(got[1], got[0]) < 2e-5
    assert np.array_equal(got[1], got[1].T)


def test_bordered_pivot_not_positive_is_flagged():
    # leading block positive definite, the Schur complement of the last row is not: pivot n
    n = 129
    M = np.eye(n, dtype=np.float32)
    M[n - 1, :n - 1] = 0.2
    M[:n - 1, n - 1] = 0.2
    M[n - 1, n - 1] = 1.0          # 1 + 0.5 - 128 * 0.04 / 1.5 < 0
    desc = kf.LayerDesc.linear(n - 1, 2, has_bias=True)
    A_inv = torch.zeros((n, n), device=gu.DEV)
    G_inv = torch.zeros((2, 2), device=gu.DEV)
    info = torch.full((2,), -1, dtype=torch.int32, device=gu.DEV)
    ws = gu.workspace(kf.kfac_workspace_bytes(desc, 8))
    kf.kfac_invert(desc, gu.to_dev(M), gu.to_dev(np.eye(2, dtype=np.float32)), 0.5, 0.5, A_inv, G_inv, info, ws)
    torch.cuda.synchronize()
    assert list(info.cpu().numpy()) == [n, 0]
    assert orc.inverse_info(M.astype(np.float64), 0.5) == n


@pytest.mark.parametrize("dA,dG", [(1, 1), (7, 3), (65, 10), (145, 16), (130, 17), (289, 32), (300, 33), (577, 64),
                                   (64, 64), (1153, 48)])
def test_two_sided_product_shapes(dA, dG):
    # P = G_inv grad A_inv called directly on given (symmetric positive definite) inverses, against fp64:
    # orders around the tile sizes of the small-product GEMM and the widths of config 2
    gen = np.random.default_rng(17 * dA + dG)
    def spd(n):
        X = gen.standard_normal((n + 5, n))
        return (X.T @ X / (n + 5) + 0.1 * np.eye(n)).astype(np.float32)
    A_inv, G_inv = spd(dA), spd(dG)
    grad = gen.standard_normal((dG, dA)).astype(np.float32)
    desc = kf.LayerDesc.linear(dA, dG, has_bias=False)
    ws = gu.workspace(kf.kfac_workspace_bytes(desc, 8))
    out = torch.full((dG, dA), float("nan"), device=gu.DEV)
    kf.kfac_precondition(desc, gu.to_dev(A_inv), gu.to_dev(G_inv), gu.to_dev(grad), out, ws)
    torch.cuda.synchronize()
    ref = G_inv.astype(np.float64) @ grad.astype(np.float64) @ A_inv.astype(np.float64)
    assert gu.rel_fro(out.cpu().numpy(), ref) < 1e-5


@pytest.mark.parametrize("dA,dG", [(2401, 256), (3000, 2100)])
def test_two_sided_product_with_k_slices(dA, dG):
    # a call of few tiles with deep products: they are cut into K slices (partials in the workspace, summed in
    # slice order), ragged last slice included; with room for the intermediate only, or with the slices
    # switched off, every product is computed in one piece -- the same result to rounding
    gen = np.random.default_rng(31 * dA + dG)
    A_inv = gen.standard_normal((dA, dA)).astype(np.float32)
    A_inv = ((A_inv + A_inv.T) / 2).astype(np.float32)
    G_inv = gen.standard_normal((dG, dG)).astype(np.float32)
    G_inv = ((G_inv + G_inv.T) / 2).astype(np.float32)
    grad = gen.standard_normal((dG, dA)).astype(np.float32)
    desc = kf.LayerDesc.linear(dA, dG, has_bias=False)
    full = kf.kfac_workspace_bytes(desc, 8)
    least = (dA * dG * 4 + 255) // 256 * 256
    assert full >= least + dA * dG * 4, "no room for K-slice partials was planned"
    dev = [gu.to_dev(x) for x in (A_inv, G_inv, grad)]
    ref = G_inv.astype(np.float64) @ grad.astype(np.float64) @ A_inv.astype(np.float64)

    def run(nbytes):
        out = torch.full((dG, dA), float("nan"), device=gu.DEV)
        kf.kfac_precondition(desc, dev[0], dev[1], dev[2], out, gu.workspace(nbytes))
        torch.cuda.synchronize()
        return out.cpu().numpy()
    sliced, again, one_piece = run(full), run(full), run(least)
    kf.kfac_tune("gemm_kslice_stages", 0)
    try:
        off = run(full)
    finally:
        kf.kfac_tune("gemm_kslice_stages", 75)
    assert gu.rel_fro(sliced, ref) < 1e-5
    assert gu.rel_fro(one_piece, ref) < 1e-5
    assert np.array_equal(sliced, again), "the sliced product is not reproducible"
    assert np.array_equal(one_piece, off)
    assert not np.array_equal(sliced, one_piece), "the slices were not used"
    assert gu.rel_fro(sliced, one_piece.astype(np.float64)) < 2e-6


def test_two_sided_products_batched_with_some_layers_sliced():
    # one batched call in which two layers have a deep second product (K slices, one with the bias column, i.e.
    # an odd pitch) and two do not; every layer against the fp64 product
    dims = [(2400, 256, True), (300, 150, False), (2305, 200, False), (65, 10, True)]
    gen = np.random.default_rng(977)
    descs, dev, refs, outs = [], [], [], []
    for d_in, d_out, bias in dims:
        desc = kf.LayerDesc.linear(d_in, d_out, has_bias=bias)
        dA, dG = kf.kfac_dim_A(desc), kf.kfac_dim_G(desc)
        A_inv = gen.standard_normal((dA, dA)).astype(np.float32)
        A_inv = ((A_inv + A_inv.T) / 2).astype(np.float32)
        G_inv = gen.standard_normal((dG, dG)).astype(np.float32)
        G_inv = ((G_inv + G_inv.T) / 2).astype(np.float32)
        grad = gen.standard_normal((dG, dA)).astype(np.float32)
        descs.append(desc)
        dev.append([gu.to_dev(x) for x in (A_inv, G_inv, grad)])
        refs.append(G_inv.astype(np.float64) @ grad.astype(np.float64) @ A_inv.astype(np.float64))
        outs.append(torch.full((dG, dA), float("nan"), device=gu.DEV))
    n = len(dims)
    ws = gu.workspace(kf.kfac_workspace_bytes_batched(descs, [8] * n, [1] * n, [1] * n))
    kf.kfac_precondition_batched(descs, [d[0] for d in dev], [d[1] for d in dev], [d[2] for d in dev], outs, ws)
    torch.cuda.synchronize()
    for i in range(n):
        assert gu.rel_fro(outs[i].cpu().numpy(), refs[i]) < 1e-5, dims[i]


def test_not_positive_definite_is_flagged():
    n = 70
    M = np.eye(n, dtype=np.float32)
    M[66, 66] = -2.0
    desc = kf.LayerDesc.linear(n, 2, has_bias=False)
    A_inv = torch.zeros((n, n), device=gu.DEV)
    G_inv = torch.zeros((2, 2), device=gu.DEV)
    info = torch.full((2,), -1, dtype=torch.int32, device=gu.DEV)
    ws = gu.workspace(kf.kfac_workspace_bytes(desc, 8))
    kf.kfac_invert(desc, gu.to_dev(M), gu.to_dev(np.eye(2, dtype=np.float32)), 0.5, 0.5, A_inv, G_inv, info, ws)
    torch.cuda.synchronize()
    assert list(info.cpu().numpy()) == [67, 0]
    assert orc.inverse_info(M.astype(np.float64), 0.5) == 67


def test_batched_mixed_layers_match_oracle_and_single_calls():
    layers = [LayerSpec("conv", 4, 6, 3, 1, 1, 8), LayerSpec("linear", 70, 20, rows=40),
              LayerSpec("conv", 8, 8, 1, 1, 0, 4), LayerSpec("conv", 16, 16, 3, 1, 1, 8),
              LayerSpec("linear", 10, 3, rows=40, has_bias=False)]
    batch = 5
    inputs = gu.draw_inputs(layers, batch, 4000, "relu_normal", 0.05)
    scales = gu.scales_for(layers, batch)
    g1 = gu.run_layers_gpu(layers, batch, inputs, scales, 0.9, 0.01, batched=True)
    g2 = gu.run_layers_gpu(layers, batch, inputs, scales, 0.9, 0.01, batched=False)
    for i, l in enumerate(layers):
        ref = gu.run_layer_oracle(l, inputs[i], scales[i], 0.9, 0.01)
        gu.check_layer(g1[i], ref, tag=f"batched {i}")
        gu.check_layer(g2[i], ref, tag=f"single {i}")
    # the same batched calls on C arrays built beforehand: the same launches, the same bits
    g3 = gu.run_layers_gpu(layers, batch, inputs, scales, 0.9, 0.01, batched=True, marshalled=True)
    for i in range(len(layers)):
        for k in ("A", "G", "A_inv", "G_inv", "P"):
            assert np.array_equal(g1[i][k], g3[i][k]), (i, k)


def test_running_average_ends_and_repeat_is_bitwise_reproducible():
    layer = LayerSpec("conv", 6, 5, 3, 1, 1, 10)
    batch = 4
    inp = gu.draw_inputs([layer], batch, 5000, "relu_normal", 0.1)
    sc = gu.scales_for([layer], batch)
    gen = np.random.default_rng(0)
    A0 = (lambda m: m @ m.T)(gen.standard_normal((layer.d_A, layer.d_A)))
    G0 = (lambda m: m @ m.T)(gen.standard_normal((layer.d_G, layer.d_G)))
    A0f, G0f = A0.astype(np.float32).astype(np.float64), G0.astype(np.float32).astype(np.float64)
    r1 = gu.run_layers_gpu([layer], batch, inp, sc, 1.0, 0.5, A0=[A0f], G0=[G0f])[0]
    assert np.array_equal(r1["A"], A0f.astype(np.float32)) and np.array_equal(r1["G"], G0f.astype(np.float32))
    r0 = gu.run_layers_gpu([layer], batch, inp, sc, 0.0, 0.5, A0=[A0f], G0=[G0f])[0]
    ref = gu.run_layer_oracle(layer, inp[0], sc[0], 0.0, 0.5, A0f, G0f)
    gu.check_layer(r0, ref, tag="decay 0")
    ra = gu.run_layers_gpu([layer], batch, inp, sc, 0.95, 0.03)[0]
    rb = gu.run_layers_gpu([layer], batch, inp, sc, 0.95, 0.03)[0]
    for k in ("A", "G", "A_inv", "G_inv", "P"):
        assert np.array_equal(ra[k], rb[k]), k


def test_bf16_inputs_match_oracle_on_the_same_bits():
    layers = [LayerSpec("linear", 96, 48, rows=200), LayerSpec("conv", 8, 8, 3, 1, 1, 8),
              LayerSpec("conv", 16, 8, 1, 1, 0, 4)]
    batch = 4
    inputs = gu.draw_inputs(layers, batch, 6000, "relu_normal", 0.05, dtype="bf16")
    scales = gu.scales_for(layers, batch)
    gpu = gu.run_layers_gpu(layers, batch, inputs, scales, 0.95, 0.03, dtype="bf16")
    for i, l in enumerate(layers):
        ref = gu.run_layer_oracle(l, inputs[i], scales[i], 0.95, 0.03)
        gu.check_layer(gpu[i], ref, tag=f"bf16 {i}")
    # against the unrounded fp32 draws the allowance is 2e-2 on the preconditioned gradient
    raw = gu.draw_inputs(layers, batch, 6000, "relu_normal", 0.05, dtype="f32")
    for i, l in enumerate(layers):
        ref = gu.run_layer_oracle(l, raw[i], scales[i], 0.95, 0.03)
        assert gu.rel_fro(gpu[i]["P"], ref["P"]) < 2e-2


@pytest.mark.parametrize("layer,batch", [
    (LayerSpec("linear", 256, 24, rows=300), 300),                 # one block tile, ragged last K stage, bias border
    (LayerSpec("linear", 520, 16, rows=77), 77),                   # three block rows, last one 8 columns wide
    (LayerSpec("linear", 104, 8, rows=40, has_bias=False), 40),    # narrower than one tile, no bias
    (LayerSpec("linear", 768, 320, rows=1500), 1500),              # A and G both on the bf16 units, several K splits
    (LayerSpec("conv", 32, 8, 3, 1, 1, 10), 3),                    # bf16 patch matrix (d = 288)
    (LayerSpec("conv", 12, 8, 3, 2, 1, 9), 5),                     # d = 108: pitch padded to 112 with zero columns
    (LayerSpec("conv", 128, 96, 1, 1, 0, 6), 3),                   # 1x1: A and G read from NCHW, HW = 36 (4-position tail)
    (LayerSpec("conv", 264, 100, 1, 1, 0, 8), 5),                  # two block columns, HW = 64 (no tail), d_G not a multiple of 8
    (LayerSpec("conv", 8, 300, 3, 1, 1, 14), 2),                   # G of a 3x3 conv, HW = 196, two block rows
    (LayerSpec("conv", 96, 96, 1, 1, 0, 5), 4),                    # HW = 25 is odd: both operands through a row-major copy
    (LayerSpec("conv", 200, 136, 1, 1, 0, 7), 6),                  # 7 x 7 maps, widths that are no multiple of 8 or 16
    (LayerSpec("conv", 16, 128, 3, 1, 1, 7), 5),                   # 3 x 3 on 7 x 7: only G takes the copy (A has its patch matrix)
    (LayerSpec("conv", 128, 40, 1, 1, 0, 3, w_in=5), 4),           # 3 x 5 map; G (40 wide) stays on the widening kernel
])
def test_bf16_mfma_factor_kernel(layer, batch):
    # row-major bf16 operands take the bf16 MFMA kernel; same bits into the oracle
    inputs = gu.draw_inputs([layer], batch, 6500 + layer.d_A, "relu_normal", 0.05, dtype="bf16")
    scales = gu.scales_for([layer], batch)
    fast = gu.run_layers_gpu([layer], batch, inputs, scales, 0.95, 0.03, dtype="bf16")[0]
    ref = gu.run_layer_oracle(layer, inputs[0], scales[0], 0.95, 0.03)
    gu.check_layer(fast, ref, tag=str(layer))
    # and the same factors as the kernel that widens bf16 to fp32 on load
    kf.kfac_tune("use_bf16_mfma", 0)
    try:
        wide = gu.run_layers_gpu([layer], batch, inputs, scales, 0.95, 0.03, dtype="bf16")[0]
    finally:
        kf.kfac_tune("use_bf16_mfma", 1)
    assert gu.rel_fro(fast["A"], wide["A"]) < 1e-5
    assert gu.rel_fro(fast["G"], wide["G"]) < 1e-5
    if layer.kind == "conv" and (layer.h_out * layer.w_out) % 2 == 1:
        # maps with an odd number of positions: with the row-major copy off, the NCHW operands go to the widening
        # kernel directly; same factors either way
        kf.kfac_tune("bf16_rows_copy", 0)
        try:
            direct = gu.run_layers_gpu([layer], batch, inputs, scales, 0.95, 0.03, dtype="bf16")[0]
        finally:
            kf.kfac_tune("bf16_rows_copy", 1)
        assert gu.rel_fro(fast["A"], direct["A"]) < 1e-5
        assert gu.rel_fro(fast["G"], direct["G"]) < 1e-5


def test_pi_damped_inverse_matches_oracle():
    # Eq. 12 split of the damping, computed on the device from the traces of the running factors
    layers = [LayerSpec("linear", 64, 32, rows=32), LayerSpec("conv", 16, 24, 3, 1, 1, 8),
              LayerSpec("linear", 300, 130, rows=100), LayerSpec("conv", 4, 6, 3, 1, 1, 8)]
    batch = 4
    gamma = 0.003
    inputs = gu.draw_inputs(layers, batch, 8100, "relu_normal", 0.0316)
    scales = gu.scales_for(layers, batch)
    descs = [kf.LayerDesc.from_spec(l, kf.KFAC_F32) for l in layers]
    b, h, w = gu.batch_args(layers, batch)
    n = len(layers)
    A_run = [torch.eye(l.d_A, device=gu.DEV) for l in layers]
    G_run = [torch.eye(l.d_G, device=gu.DEV) for l in layers]
    A_inv = [torch.full((l.d_A, l.d_A), float("nan"), device=gu.DEV) for l in layers]
    G_inv = [torch.full((l.d_G, l.d_G), float("nan"), device=gu.DEV) for l in layers]
    info = torch.full((2 * n,), -1, dtype=torch.int32, device=gu.DEV)
    lam = torch.full((2 * n,), float("nan"), device=gu.DEV)
    ws = gu.workspace(kf.kfac_workspace_bytes_batched(descs, b, h, w))
    kf.kfac_update_factors_batched(descs, [gu.to_dev(i[0]) for i in inputs], [gu.to_dev(i[1]) for i in inputs],
                                   b, h, w, [s[0] for s in scales], [s[1] for s in scales], 0.95, A_run, G_run, ws)
    kf.kfac_invert_pi_batched(descs, A_run, G_run, gamma, A_inv, G_inv, info, lam, ws)
    torch.cuda.synchronize()
    assert not info.cpu().numpy().any()
    lam_h = lam.cpu().numpy().astype(np.float64)
    for i, l in enumerate(layers):
        A = A_run[i].cpu().numpy().astype(np.float64)
        G = G_run[i].cpu().numpy().astype(np.float64)
        Ai, Gi, lA, lG = orc.invert_layer_pi(A, G, gamma)
        assert abs(lam_h[2 * i] - lA) < 1e-5 * lA and abs(lam_h[2 * i + 1] - lG) < 1e-5 * lG
        assert gu.rel_fro(A_inv[i].cpu().numpy(), Ai) < 1e-4
        assert gu.rel_fro(G_inv[i].cpu().numpy(), Gi) < 1e-4
    # single-layer call without the damping output, on the path for large orders
    kf.kfac_tune("invert_fused_max_n", 100)
    try:
        ws1 = gu.workspace(kf.kfac_workspace_bytes(descs[2], b[2]))
        A1 = torch.empty_like(A_inv[2]); G1 = torch.empty_like(G_inv[2])
        kf.kfac_invert_pi(descs[2], A_run[2], G_run[2], gamma, A1, G1, info[:2], None, ws1)
        torch.cuda.synchronize()
    finally:
        kf.kfac_tune("invert_fused_max_n", 1280)
    assert gu.rel_fro(A1.cpu().numpy(), A_inv[2].cpu().numpy()) < 1e-5
    assert gu.rel_fro(G1.cpu().numpy(), G_inv[2].cpu().numpy()) < 1e-5


@pytest.mark.parametrize("d_in,rows,steps,lam", [(576, 24, 12, 1e-3), (1152, 32, 20, 1e-3), (2048, 32, 30, 1e-2),
                                                 (2048, 32, 30, 1e-3)])
def test_inverse_of_ill_conditioned_rank_deficient_running_average(d_in, rows, steps, lam):
    """The factor K-FAC meets late in training: the identity it started from has decayed away (decay 0.5 for
    `steps` updates here), what is left is a running average of a few low-rank batches of post-ReLU rows (rank < d,
    one dominant eigenvalue along the mean), and only the damping keeps it invertible: condition numbers of 3e4
    to 3e5, against at most 3e4 in the benchmark configurations.  Any fp32 elimination loses accuracy in proportion
    to the condition number; LAPACK's fp32 Cholesky inverse of the same matrix is printed beside the library's
    result as the yardstick.  The library stays within a factor two of it: 4.5e-4 against 2.7e-4 at order 577 and
    condition number 7.5e4, 8.5e-4 against 6.6e-4 at order 1153 and 1.9e5, 1.9e-4 against 1.5e-4 at order 2049 and
    3.3e4, 2.8e-3 against 1.5e-3 at 3.3e5.  Three measures get it there, each gated on the device by the condition
    number of the pivot block at hand so that well-conditioned factors do not pay: one step of iterative refinement
    of every panel product W = V P in the one-launch-per-step sweep (64 x 64 pivot blocks) and in the two-level sweep
    (256 x 256), and a second-order correction of the pivot of the bordering step of orders 64 k + 1.  Without
    them the errors were 1.1e-2, 2.7e-3, 7.7e-3 and a breakdown (a non-positive pivot on a positive definite
    matrix).  This test pins that: the error against the oracle's inverse of the very same running factor stays
    within 0.5 x cond x eps (and within the 1e-4 of the well-conditioned tests wherever that is larger), the result
    is bitwise symmetric, and a breakdown (a pivot that turns non-positive on
    a matrix that is positive definite) would have to be REPORTED through d_info."""
    decay = 0.5
    l = LayerSpec("linear", d_in, 8, rows=rows)
    desc = kf.LayerDesc.from_spec(l)
    dA = l.d_A
    A_run = torch.eye(dA, device=gu.DEV)
    G_run = torch.eye(8, device=gu.DEV)
    ws = gu.workspace(kf.kfac_workspace_bytes(desc, rows))
    for t in range(steps):
        act = rng.draw_relu_normal(4200 + t, 0, (rows, d_in))
        gout = rng.draw_normal(4200 + t, 1, (rows, 8), std=0.1)
        kf.kfac_update_factors(desc, gu.to_dev(act), gu.to_dev(gout), rows, 1, 1, 1.0 / rows, 1.0 / rows, decay,
                               A_run, G_run, ws)
    A_inv = torch.full((dA, dA), float("nan"), device=gu.DEV)
    G_inv = torch.full((8, 8), float("nan"), device=gu.DEV)
    info = torch.full((2,), -1, dtype=torch.int32, device=gu.DEV)
    kf.kfac_invert(desc, A_run, G_run, lam, lam, A_inv, G_inv, info, ws)
    torch.cuda.synchronize()
    flags = info.cpu().tolist()
    M = A_run.cpu().numpy().astype(np.float64)
    ev = np.linalg.eigvalsh(M + lam * np.eye(dA))
    cond = ev[-1] / ev[0]
    eps = 2.0 ** -24
    assert cond > 1e4 and ev[0] > 0.0 and flags[1] == 0
    if flags[0] != 0:
        # the sweep met a non-positive pivot on a matrix that IS positive definite: fp32 has run out
        print(f"order {dA}: cond {cond:.2e}, cond*eps {cond * eps:.2e}: breakdown reported at pivot {flags[0]}", flush=True)
        assert cond * eps > 1e-2 and 1 <= flags[0] <= dA
        return
    X = A_inv.cpu().numpy().astype(np.float64)
    ref = orc.inverse(M, lam)
    err = gu.rel_fro(X, ref)
    resid = np.linalg.norm((M + lam * np.eye(dA)) @ X - np.eye(dA)) / np.sqrt(dA)
    # for scale: what LAPACK's fp32 Cholesky inverse (spotrf + spotri through torch on the CPU) achieves on the same
    # matrix (printed, not asserted).  numpy.linalg.inv is no such yardstick: it computes float32 input in double.
    M32 = torch.from_numpy((M + lam * np.eye(dA)).astype(np.float32))
    Xl = torch.cholesky_inverse(torch.linalg.cholesky(M32)).numpy().astype(np.float64)
    err_l = gu.rel_fro(Xl, ref)
    print(f"order {dA}: rank <= {rows * steps}, cond {cond:.2e}, cond*eps {cond * eps:.2e}, "
          f"rel. error {err:.2e} (fp32 LAPACK: {err_l:.2e}), residual/sqrt(n) {resid:.2e}", flush=True)
    assert np.array_equal(A_inv.cpu().numpy(), A_inv.cpu().numpy().T)
    assert err < max(1e-4, 0.5 * cond * eps)
    assert resid < max(1e-4, 2.0 * cond * eps)
    # the gated refinements are what gets it there: switched off, the same call is several times less accurate
    # (or breaks down), which also shows that the gates open on such a factor
    kf.kfac_tune("invert_refine", 0)
    try:
        kf.kfac_invert(desc, A_run, G_run, lam, lam, A_inv, G_inv, info, ws)
        torch.cuda.synchronize()
    finally:
        kf.kfac_tune("invert_refine", 1)
    if info.cpu().tolist()[0] == 0:
        err_off = gu.rel_fro(A_inv.cpu().numpy().astype(np.float64), ref)
        print(f"          without the refinements: rel. error {err_off:.2e}", flush=True)
        assert err_off > 2.0 * err

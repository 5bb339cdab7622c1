"""Shape tables and the seeded generator (no K-FAC arithmetic here)."""
import os

import numpy as np

from workloads import shapes, rng

GOLD = os.path.join(os.path.dirname(__file__), "golden", "resnet50_sizes.txt")


def _gold():
    out = {}
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split()
        out[k] = float(v)
    return out


def test_resnet50_sizes_match_paper_section_3_2():
    # N_f = sum d_{i-1}^2 + d_i^2 and N_g = sum d_i d_{i-1} (section 3); the
    # paper counts all parameters (incl. the 53 batch-norm layers) in N_g.
    gold = _gold()
    layers = shapes.config_layers("resnet50_imagenet")
    assert len(layers) == 54
    nf, ng = shapes.factor_counts(layers)
    assert abs(nf / 1e6 - gold["N_f_millions"]) < 0.1
    assert abs(ng / 1e6 - gold["N_g_millions"]) < 0.1
    assert nf / ng >= 2.0          # N_f / N_g >= 2 (section 3)


def test_layer_counts_and_dims():
    l2 = shapes.config_layers("resnet110_cifar")
    assert len(l2) == 110
    assert sorted({l.d_A for l in l2}) == [28, 65, 145, 289, 577]
    assert sorted({l.d_G for l in l2}) == [10, 16, 32, 64]
    assert {l.n_rows(128) for l in l2 if l.kind == "conv"} == {131072, 32768, 8192}
    l3 = shapes.config_layers("resnet50_imagenet")
    assert max(l.d_A for l in l3) == 4609 and max(l.d_G for l in l3) == 2048
    assert sum(1 for l in l3 if l.kind == "conv" and l.k > 1) == 17
    l5 = shapes.config_layers("transformer_encoder_bf16")
    assert len(l5) == 144 and {l.d_A for l in l5} == {1025, 4097}
    l1 = shapes.config_layers("fc_tiny")
    assert (l1[0].d_A, l1[0].d_G, l1[0].rows) == (65, 32, 32)


def test_further_layer_sets():
    v = shapes.config_layers("vgg16_cifar")
    assert len(v) == 16 and sum(1 for l in v if l.kind == "conv") == 13
    assert max(l.d_A for l in v) == 4609 and {l.h_in for l in v if l.kind == "conv"} == {32, 16, 8, 4, 2}
    inc = shapes.config_layers("inception_nonsquare")
    assert all(l.k != l.kw for l in inc)
    l = inc[2]                                             # 1x7 kernel on a 17 x 23 map, 3 columns of padding
    assert (l.pad, l.pw, l.h_out, l.w_out, l.d_A, l.n_rows(32)) == (0, 3, 17, 23, 224 * 7 + 1, 32 * 17 * 23)
    a, g, _ = rng.layer_inputs(l, 2, 5, "relu_normal", 0.1)
    assert a.shape == (2, 224, 17, 23) and g.shape == (2, 256, 17, 23)
    assert all((x.h_out, x.w_out) == (x.h_in, x.w) for x in inc[:6])      # "same" padding keeps the map
    assert (inc[6].pad, inc[6].pw, inc[6].w_out) == (0, 0, 11)            # and one layer without
    assert (inc[1].pad, inc[1].pw) == (3, 0) and (inc[4].pad, inc[4].pw) == (1, 0)
    dn = shapes.config_layers("densenet201_imagenet")
    assert len(dn) == 201 and sum(1 for x in dn if x.kind == "conv" and x.k == 3) == 98
    assert dn[-1].c_in == 1920 and dn[1].c_in == 64 and dn[2] == shapes.LayerSpec("conv", 128, 32, 3, 1, 1, 56)
    for cin, h in ((256, 56), (512, 28), (1792, 14)):                      # the three transitions
        assert shapes.LayerSpec("conv", cin, cin // 2, 1, 1, 0, h) in dn
    assert {x.h_in for x in dn if x.kind == "conv"} == {224, 56, 28, 14, 7}
    b = shapes.config_layers("bert_base_small_batch")
    assert len(b) == 72 and all(l.rows == 512 and l.rows < l.d_A for l in b)
    # the square shorthand still means what it meant
    s = shapes.LayerSpec("conv", 4, 8, 3, 1, 1, 10)
    assert (s.kw, s.w, s.w_out, s.d_core) == (3, 10, 10, 36)


def test_generator_is_counter_based_and_seeded():
    a = rng.draw_normal(7, 0, (1000,))
    b = rng.draw_normal(7, 0, (5000,))
    assert np.array_equal(a, b[:1000])                  # element i depends on (seed, stream, i) only
    assert not np.array_equal(a, rng.draw_normal(8, 0, (1000,)))
    assert not np.array_equal(a, rng.draw_normal(7, 1, (1000,)))
    big = rng.draw_normal(3, 0, (400000,), std=0.1)
    assert abs(big.mean()) < 1e-3 and abs(big.std() - 0.1) < 1e-3
    r = rng.draw_relu_normal(3, 0, (400000,))
    assert abs((r == 0).mean() - 0.5) < 5e-3 and abs((r ** 2).mean() - 0.5) < 5e-3


def test_bf16_rounding_nearest_even():
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -2.5, 1e-3], dtype=np.float32)
    y = rng.bf16_bits_to_f32(rng.to_bf16_bits(x))
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7 -> even mantissa (1.0); 1 + 3*2^-8 ties up to 1 + 2^-6
    assert y[0] == 1.0 and y[1] == 1.0 and y[2] == np.float32(1.0 + 2.0 ** -6) and y[3] == -2.5
    assert abs(y[4] - x[4]) <= abs(x[4]) * 2.0 ** -8
    import torch
    t = torch.from_numpy(rng.draw_normal(1, 0, (4096,))).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(t, rng.bf16_bits_to_f32(rng.to_bf16_bits(rng.draw_normal(1, 0, (4096,)))))

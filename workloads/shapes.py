"""Layer-shape tables of the synthetic workloads (five headline configurations and four further sets).

The shapes stand in for the networks the paper trains (section 6.1: ResNet-110
on Cifar-10, ResNet-50 on ImageNet, Transformer encoder blocks).  Only the
layer geometry is taken; no dataset item is reproduced.  Each layer is the
linear map of the paper's layer model (section 3, s = W a), with convolutions
viewed as linear maps over im2col patches (footnote of section 3).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List


@dataclass(frozen=True)
class LayerSpec:
    kind: str            # "linear" | "conv"
    c_in: int            # linear: input features; conv: input channels
    c_out: int           # linear: output features; conv: output channels
    k: int = 1           # conv kernel size (square)
    stride: int = 1
    pad: int = 0         # zero padding of the rows of the map, and of its columns unless pad_w says otherwise
    h_in: int = 1        # conv input spatial size (square)
    rows: int = 0        # linear: number of rows (samples / tokens)
    has_bias: bool = True
    k_w: int = 0         # conv kernel width when it differs from k (0: square)
    w_in: int = 0        # conv input width when it differs from h_in (0: square)
    pad_w: int = -1      # conv padding of the columns when it differs from pad (-1: the same)

    @property
    def kw(self) -> int:
        return self.k_w if self.k_w > 0 else self.k

    @property
    def w(self) -> int:
        return self.w_in if self.w_in > 0 else self.h_in

    @property
    def pw(self) -> int:
        return self.pad_w if self.pad_w >= 0 else self.pad

    @property
    def h_out(self) -> int:
        return (self.h_in + 2 * self.pad - self.k) // self.stride + 1

    @property
    def w_out(self) -> int:
        return (self.w + 2 * self.pw - self.kw) // self.stride + 1

    @property
    def d_core(self) -> int:
        return self.c_in * self.k * self.kw if self.kind == "conv" else self.c_in

    @property
    def d_A(self) -> int:
        return self.d_core + (1 if self.has_bias else 0)

    @property
    def d_G(self) -> int:
        return self.c_out

    def n_rows(self, batch: int) -> int:
        """Rows R of the patch matrix (conv: batch * H_out * W_out)."""
        if self.kind == "conv":
            return batch * self.h_out * self.w_out
        return self.rows

    def needs_im2col(self) -> bool:
        return self.kind == "conv" and (self.k > 1 or self.kw > 1 or self.stride > 1 or self.pad > 0 or self.pw > 0)


def _conv(cin, cout, k, h, stride=1, pad=None):
    if pad is None:
        pad = (k - 1) // 2
    return LayerSpec("conv", cin, cout, k, stride, pad, h)


def _cfg1() -> List[LayerSpec]:
    return [LayerSpec("linear", 64, 32, rows=32)]


def _cfg2() -> List[LayerSpec]:
    layers = [_conv(3, 16, 3, 32)]
    layers += [_conv(16, 16, 3, 32)] * 36
    layers += [_conv(32, 32, 3, 16)] * 36
    layers += [_conv(64, 64, 3, 8)] * 36
    layers += [LayerSpec("linear", 64, 10, rows=128)]
    return layers


def _resnet50(batch: int) -> List[LayerSpec]:
    layers = [_conv(3, 64, 7, 224, stride=2, pad=3)]
    h = 56
    cin = 64
    for mid, blocks, first_stride in ((64, 3, 1), (128, 4, 2), (256, 6, 2), (512, 3, 2)):
        for b in range(blocks):
            s = first_stride if b == 0 else 1
            layers.append(_conv(cin, mid, 1, h))                      # 1x1 reduce
            layers.append(_conv(mid, mid, 3, h, stride=s))            # 3x3 (carries the stride)
            h_next = h // s
            layers.append(_conv(mid, 4 * mid, 1, h_next))             # 1x1 expand
            if b == 0:
                layers.append(_conv(cin, 4 * mid, 1, h, stride=s))    # projection shortcut
            cin = 4 * mid
            h = h_next
    layers.append(LayerSpec("linear", 2048, 1000, rows=batch))
    return layers


def _cfg5() -> List[LayerSpec]:
    block = [LayerSpec("linear", 1024, 1024, rows=4096)] * 4
    block += [LayerSpec("linear", 1024, 4096, rows=4096)]
    block += [LayerSpec("linear", 4096, 1024, rows=4096)]
    return block * 24


def _vgg16_cifar(batch: int) -> List[LayerSpec]:
    """VGG-16-shaped stack for 32x32 inputs (one of the CNNs of section 6.1): thirteen 3x3 convolutions
    with 64..512 channels (A dims up to 4609), three fully connected layers."""
    layers = []
    cin, h = 3, 32
    for cout, reps in ((64, 2), (128, 2), (256, 3), (512, 3), (512, 3)):
        for _ in range(reps):
            layers.append(_conv(cin, cout, 3, h))
            cin = cout
        h //= 2                                                        # 2x2 pooling between the groups
    layers += [LayerSpec("linear", 512, 512, rows=batch), LayerSpec("linear", 512, 512, rows=batch),
               LayerSpec("linear", 512, 10, rows=batch)]
    return layers


def _inception_nonsquare() -> List[LayerSpec]:
    """Factorised 1x7 / 7x1 and 1x3 / 3x1 convolutions with the channel counts of Inception-v4's 17x17 and
    8x8 stages (section 6.1 lists Inception-v4), padded as in the network: (k - 1) / 2 along the long side of
    the kernel only, so the map keeps its size.  One layer of each stage is also taken on a non-square map, and one
    unpadded."""
    def ns(cin, cout, kh, kw, h, w=0, same=True):
        ph, pw = ((kh - 1) // 2, (kw - 1) // 2) if same else (0, 0)
        return LayerSpec("conv", cin, cout, kh, 1, ph, h, k_w=kw, w_in=w, pad_w=pw)
    return [ns(192, 192, 1, 7, 17), ns(192, 224, 7, 1, 17), ns(224, 256, 1, 7, 17, 23),
            ns(384, 256, 1, 3, 8), ns(384, 256, 3, 1, 8), ns(448, 512, 3, 1, 8, 12),
            ns(192, 224, 1, 7, 17, same=False)]


def _densenet201(batch: int) -> List[LayerSpec]:
    """DenseNet-201-shaped layer set (section 6.1 lists DenseNet-201): growth rate 32, dense blocks of 6, 12, 48
    and 32 layers on 56, 28, 14 and 7 pixel maps.  Dense layer j of a block sees all earlier outputs, c0 + 32 j
    channels: a 1x1 bottleneck to 128 channels, then a 3x3 convolution (pad 1) to 32 new channels.  Between the
    blocks a 1x1 transition halves the channels (the 2x2 pooling after it halves the map).  201 layers: the 7x7
    stem, 2 x 98 dense-layer convolutions, 3 transitions, the classifier."""
    layers = [_conv(3, 64, 7, 224, stride=2, pad=3)]
    c, h = 64, 56
    for bi, reps in enumerate((6, 12, 48, 32)):
        for j in range(reps):
            layers.append(_conv(c + 32 * j, 128, 1, h))
            layers.append(_conv(128, 32, 3, h))
        c += 32 * reps
        if bi < 3:
            layers.append(_conv(c, c // 2, 1, h))
            c //= 2
            h //= 2
    layers.append(LayerSpec("linear", c, 1000, rows=batch))
    return layers


def _bert_small_batch() -> List[LayerSpec]:
    """BERT-base-shaped linear layers (hidden 768, FFN 3072, 12 blocks) with 4 sequences of 128 tokens per
    update (the fine-tuning batch size of section 6.1): 512 rows, so every un-averaged factor is rank-deficient."""
    block = [LayerSpec("linear", 768, 768, rows=512)] * 4
    block += [LayerSpec("linear", 768, 3072, rows=512), LayerSpec("linear", 3072, 768, rows=512)]
    return block * 12


# name -> (layers, hyper-parameters)
CONFIGS: Dict[str, dict] = {
    "fc_tiny": dict(index=1, batch=32, dtype="f32", act="normal", gout_var=1e-2,
                    damping=0.03, decay=0.95),
    "resnet110_cifar": dict(index=2, batch=128, dtype="f32", act="relu_normal", gout_var=1e-3,
                            damping=0.03, decay=0.95),
    "resnet50_imagenet": dict(index=3, batch=32, dtype="f32", act="relu_normal", gout_var=1e-3,
                              damping=0.001, decay=0.95),
    "resnet50_imagenet_bf16": dict(index=4, batch=64, dtype="bf16", act="relu_normal", gout_var=1e-3,
                                   damping=0.001, decay=0.95),
    "transformer_encoder_bf16": dict(index=5, batch=32, dtype="bf16", act="normal", gout_var=1e-4,
                                     damping=0.003, decay=0.95),
    # further layer sets of the networks section 6.1 names (not headline configurations)
    "vgg16_cifar": dict(index=6, batch=128, dtype="f32", act="relu_normal", gout_var=1e-3,
                        damping=0.03, decay=0.95),
    "inception_nonsquare": dict(index=7, batch=32, dtype="f32", act="relu_normal", gout_var=1e-3,
                                damping=0.001, decay=0.95),
    "bert_base_small_batch": dict(index=8, batch=4, dtype="f32", act="normal", gout_var=1e-4,
                                  damping=0.003, decay=0.95),
    "densenet201_imagenet": dict(index=9, batch=16, dtype="f32", act="relu_normal", gout_var=1e-3,
                                 damping=0.001, decay=0.95),
}


def config_hparams(name: str) -> dict:
    return dict(CONFIGS[name])


def config_layers(name: str) -> List[LayerSpec]:
    hp = CONFIGS[name]
    idx = hp["index"]
    if idx == 1:
        return _cfg1()
    if idx == 2:
        return _cfg2()
    if idx in (3, 4):
        return _resnet50(hp["batch"])
    if idx == 5:
        return _cfg5()
    if idx == 6:
        return _vgg16_cifar(hp["batch"])
    if idx == 7:
        return _inception_nonsquare()
    if idx == 8:
        return _bert_small_batch()
    if idx == 9:
        return _densenet201(hp["batch"])
    raise KeyError(name)


def layer_scales(layer: LayerSpec, batch: int):
    """Normalisation of the two factors: conv layers sum over spatial
    positions and average over the examples of the batch, linear layers
    average over their rows."""
    if layer.kind == "conv":
        return 1.0 / batch, 1.0 / batch
    return 1.0 / layer.rows, 1.0 / layer.rows


def factor_counts(layers: List[LayerSpec]):
    """(N_f, N_g) of section 3: sum of d_A^2 + d_G^2 and of d_G * d_A."""
    nf = sum(l.d_A ** 2 + l.d_G ** 2 for l in layers)
    ng = sum(l.d_A * l.d_G for l in layers)
    return nf, ng


def algorithmic_work(layers: List[LayerSpec], batch: int, in_bytes: int) -> dict:
    """Flops and bytes the method itself needs (triangle SYRK, n^3 inverse,
    two-sided product, patch read + write)."""
    w = dict(syrk_A=0, syrk_G=0, invert=0, precond=0, im2col_read=0, im2col_write=0,
             syrk_in_bytes=0, ema_bytes=0)
    for l in layers:
        R = l.n_rows(batch)
        w["syrk_A"] += R * l.d_A * (l.d_A + 1)
        w["syrk_G"] += R * l.d_G * (l.d_G + 1)
        w["invert"] += l.d_A ** 3 + l.d_G ** 3
        w["precond"] += 2 * l.d_G * l.d_G * l.d_A + 2 * l.d_G * l.d_A * l.d_A
        if l.kind == "conv" and (l.k > 1 or l.kw > 1):
            w["im2col_read"] += batch * l.c_in * l.h_in * l.w * in_bytes
            w["im2col_write"] += R * l.d_A * in_bytes
        w["syrk_in_bytes"] += R * (l.d_A + l.d_G) * in_bytes
        w["ema_bytes"] += 4 * (l.d_A * (l.d_A + 1) + l.d_G * (l.d_G + 1))
    return w

"""Layer-shape tables of the five synthetic workloads.

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
    pad: int = 0
    h_in: int = 1        # conv input spatial size (square)
    rows: int = 0        # linear: number of rows (samples / tokens)
    has_bias: bool = True

    @property
    def h_out(self) -> int:
        return (self.h_in + 2 * self.pad - self.k) // self.stride + 1

    @property
    def d_core(self) -> int:
        return self.c_in * self.k * self.k if self.kind == "conv" else self.c_in

    @property
    def d_A(self) -> int:
        return self.d_core + (1 if self.has_bias else 0)

    @property
    def d_G(self) -> int:
        return self.c_out

    def n_rows(self, batch: int) -> int:
        """Rows R of the patch matrix (conv: batch * H_out * W_out)."""
        if self.kind == "conv":
            return batch * self.h_out * self.h_out
        return self.rows

    def needs_im2col(self) -> bool:
        return self.kind == "conv" and (self.k > 1 or self.stride > 1 or self.pad > 0)


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
        if l.kind == "conv" and l.k > 1:
            w["im2col_read"] += batch * l.c_in * l.h_in * l.h_in * in_bytes
            w["im2col_write"] += R * l.d_A * in_bytes
        w["syrk_in_bytes"] += R * (l.d_A + l.d_G) * in_bytes
        w["ema_bytes"] += 4 * (l.d_A * (l.d_A + 1) + l.d_G * (l.d_G + 1))
    return w

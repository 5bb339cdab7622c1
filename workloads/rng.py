"""Counter-based seeded generator for the synthetic tensors.

Element ``i`` of the tensor keyed ``(seed, stream)`` is a pure function of
``(seed, stream, i)``: the splitmix64 output at counter ``i`` is split into
two 32-bit uniforms and mapped to one standard normal by Box-Muller.  The
tensors are drawn on the host so that the CPU oracle and the HIP library
consume the very same bits.  bf16 inputs are the fp32 draws rounded once to
bfloat16 on the host, round-to-nearest-even.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 20


def _mix64(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _key(seed: int, stream: int) -> np.uint64:
    with np.errstate(over="ignore"):
        k = _mix64(np.array([np.uint64(seed & 0xFFFFFFFFFFFFFFFF)], dtype=np.uint64))
        k = _mix64(k + np.uint64(stream + 1) * _GAMMA)
    return k[0]


def draw_normal(seed: int, stream: int, shape, std: float = 1.0) -> np.ndarray:
    """fp32 tensor of i.i.d. N(0, std^2) draws."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32)
    key = _key(seed, stream)

    def fill(lo):
        hi = min(n, lo + _CHUNK)
        with np.errstate(over="ignore"):
            ctr = np.arange(lo + 1, hi + 1, dtype=np.uint64)
            z = _mix64(key + ctr * _GAMMA)
        u1 = ((z >> np.uint64(32)).astype(np.float64) + 1.0) * (1.0 / 4294967296.0)   # (0, 1]
        u2 = (z & np.uint64(0xFFFFFFFF)).astype(np.float64) * (1.0 / 4294967296.0)    # [0, 1)
        g = np.sqrt(-2.0 * np.log(u1)) * np.cos((2.0 * np.pi) * u2)
        out[lo:hi] = (g * std).astype(np.float32)

    starts = range(0, n, _CHUNK)
    if len(starts) > 1:     # chunks are independent (counter based): fill them on a few threads
        with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
            list(ex.map(fill, starts))
    else:
        for lo in starts:
            fill(lo)
    return out.reshape(shape)


def draw_relu_normal(seed: int, stream: int, shape) -> np.ndarray:
    """max(z, 0) of N(0,1) draws: post-ReLU-like activations, about half zeros."""
    x = draw_normal(seed, stream, shape)
    np.maximum(x, 0.0, out=x)
    return x


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bfloat16 (nearest even); returns the uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to fp32."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def layer_inputs(layer, batch: int, seed: int, act_kind: str, gout_std: float, dtype: str = "f32"):
    """Draw (act, gout, grad) for one layer.

    act : linear [rows, d_in]; conv NCHW [B, C_in, H, W]
    gout: linear [rows, d_out]; conv NCHW [B, C_out, H_out, W_out]
    grad: [d_G, d_A] fp32, bias gradient in the last column
    For dtype "bf16", act and gout are returned as fp32 arrays whose values
    are exactly representable in bfloat16 (already rounded).
    """
    if layer.kind == "conv":
        ashape = (batch, layer.c_in, layer.h_in, layer.w)
        gshape = (batch, layer.c_out, layer.h_out, layer.w_out)
    else:
        ashape = (layer.rows, layer.c_in)
        gshape = (layer.rows, layer.c_out)
    if act_kind == "relu_normal":
        act = draw_relu_normal(seed, 0, ashape)
    else:
        act = draw_normal(seed, 0, ashape)
    gout = draw_normal(seed, 1, gshape, std=gout_std)
    grad = draw_normal(seed, 2, (layer.d_G, layer.d_A))
    if dtype == "bf16":
        act = bf16_bits_to_f32(to_bf16_bits(act)).reshape(ashape)
        gout = bf16_bits_to_f32(to_bf16_bits(gout)).reshape(gshape)
    return act, gout, grad

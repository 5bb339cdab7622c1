"""ctypes front end of the CPU oracle.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
CPU-baseline leg of bench.py.  The HIP library never touches it.

All functions take numpy arrays; floating-point inputs are the float32 values
the GPU consumes (bf16 inputs arrive already widened, exactly), all results
are float64.  The three ``*_layer`` helpers mirror the calls of the C-ABI
(update factors -> invert -> precondition) for one layer.
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from .build import build

_lib = C.CDLL(build())
_dp = C.POINTER(C.c_double)
_fp = C.POINTER(C.c_float)


def _d(a):
    return a.ctypes.data_as(_dp)


def _f(a):
    return a.ctypes.data_as(_fp)


_lib.oracle_num_threads.restype = C.c_int
_lib.oracle_factor_entry.restype = C.c_double
_lib.oracle_factor_entry.argtypes = [_dp, C.c_long, C.c_int, C.c_double, C.c_int, C.c_int]
_lib.oracle_inverse_gj.restype = C.c_int
_lib.oracle_inverse_chol.restype = C.c_int


def num_threads() -> int:
    return int(_lib.oracle_num_threads())


def patches(x: np.ndarray, kh: int, kw: int, stride: int, pad: int, has_bias: bool, pad_w: int = -1) -> np.ndarray:
    """`pad` pads the rows of the map and, unless `pad_w` >= 0 is given, its columns too."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    B, Cc, H, W = x.shape
    pad_w = pad if pad_w < 0 else pad_w
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (W + 2 * pad_w - kw) // stride + 1
    dA = Cc * kh * kw + (1 if has_bias else 0)
    out = np.empty((B * Ho * Wo, dA), dtype=np.float64)
    _lib.oracle_patches(_f(x), C.c_int(B), C.c_int(Cc), C.c_int(H), C.c_int(W), C.c_int(kh), C.c_int(kw),
                        C.c_int(stride), C.c_int(pad), C.c_int(pad_w), C.c_int(int(has_bias)), _d(out))
    return out


def linear_rows(a: np.ndarray, has_bias: bool) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    R, d = a.shape
    out = np.empty((R, d + (1 if has_bias else 0)), dtype=np.float64)
    _lib.oracle_linear_rows(_f(a), C.c_long(R), C.c_int(d), C.c_int(int(has_bias)), _d(out))
    return out


def rows_from_nchw(g: np.ndarray) -> np.ndarray:
    g = np.ascontiguousarray(g, dtype=np.float32)
    B, Cc, H, W = g.shape
    out = np.empty((B * H * W, Cc), dtype=np.float64)
    _lib.oracle_rows_from_nchw(_f(g), C.c_int(B), C.c_int(Cc), C.c_int(H), C.c_int(W), _d(out))
    return out


def factor(X: np.ndarray, scale: float) -> np.ndarray:
    X = np.ascontiguousarray(X, dtype=np.float64)
    R, d = X.shape
    F = np.empty((d, d), dtype=np.float64)
    _lib.oracle_factor(_d(X), C.c_long(R), C.c_int(d), C.c_double(scale), _d(F))
    return F


def factor_entry(X: np.ndarray, scale: float, u: int, v: int) -> float:
    assert X.dtype == np.float64 and X.flags.c_contiguous
    R, d = X.shape
    return float(_lib.oracle_factor_entry(_d(X), R, d, scale, u, v))


def running_average(F_run: np.ndarray, F_new: np.ndarray, decay: float) -> np.ndarray:
    out = np.array(F_run, dtype=np.float64, order="C")
    F_new = np.ascontiguousarray(F_new, dtype=np.float64)
    _lib.oracle_running_average(_d(out), _d(F_new), C.c_int(out.shape[0]), C.c_double(decay))
    return out


def inverse(M: np.ndarray, damping: float, method: str = "gj") -> np.ndarray:
    M = np.ascontiguousarray(M, dtype=np.float64)
    n = M.shape[0]
    out = np.empty((n, n), dtype=np.float64)
    fn = _lib.oracle_inverse_gj if method == "gj" else _lib.oracle_inverse_chol
    info = fn(_d(M), C.c_int(n), C.c_double(damping), _d(out))
    if info != 0:
        raise np.linalg.LinAlgError(f"oracle inverse ({method}) failed at pivot {info}")
    return out


def inverse_info(M: np.ndarray, damping: float) -> int:
    """Cholesky route only: 0, or the 1-based index of the first non-positive pivot."""
    M = np.ascontiguousarray(M, dtype=np.float64)
    n = M.shape[0]
    out = np.empty((n, n), dtype=np.float64)
    return int(_lib.oracle_inverse_chol(_d(M), C.c_int(n), C.c_double(damping), _d(out)))


def precondition(Ginv: np.ndarray, grad: np.ndarray, Ainv: np.ndarray) -> np.ndarray:
    Ginv = np.ascontiguousarray(Ginv, dtype=np.float64)
    Ainv = np.ascontiguousarray(Ainv, dtype=np.float64)
    grad = np.ascontiguousarray(grad, dtype=np.float64)
    dG, dA = grad.shape
    out = np.empty((dG, dA), dtype=np.float64)
    _lib.oracle_precondition(_d(Ginv), _d(grad), _d(Ainv), C.c_int(dG), C.c_int(dA), _d(out))
    return out


def eigh(M: np.ndarray):
    """(v ascending, Q with the eigenvectors in its columns) of a symmetric matrix, cyclic Jacobi."""
    M = np.ascontiguousarray(M, dtype=np.float64)
    n = M.shape[0]
    Q = np.empty((n, n), dtype=np.float64)
    v = np.empty(n, dtype=np.float64)
    _lib.oracle_eigh_jacobi(_d(M), C.c_int(n), _d(Q), _d(v))
    return v, Q


def precondition_eigen_layer(A_run, G_run, grad, gamma: float) -> np.ndarray:
    """Eq. 13 from the running factors: decompose both, then precondition."""
    vA, QA = eigh(A_run)
    vG, QG = eigh(G_run)
    return precondition_eigen(QG, vG, QA, vA, grad, gamma)


def precondition_eigen(QG, vG, QA, vA, grad, gamma: float) -> np.ndarray:
    QG = np.ascontiguousarray(QG, dtype=np.float64)
    QA = np.ascontiguousarray(QA, dtype=np.float64)
    vG = np.ascontiguousarray(vG, dtype=np.float64)
    vA = np.ascontiguousarray(vA, dtype=np.float64)
    grad = np.ascontiguousarray(grad, dtype=np.float64)
    dG, dA = grad.shape
    out = np.empty((dG, dA), dtype=np.float64)
    _lib.oracle_precondition_eigen(_d(QG), _d(vG), _d(QA), _d(vA), _d(grad), C.c_int(dG), C.c_int(dA),
                                   C.c_double(gamma), _d(out))
    return out


# ---------------------------------------------------------------------------
# one-layer helpers mirroring the C-ABI calls
# ---------------------------------------------------------------------------

def layer_rows(layer, act: np.ndarray, gout: np.ndarray):
    """(a_bar [R, d_A], g [R, d_G]) for a workloads.LayerSpec."""
    if layer.kind == "conv":
        abar = patches(act, layer.k, layer.kw, layer.stride, layer.pad, layer.has_bias, layer.pw)
        g = rows_from_nchw(gout)
    else:
        abar = linear_rows(act, layer.has_bias)
        g = np.ascontiguousarray(gout, dtype=np.float64)
    return abar, g


def update_factors_layer(layer, act, gout, scale_A, scale_G, decay, A_run, G_run):
    abar, g = layer_rows(layer, act, gout)
    A_new = factor(abar, scale_A)
    G_new = factor(g, scale_G)
    return running_average(A_run, A_new, decay), running_average(G_run, G_new, decay)


def pi_damping(A_run: np.ndarray, G_run: np.ndarray, gamma: float):
    """(lambda_A, lambda_G) of the factored Tikhonov split, Eq. 12."""
    A = np.ascontiguousarray(A_run, dtype=np.float64)
    G = np.ascontiguousarray(G_run, dtype=np.float64)
    out = np.empty(2, dtype=np.float64)
    _lib.oracle_pi_damping(_d(A), C.c_int(A.shape[0]), _d(G), C.c_int(G.shape[0]), C.c_double(gamma), _d(out))
    return float(out[0]), float(out[1])


def invert_layer_pi(A_run, G_run, gamma):
    lam_A, lam_G = pi_damping(A_run, G_run, gamma)
    return inverse(A_run, lam_A), inverse(G_run, lam_G), lam_A, lam_G


def invert_layer(A_run, G_run, damping_A, damping_G):
    return inverse(A_run, damping_A), inverse(G_run, damping_G)


def precondition_layer(A_inv, G_inv, grad):
    return precondition(G_inv, grad, A_inv)

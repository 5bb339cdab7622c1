"""ctypes binding with the same names as include/kfac.h (argument marshalling only).

Tensors are torch CUDA tensors (or anything with ``data_ptr()``); raw integer
device addresses are accepted too.  The HIP library must have been built
(``python -m paper_2206_15143_amd.build``); there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from array import array
from typing import Optional, Sequence

KFAC_F32, KFAC_BF16 = 0, 1
KFAC_LINEAR, KFAC_CONV2D = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libkfac_hip.so"
_lib = None


class KfacError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = int(status)
        super().__init__(f"{where}: {kfac_status_string(status)} (status {int(status)})")


class LayerDesc(C.Structure):
    _fields_ = [("kind", C.c_int), ("d_in", C.c_int), ("d_out", C.c_int), ("kh", C.c_int), ("kw", C.c_int),
                ("stride", C.c_int), ("pad", C.c_int), ("has_bias", C.c_int), ("in_dtype", C.c_int),
                ("pad_h", C.c_int), ("pad_w", C.c_int)]

    @staticmethod
    def linear(d_in: int, d_out: int, has_bias: bool = True, dtype: int = KFAC_F32) -> "LayerDesc":
        return LayerDesc(KFAC_LINEAR, d_in, d_out, 1, 1, 1, 0, int(has_bias), dtype)

    @staticmethod
    def conv2d(c_in: int, c_out: int, k: int, stride: int = 1, pad: int = 0, has_bias: bool = True,
               dtype: int = KFAC_F32, kw: Optional[int] = None, pad_w: Optional[int] = None) -> "LayerDesc":
        """`pad` pads the rows of the map and, unless `pad_w` is given, its columns too."""
        pw = pad if pad_w is None else pad_w
        both = min(pad, pw)
        return LayerDesc(KFAC_CONV2D, c_in, c_out, k, k if kw is None else kw, stride, both, int(has_bias), dtype,
                         pad - both, pw - both)

    @staticmethod
    def from_spec(spec, dtype: int = KFAC_F32) -> "LayerDesc":
        """From a workloads.LayerSpec-like object (kind, c_in, c_out, k, stride, pad, has_bias; kw and pw, the
        kernel width and the column padding, if present)."""
        if spec.kind == "conv":
            return LayerDesc.conv2d(spec.c_in, spec.c_out, spec.k, spec.stride, spec.pad, spec.has_bias, dtype,
                                    kw=getattr(spec, "kw", None), pad_w=getattr(spec, "pw", None))
        return LayerDesc.linear(spec.c_in, spec.c_out, spec.has_bias, dtype)


def lib_path() -> str:
    return os.path.join(_HERE, _LIB_NAME)


def load_library():
    """Load libkfac_hip.so; raises ImportError when it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -m paper_2206_15143_amd.build` "
                          "(there is no CPU or PyTorch fallback)")
    # The caller's device memory and streams come from PyTorch, which ships its own HIP runtime.  Import it
    # first so that this library binds to that same runtime: loaded the other way round the process holds
    # two runtimes and a torch stream handle means nothing to the one the kernels are launched through
    # (every launch then fails).
    import torch  # noqa: F401
    lib = C.CDLL(path)
    vp, ip, fp, sz = C.c_void_p, C.POINTER(C.c_int), C.POINTER(C.c_float), C.c_size_t
    dp = C.POINTER(LayerDesc)
    vpp = C.POINTER(C.c_void_p)
    lib.kfac_dim_A.argtypes = [dp]; lib.kfac_dim_A.restype = C.c_int
    lib.kfac_dim_G.argtypes = [dp]; lib.kfac_dim_G.restype = C.c_int
    lib.kfac_patch_ld.argtypes = [dp]; lib.kfac_patch_ld.restype = C.c_int
    lib.kfac_workspace_bytes.argtypes = [dp, C.c_int, C.c_int, C.c_int]; lib.kfac_workspace_bytes.restype = sz
    lib.kfac_workspace_bytes_batched.argtypes = [C.c_int, dp, ip, ip, ip]
    lib.kfac_workspace_bytes_batched.restype = sz
    lib.kfac_im2col.argtypes = [dp, vp, C.c_int, C.c_int, C.c_int, vp, vp]; lib.kfac_im2col.restype = C.c_int
    lib.kfac_update_factors.argtypes = [dp, vp, vp, C.c_int, C.c_int, C.c_int, C.c_float, C.c_float, C.c_float,
                                        vp, vp, vp, sz, vp]
    lib.kfac_update_factors.restype = C.c_int
    lib.kfac_invert.argtypes = [dp, vp, vp, C.c_float, C.c_float, vp, vp, vp, vp, sz, vp]
    lib.kfac_invert.restype = C.c_int
    lib.kfac_invert_pi.argtypes = [dp, vp, vp, C.c_float, vp, vp, vp, vp, vp, sz, vp]
    lib.kfac_invert_pi.restype = C.c_int
    lib.kfac_invert_pi_batched.argtypes = [C.c_int, dp, vpp, vpp, C.c_float, vpp, vpp, vp, vp, vp, sz, vp]
    lib.kfac_invert_pi_batched.restype = C.c_int
    lib.kfac_precondition.argtypes = [dp, vp, vp, vp, vp, vp, sz, vp]; lib.kfac_precondition.restype = C.c_int
    lib.kfac_precondition_static.argtypes = [dp, vp, vp, vp, vp, vp]; lib.kfac_precondition_static.restype = C.c_int
    lib.kfac_update_factors_batched.argtypes = [C.c_int, dp, vpp, vpp, ip, ip, ip, fp, fp, C.c_float, vpp, vpp,
                                                vp, sz, vp]
    lib.kfac_update_factors_batched.restype = C.c_int
    lib.kfac_invert_batched.argtypes = [C.c_int, dp, vpp, vpp, C.c_float, C.c_float, vpp, vpp, vp, vp, sz, vp]
    lib.kfac_invert_batched.restype = C.c_int
    lib.kfac_precondition_batched.argtypes = [C.c_int, dp, vpp, vpp, vpp, vpp, vp, sz, vp]
    lib.kfac_precondition_batched.restype = C.c_int
    lib.kfac_eigen.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]; lib.kfac_eigen.restype = C.c_int
    lib.kfac_eigen_batched.argtypes = [C.c_int, dp, vpp, vpp, vpp, vpp, vpp, vpp, vp, vp, sz, vp]
    lib.kfac_eigen_batched.restype = C.c_int
    lib.kfac_precondition_eigen.argtypes = [dp, vp, vp, vp, vp, C.c_float, vp, vp, vp, sz, vp]
    lib.kfac_precondition_eigen.restype = C.c_int
    lib.kfac_precondition_eigen_batched.argtypes = [C.c_int, dp, vpp, vpp, vpp, vpp, C.c_float, vpp, vpp, vp, sz, vp]
    lib.kfac_precondition_eigen_batched.restype = C.c_int
    lib.kfac_status_string.argtypes = [C.c_int]; lib.kfac_status_string.restype = C.c_char_p
    lib.kfac_version.argtypes = []; lib.kfac_version.restype = C.c_int
    lib.kfac_tune.argtypes = [C.c_char_p, C.c_long]; lib.kfac_tune.restype = C.c_int
    lib.kfac_timing_enable.argtypes = [C.c_int]; lib.kfac_timing_enable.restype = C.c_int
    lib.kfac_timing_collect.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_long), C.POINTER(C.c_double)]
    lib.kfac_timing_collect.restype = C.c_int
    lib.kfac_timing_collect_ex.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_long), C.POINTER(C.c_double),
                                           C.POINTER(C.c_double)]
    lib.kfac_timing_collect_ex.restype = C.c_int
    lib.kfac_profile_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.kfac_profile_copy.restype = C.c_int
    lib.kfac_timing_class_name.argtypes = [C.c_int]; lib.kfac_timing_class_name.restype = C.c_char_p
    lib.kfac_profile_gemm.argtypes = [vp, vp, vp, C.c_int, C.c_int, C.c_int, C.c_long, C.c_long, C.c_long, C.c_int,
                                      C.c_int, C.c_int, vp]
    lib.kfac_profile_gemm.restype = C.c_int
    _lib = lib
    return lib


def _addr(t) -> int:
    """Device address of a tensor, after the two checks a raw pointer cannot make for itself: the library
    assumes dense row-major storage, and knows 4-byte (fp32, int32), 2-byte (bfloat16) and byte (workspace)
    elements only, so a strided view or a float64 tensor is refused here instead of being misread there."""
    contiguous = getattr(t, "is_contiguous", None)
    if contiguous is not None and not contiguous():
        raise ValueError(f"tensor of shape {tuple(t.shape)} is not contiguous: the library takes dense row-major buffers")
    size = getattr(t, "element_size", None)
    if size is not None and size() not in (1, 2, 4):
        raise TypeError(f"tensor of dtype {getattr(t, 'dtype', '?')}: the library takes fp32 / int32, bfloat16 or byte buffers")
    return int(t.data_ptr())


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return _addr(t)


def _nbytes(t) -> int:
    if t is None:
        return 0
    return int(t.numel() * t.element_size())


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream) or None
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream) or None


def _check(st: int, where: str):
    if st != 0:
        raise KfacError(st, where)


def _descs(descs):
    if isinstance(descs, C.Array):
        return descs
    return (LayerDesc * len(descs))(*descs)


def _ints(v):
    if isinstance(v, C.Array):
        return v
    return (C.c_int * len(v)).from_buffer(array("i", [int(x) for x in v]))


def _floats(v):
    if isinstance(v, C.Array):
        return v
    return (C.c_float * len(v)).from_buffer(array("f", [float(x) for x in v]))


def _ptrs(ts):
    if isinstance(ts, C.Array):
        return ts
    return (C.c_void_p * len(ts)).from_buffer(array("Q", [0 if t is None else t if isinstance(t, int)
                                                          else _addr(t) for t in ts]))


def marshal_descs(descs: Sequence[LayerDesc]):
    """The C array of layer descriptors a batched call takes, built once.

    Every batched call accepts the result of a ``marshal_*`` function in place of the Python list it was
    made from, and then skips the conversion: a training loop whose layers and buffers are fixed converts
    them once instead of on every call (for a hundred layers the conversion costs as much host time as the
    preconditioning kernels take on the GPU)."""
    return _descs(list(descs))


def marshal_ptrs(tensors):
    """The C array of device addresses of ``tensors`` (see marshal_descs).  The array holds addresses, not
    references: the caller keeps the tensors alive and at the same addresses for as long as it is used."""
    return _ptrs(list(tensors))


def marshal_ints(values: Sequence[int]):
    """The C int array of ``values`` (see marshal_descs)."""
    return _ints(list(values))


def marshal_floats(values: Sequence[float]):
    """The C float array of ``values`` (see marshal_descs)."""
    return _floats(list(values))


def kfac_status_string(status: int) -> str:
    return load_library().kfac_status_string(int(status)).decode()


def kfac_version() -> int:
    return int(load_library().kfac_version())


def kfac_tune(key: str, value: int) -> None:
    if load_library().kfac_tune(key.encode(), int(value)) != 0:
        raise KeyError(key)


KFAC_K_COUNT = 21


def kfac_profile_copy(dst, src, nbytes: int, stream=None) -> None:
    if load_library().kfac_profile_copy(_ptr(dst), _ptr(src), C.c_size_t(nbytes), _stream(stream)) != 0:
        raise RuntimeError("kfac_profile_copy failed")


def kfac_profile_gemm(A, B, Cm, M, N, K, lda, ldb, ldc, mode=0, p0=0, p1=0, stream=None) -> None:
    if load_library().kfac_profile_gemm(_ptr(A), _ptr(B), _ptr(Cm), M, N, K, lda, ldb, ldc, mode, p0, p1,
                                        _stream(stream)) != 0:
        raise RuntimeError("kfac_profile_gemm failed")


def kfac_timing_enable(on: bool) -> None:
    load_library().kfac_timing_enable(int(bool(on)))


def kfac_timing_collect() -> dict:
    """{class name: (milliseconds, launches, work)} accumulated since the last collect; work is the
    algorithmic flop count of the KF-GEMM classes (0 for the others)."""
    lib = load_library()
    ms = (C.c_double * KFAC_K_COUNT)()
    cnt = (C.c_long * KFAC_K_COUNT)()
    work = (C.c_double * KFAC_K_COUNT)()
    if lib.kfac_timing_collect(ms, cnt, work) != 0:
        raise RuntimeError("kfac_timing_collect: HIP event error")
    return {lib.kfac_timing_class_name(i).decode(): (float(ms[i]), int(cnt[i]), float(work[i]))
            for i in range(KFAC_K_COUNT)}


def kfac_timing_collect_ex() -> dict:
    """{class name: (milliseconds, launches, work, executed)}: as kfac_timing_collect plus the flops the class's
    kernels execute on the MFMA units by their own method."""
    lib = load_library()
    ms = (C.c_double * KFAC_K_COUNT)()
    cnt = (C.c_long * KFAC_K_COUNT)()
    work = (C.c_double * KFAC_K_COUNT)()
    ex = (C.c_double * KFAC_K_COUNT)()
    if lib.kfac_timing_collect_ex(ms, cnt, work, ex) != 0:
        raise RuntimeError("kfac_timing_collect_ex: HIP event error")
    return {lib.kfac_timing_class_name(i).decode(): (float(ms[i]), int(cnt[i]), float(work[i]), float(ex[i]))
            for i in range(KFAC_K_COUNT)}


def kfac_dim_A(desc: LayerDesc) -> int:
    return int(load_library().kfac_dim_A(C.byref(desc)))


def kfac_dim_G(desc: LayerDesc) -> int:
    return int(load_library().kfac_dim_G(C.byref(desc)))


def kfac_patch_ld(desc: LayerDesc) -> int:
    return int(load_library().kfac_patch_ld(C.byref(desc)))


def kfac_workspace_bytes(desc: LayerDesc, batch: int, h: int = 1, w: int = 1) -> int:
    return int(load_library().kfac_workspace_bytes(C.byref(desc), batch, h, w))


def kfac_workspace_bytes_batched(descs, batch, h, w) -> int:
    return int(load_library().kfac_workspace_bytes_batched(len(descs), _descs(descs), _ints(batch), _ints(h),
                                                           _ints(w)))


def kfac_im2col(desc, act, batch, h, w, patches, stream=None) -> None:
    _check(load_library().kfac_im2col(C.byref(desc), _ptr(act), batch, h, w, _ptr(patches), _stream(stream)),
           "kfac_im2col")


def kfac_update_factors(desc, act, gout, batch, h, w, scale_A, scale_G, decay, A_run, G_run, work,
                        stream=None) -> None:
    _check(load_library().kfac_update_factors(C.byref(desc), _ptr(act), _ptr(gout), batch, h, w, scale_A, scale_G,
                                              decay, _ptr(A_run), _ptr(G_run), _ptr(work), _nbytes(work),
                                              _stream(stream)), "kfac_update_factors")


def kfac_invert(desc, A_run, G_run, damping_A, damping_G, A_inv, G_inv, info, work, stream=None) -> None:
    _check(load_library().kfac_invert(C.byref(desc), _ptr(A_run), _ptr(G_run), damping_A, damping_G, _ptr(A_inv),
                                      _ptr(G_inv), _ptr(info), _ptr(work), _nbytes(work), _stream(stream)),
           "kfac_invert")


def kfac_invert_pi(desc, A_run, G_run, gamma, A_inv, G_inv, info, damping, work, stream=None) -> None:
    _check(load_library().kfac_invert_pi(C.byref(desc), _ptr(A_run), _ptr(G_run), gamma, _ptr(A_inv), _ptr(G_inv),
                                         _ptr(info), _ptr(damping), _ptr(work), _nbytes(work), _stream(stream)),
           "kfac_invert_pi")


def kfac_precondition(desc, A_inv, G_inv, grad, out, work, stream=None) -> None:
    _check(load_library().kfac_precondition(C.byref(desc), _ptr(A_inv), _ptr(G_inv), _ptr(grad), _ptr(out),
                                            _ptr(work), _nbytes(work), _stream(stream)), "kfac_precondition")


KFAC_STATIC_SCRATCH_BYTES = 32 << 20


def kfac_precondition_static(desc, A_inv, G_inv, grad, out, stream=None) -> None:
    _check(load_library().kfac_precondition_static(C.byref(desc), _ptr(A_inv), _ptr(G_inv), _ptr(grad), _ptr(out),
                                                   _stream(stream)), "kfac_precondition_static")


def kfac_update_factors_batched(descs, acts, gouts, batch, h, w, scale_A, scale_G, decay, A_runs, G_runs, work,
                                stream=None) -> None:
    n = len(descs)
    _check(load_library().kfac_update_factors_batched(n, _descs(descs), _ptrs(acts), _ptrs(gouts), _ints(batch),
                                                      _ints(h), _ints(w), _floats(scale_A), _floats(scale_G), decay,
                                                      _ptrs(A_runs), _ptrs(G_runs), _ptr(work), _nbytes(work),
                                                      _stream(stream)), "kfac_update_factors_batched")


def kfac_invert_batched(descs, A_runs, G_runs, damping_A, damping_G, A_invs, G_invs, info, work,
                        stream=None) -> None:
    n = len(descs)
    _check(load_library().kfac_invert_batched(n, _descs(descs), _ptrs(A_runs), _ptrs(G_runs), damping_A, damping_G,
                                              _ptrs(A_invs), _ptrs(G_invs), _ptr(info), _ptr(work), _nbytes(work),
                                              _stream(stream)), "kfac_invert_batched")


def kfac_invert_pi_batched(descs, A_runs, G_runs, gamma, A_invs, G_invs, info, damping, work, stream=None) -> None:
    n = len(descs)
    _check(load_library().kfac_invert_pi_batched(n, _descs(descs), _ptrs(A_runs), _ptrs(G_runs), gamma,
                                                 _ptrs(A_invs), _ptrs(G_invs), _ptr(info), _ptr(damping),
                                                 _ptr(work), _nbytes(work), _stream(stream)),
           "kfac_invert_pi_batched")


def kfac_eigen(desc, A_run, G_run, Q_A, v_A, Q_G, v_G, info, work, stream=None) -> None:
    _check(load_library().kfac_eigen(C.byref(desc), _ptr(A_run), _ptr(G_run), _ptr(Q_A), _ptr(v_A), _ptr(Q_G),
                                     _ptr(v_G), _ptr(info), _ptr(work), _nbytes(work), _stream(stream)),
           "kfac_eigen")


def kfac_eigen_batched(descs, A_runs, G_runs, Q_As, v_As, Q_Gs, v_Gs, info, work, stream=None) -> None:
    n = len(descs)
    _check(load_library().kfac_eigen_batched(n, _descs(descs), _ptrs(A_runs), _ptrs(G_runs), _ptrs(Q_As),
                                             _ptrs(v_As), _ptrs(Q_Gs), _ptrs(v_Gs), _ptr(info), _ptr(work),
                                             _nbytes(work), _stream(stream)), "kfac_eigen_batched")


def kfac_precondition_eigen(desc, Q_A, v_A, Q_G, v_G, gamma, grad, out, work, stream=None) -> None:
    _check(load_library().kfac_precondition_eigen(C.byref(desc), _ptr(Q_A), _ptr(v_A), _ptr(Q_G), _ptr(v_G), gamma,
                                                  _ptr(grad), _ptr(out), _ptr(work), _nbytes(work),
                                                  _stream(stream)), "kfac_precondition_eigen")


def kfac_precondition_eigen_batched(descs, Q_As, v_As, Q_Gs, v_Gs, gamma, grads, outs, work, stream=None) -> None:
    n = len(descs)
    _check(load_library().kfac_precondition_eigen_batched(n, _descs(descs), _ptrs(Q_As), _ptrs(v_As), _ptrs(Q_Gs),
                                                          _ptrs(v_Gs), gamma, _ptrs(grads), _ptrs(outs),
                                                          _ptr(work), _nbytes(work), _stream(stream)),
           "kfac_precondition_eigen_batched")


def kfac_precondition_batched(descs, A_invs, G_invs, grads, outs, work, stream=None) -> None:
    n = len(descs)
    _check(load_library().kfac_precondition_batched(n, _descs(descs), _ptrs(A_invs), _ptrs(G_invs), _ptrs(grads),
                                                    _ptrs(outs), _ptr(work), _nbytes(work), _stream(stream)),
           "kfac_precondition_batched")

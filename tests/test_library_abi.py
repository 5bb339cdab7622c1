"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
symbol the header declares, and rejects bad arguments before any launch."""
import ctypes
import os
import re

import pytest

import paper_2206_15143_amd as kf

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    """Every function declared in include/*.h (comments stripped)."""
    syms = set()
    inc = os.path.join(ROOT, "include")
    for name in sorted(os.listdir(inc)):
        if not name.endswith(".h"):
            continue
        text = open(os.path.join(inc, name)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        syms |= set(re.findall(r"\b(kfac_[A-Za-z0-9_]+)\s*\(", text))
    return sorted(syms)


def test_library_loads_and_exports_every_declared_symbol():
    lib = kf.load_library()
    syms = _declared_symbols()
    assert "kfac_update_factors" in syms and "kfac_invert" in syms and "kfac_precondition" in syms
    assert len(syms) >= 21 and "kfac_invert_pi" in syms and "kfac_timing_collect" in syms
    for s in syms:
        assert hasattr(lib, s), s
    assert kf.kfac_version() >= 100
    assert kf.kfac_status_string(0) == "ok"


def test_dimension_queries():
    d = kf.LayerDesc.conv2d(16, 32, 3, 1, 1)
    assert (kf.kfac_dim_A(d), kf.kfac_dim_G(d), kf.kfac_patch_ld(d)) == (145, 32, 144)
    d = kf.LayerDesc.conv2d(3, 64, 7, 2, 3, dtype=kf.KFAC_BF16)
    assert (kf.kfac_dim_A(d), kf.kfac_patch_ld(d)) == (148, 152)
    d = kf.LayerDesc.linear(64, 32)
    assert (kf.kfac_dim_A(d), kf.kfac_dim_G(d)) == (65, 32)
    assert kf.kfac_workspace_bytes(d, 32) > 0
    assert kf.kfac_dim_A(kf.LayerDesc.linear(64, 32, has_bias=False)) == 64
    bad = kf.LayerDesc.linear(0, 32)
    assert kf.kfac_dim_A(bad) == -1


def _gpu_visible():
    import torch
    return torch.cuda.is_available()


@pytest.mark.skipif(_gpu_visible(), reason="uses fake device addresses: host-only check, never run beside a GPU")
def test_bad_arguments_are_rejected_on_the_host():
    lib = kf.load_library()
    d = kf.LayerDesc.linear(8, 4)
    fake = 0x1000   # never dereferenced: every call below must fail validation first
    # null pointers
    assert lib.kfac_update_factors(ctypes.byref(d), None, fake, 4, 1, 1, 1.0, 1.0, 0.9, fake, fake, fake, 1 << 20,
                                   None) == 1
    # decay outside [0, 1], non-positive scale, negative damping
    assert lib.kfac_update_factors(ctypes.byref(d), fake, fake, 4, 1, 1, 1.0, 1.0, 1.5, fake, fake, fake, 1 << 20,
                                   None) == 5
    assert lib.kfac_update_factors(ctypes.byref(d), fake, fake, 4, 1, 1, 0.0, 1.0, 0.5, fake, fake, fake, 1 << 20,
                                   None) == 5
    assert lib.kfac_invert(ctypes.byref(d), fake, fake, -1.0, 0.1, 0x2000, 0x3000, fake, fake, 1 << 20, None) == 5
    # bad shapes / dtype
    assert lib.kfac_update_factors(ctypes.byref(d), fake, fake, 0, 1, 1, 1.0, 1.0, 0.5, fake, fake, fake, 1 << 20,
                                   None) == 2
    bad = kf.LayerDesc.conv2d(8, 4, 3, 1, 0)
    assert lib.kfac_update_factors(ctypes.byref(bad), fake, fake, 2, 2, 2, 1.0, 1.0, 0.5, fake, fake, fake, 1 << 20,
                                   None) == 2      # 3x3 kernel does not fit a 2x2 input without padding
    # a map too wide for the patch kernel's on-chip row buffer is refused before any launch (7 x 7 fp32: 4 channels
    # x 7 rows x (w_out - 1 + 7) floats > 60 KB from 541 output columns on), by the size query as well
    wide = kf.LayerDesc.conv2d(4, 4, 7, 1, 3)
    assert lib.kfac_im2col(ctypes.byref(wide), fake, 1, 8, 600, fake, None) == 2
    assert lib.kfac_update_factors(ctypes.byref(wide), fake, fake, 1, 8, 600, 1.0, 1.0, 0.5, fake, fake, fake, 1 << 30,
                                   None) == 2
    assert kf.kfac_workspace_bytes(wide, 1, 8, 600) == 0 and kf.kfac_workspace_bytes(wide, 1, 8, 500) > 0
    # padding: negative values are refused; the two directions are separate
    neg = kf.LayerDesc.conv2d(8, 4, 3, 1, 1)
    neg.pad_w = -1
    assert lib.kfac_update_factors(ctypes.byref(neg), fake, fake, 2, 8, 8, 1.0, 1.0, 0.5, fake, fake, fake, 1 << 20,
                                   None) == 2
    tall = kf.LayerDesc.conv2d(8, 4, 7, 1, 3, kw=1, pad_w=0)       # 7 x 1 kernel, rows padded by 3, columns not
    assert (tall.pad, tall.pad_h, tall.pad_w) == (0, 3, 0)
    assert lib.kfac_im2col(ctypes.byref(tall), fake, 1, 2, 2, None, None) == 1      # shape is fine: the null pointer is what fails
    flat = kf.LayerDesc.conv2d(8, 4, 7, 1, 0, kw=1, pad_w=3)       # the same kernel with the padding on the wrong side
    assert lib.kfac_im2col(ctypes.byref(flat), fake, 1, 2, 2, fake, None) == 2
    bad = kf.LayerDesc.linear(8, 4)
    bad.in_dtype = 7
    assert lib.kfac_update_factors(ctypes.byref(bad), fake, fake, 4, 1, 1, 1.0, 1.0, 0.5, fake, fake, fake, 1 << 20,
                                   None) == 3
    # workspace too small / misaligned pointer
    assert kf.kfac_workspace_bytes(d, 4) > 64
    assert lib.kfac_update_factors(ctypes.byref(d), fake, fake, 4, 1, 1, 1.0, 1.0, 0.5, fake, fake, fake, 64,
                                   None) == 4
    assert lib.kfac_update_factors(ctypes.byref(d), fake + 2, fake, 4, 1, 1, 1.0, 1.0, 0.5, fake, fake, fake,
                                   1 << 20, None) == 7
    assert lib.kfac_precondition(ctypes.byref(d), fake, fake, fake, fake, fake, 16, None) == 4
    with pytest.raises(kf.KfacError):
        kf.kfac_precondition(d, fake, fake, fake, fake, None, stream=0)


def test_marshalled_arrays_hold_the_values_and_pass_through():
    descs = [kf.LayerDesc.linear(8, 4), kf.LayerDesc.conv2d(3, 16, 3, 1, 1, has_bias=False)]
    md = kf.marshal_descs(descs)
    assert len(md) == 2 and md[1].d_out == 16 and md[1].has_bias == 0 and md[0].d_in == 8
    mp = kf.marshal_ptrs([0x1000, None, 0x7f0000001000])
    assert [mp[i] for i in range(3)] == [0x1000, None, 0x7f0000001000]
    mi, mf = kf.marshal_ints([3, 0, -1]), kf.marshal_floats([0.5, 2.0])
    assert list(mi) == [3, 0, -1] and list(mf) == [0.5, 2.0]
    # a batched call takes the arrays in place of the lists: same answer, no conversion
    b = kf.marshal_ints([4, 2])
    one = kf.marshal_ints([1, 1])
    hw = kf.marshal_ints([1, 8])
    assert kf.kfac_workspace_bytes_batched(md, b, one, hw) == kf.kfac_workspace_bytes_batched(descs, [4, 2], [1, 1],
                                                                                              [1, 8])
    from paper_2206_15143_amd import binding
    assert binding._descs(md) is md and binding._ptrs(mp) is mp and binding._ints(mi) is mi


def test_binding_refuses_strided_views_and_float64_before_the_call():
    """The binding hands raw addresses to the library: what a pointer cannot say for itself is checked first."""
    import torch
    from paper_2206_15143_amd import binding
    x = torch.zeros(8, 8)
    assert binding._ptr(x) == x.data_ptr() and binding._ptr(None) is None and binding._ptr(4096) == 4096
    with pytest.raises(ValueError, match="not contiguous"):
        binding._ptr(x.t()[:, :4])
    with pytest.raises(TypeError, match="fp32"):
        binding._ptr(torch.zeros(4, dtype=torch.float64))
    with pytest.raises(ValueError, match="not contiguous"):
        kf.marshal_ptrs([x, x[:, ::2]])

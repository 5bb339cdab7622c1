"""MI355X (gfx950) K-FAC second-order update: thin Python binding over the C-ABI HIP library.

Every arithmetic step runs in the HIP kernels of libkfac_hip.so; this package
only marshals arguments.  PyTorch is used for device memory and streams.
"""
from .binding import (  # noqa: F401
    LayerDesc, KfacError, lib_path, load_library, marshal_descs, marshal_ptrs, marshal_ints, marshal_floats,
    kfac_dim_A, kfac_dim_G, kfac_patch_ld, kfac_workspace_bytes, kfac_workspace_bytes_batched,
    kfac_im2col, kfac_update_factors, kfac_invert, kfac_precondition, kfac_precondition_static,
    KFAC_STATIC_SCRATCH_BYTES,
    kfac_update_factors_batched, kfac_invert_batched, kfac_invert_pi, kfac_invert_pi_batched, kfac_precondition_batched,
    kfac_eigen, kfac_eigen_batched, kfac_precondition_eigen, kfac_precondition_eigen_batched,
    kfac_status_string, kfac_version, kfac_tune, kfac_timing_enable, kfac_timing_collect, kfac_timing_collect_ex, kfac_profile_copy, kfac_profile_gemm,
    KFAC_F32, KFAC_BF16, KFAC_LINEAR, KFAC_CONV2D,
)

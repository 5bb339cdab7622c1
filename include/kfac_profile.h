/*
 * kfac_profile.h - measurement hooks of the K-FAC HIP library (not needed by
 * callers of kfac.h).  Used by bench.py to time single kernel classes with HIP
 * events on the launch stream, and by tuning sweeps.
 */
#ifndef KFAC_PROFILE_H
#define KFAC_PROFILE_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Kernel classes the library launches. */
enum {
    KFAC_K_IM2COL = 0,       /* patch extraction */
    KFAC_K_SYRK = 1,         /* MFMA X^T X partial tiles (the KF-GEMM), block-tile kernel */
    KFAC_K_SYRK_REDUCE = 2,  /* split reduction + running average epilogue */
    KFAC_K_INV_INIT = 3,
    KFAC_K_INV_PIVOT = 4,
    KFAC_K_INV_PANEL = 5,
    KFAC_K_INV_FINISH = 6,
    KFAC_K_GEMM = 7,         /* A^T B MFMA GEMM (preconditioning and inverse updates) */
    KFAC_K_SYRK_WAVE = 8,    /* KF-GEMM, wave-unit kernel for row-major fp32 operands */
    KFAC_K_SYRK_CONV3 = 9,   /* KF-GEMM fused with 3x3 patch extraction (reads the NCHW input) */
    KFAC_K_SYRK_SMALL = 10,  /* KF-GEMM, direct kernel for narrow NCHW operands */
    KFAC_K_INV_STEP = 11,    /* fused sweep step: panel + update + next pivot in one launch */
    KFAC_K_SYRK_BF16 = 12,   /* KF-GEMM on the bf16 MFMA units (row-major bf16 operands) */
    KFAC_K_GEMM_WAVE = 13,   /* A^T B on the wave-unit GEMM (large preconditioning and inverse products) */
    KFAC_K_EIG_INIT = 14,    /* eigen-decomposition: working copies W = M, V = I */
    KFAC_K_EIG_ROUND = 15,   /* eigen-decomposition: one round of the block Jacobi sweep */
    KFAC_K_EIG_FINAL = 16,   /* eigen-decomposition: eigenvalues and Q = V^T; transposes for Eq. 13 */
    KFAC_K_SYRK_CORR3 = 17,  /* KF-GEMM of 3x3 convolutions from input autocorrelations (lag matrices) */
    KFAC_K_CORR3_ASM = 18,   /* border terms, sums and assembly (+ running average) of that path */
    KFAC_K_GEMM_SPLIT = 19,  /* A^T B of fp32 operands as six bf16 MFMA products of their bf16 pieces */
    KFAC_K_SYRK_SPLIT = 20,  /* KF-GEMM of wide fp32 inputs as six bf16 MFMA products of their bf16 pieces */
    KFAC_K_COUNT = 21
};

/* When enabled, every kernel launch is bracketed by a pair of HIP events
 * recorded on the launch stream (this allocates events; leave it off in
 * production), and the inversion calls keep all their kernels on the caller's
 * stream instead of spreading them over the library's streams: an event pair
 * around a kernel that has to wait for another stream's kernel to leave the
 * chip would time the wait as well.  The per-class times are therefore those
 * of each kernel running alone; their sum exceeds the wall time of a call that
 * overlaps them.  Host arrays; returns 0. */
int kfac_timing_enable(int on);
/* Waits for the recorded events, ADDS per-class elapsed milliseconds, launch
 * counts and algorithmic work into the host arrays of KFAC_K_COUNT entries (any
 * may be NULL) and forgets the recorded launches.  Work is counted for the
 * KF-GEMM classes: sum over the launch's problems of rows * d * (d + 1) flops
 * (one triangle, d including the bias column); and for KFAC_K_SYRK_REDUCE:
 * bytes, 4 * ((splits + 1) * d (d + 1) / 2 + d * d) per problem (split slices
 * and old factor read, factor written to both triangles).  Returns 0, or
 * non-zero on a HIP error. */
int kfac_timing_collect(double *ms_per_class, long *launches_per_class, double *work_per_class);
/* The same with a fourth array: the flops each class's kernels execute on the MFMA units by their own method
 * (equal to the work of the definition except where the method differs: fewer for the factors built from
 * autocorrelations, six bf16 products per fp32 product for the split-bf16 GEMM).  Set for the KF-GEMM and
 * GEMM classes, 0 elsewhere. */
int kfac_timing_collect_ex(double *ms_per_class, long *launches_per_class, double *work_per_class,
                           double *executed_per_class);
const char *kfac_timing_class_name(int cls);

/* Plain device-to-device copy kernel (calib_copy_kernel) of `bytes` bytes (a
 * multiple of 16; both pointers 16-byte aligned): a launch of known HBM traffic
 * against which hardware byte counters are scaled.  Returns 0 on success. */
int kfac_profile_copy(void *d_dst, const void *d_src, size_t bytes, void *hip_stream);

/* One product C = A^T B (A stored [K, lda], B stored [K, ldb], C [M, ldc], all fp32 device pointers) through the
 * library's GEMM routing, for timing a kernel on a shape of one's own.  mode: 0 store, 2 subtract from the lower
 * triangle outside rows / columns [p0, p1) (M == N).  Returns 0 on success. */
int kfac_profile_gemm(const float *d_A, const float *d_B, float *d_C, int M, int N, int K, long lda, long ldb,
                      long ldc, int mode, int p0, int p1, void *hip_stream);

/* Development knobs (planner targets, kernel selection switches; the keys are listed in
 * kfac_tune() in csrc/api.hip, e.g. "target_blocks", "patch_chunk_bytes", "fuse_conv3",
 * "use_bf16_mfma", "invert_fused_max_n").  Returns 0 when the key is known.  Changing a knob can
 * change the workspace requirement: query kfac_workspace_bytes* again afterwards. */
int kfac_tune(const char *key, long value);

#ifdef __cplusplus
}
#endif
#endif

// Shared host/device declarations of the K-FAC HIP library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "../../include/kfac_profile.h"

namespace kfac {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kMaxProblems = 40;   // problems per grouped launch (table travels as a kernel argument)

enum Layout : int {
    kRows = 0,   // X is [K, ld] row-major: element (k, c) at k*ld + c
    kNCHW = 1,   // X is [n][ctot][hw]: element (k = n*hw + p, c) at (n*ctot + c)*hw + p
    kConv3 = 2   // X is the NCHW input of a 3x3/stride 1/pad 1 convolution; the patch rows are implicit
};

// One factor to build: F <- decay*F + (1-decay)*scale*X^T X  (+ bias border).
struct FactorJob {
    const void *x;
    int dtype;       // 0 fp32, 1 bf16
    int layout;      // Layout
    long K;          // number of rows (samples x positions)
    long ld;         // kRows: row pitch in elements
    int d_core;      // real columns of X
    int hw, ctot;    // kNCHW / kConv3 addressing (ctot = channels)
    int h, w;        // kConv3: image size
    int has_bias;    // factor has one more row/column: column sums and the count K
    float scale, decay;
    float *F;        // [d, d], d = d_core + has_bias
};

// One SPD matrix to invert: Minv = (M + damping I)^{-1}
struct InvertJob {
    const float *M;  // [n, n], lower triangle read
    float *Minv;     // [n, n], full symmetric on exit
    int n;
    float damping;
    int *info;       // device int
    const float *damping_dev = nullptr;   // when set, the damping is read from this device float instead
    int ldm = 0;     // row pitch of M (0 = n)
    int ldo = 0;     // row pitch of Minv (0 = n)
};

// C[M, N] = A^T B with A stored [K, lda] (element (k, m)), B stored [K, ldb].
struct GemmJob {
    const float *A;
    const float *B;
    float *C;
    int M, N, K;
    long lda, ldb, ldc;
    int mode;        // GemmMode
    int p0, p1;      // kSubLowerSkip: rows/cols in [p0, p1) are left untouched; kSubRect: columns in [p0, p1)
    long doff = 0;   // kSubRect: only entries with n <= m + doff are touched
    const float *rv = nullptr, *cv = nullptr;   // kStoreDiv
    float gamma = 0.f;
    // kSubRect / kAddRect: two device words holding float bit patterns; the product is skipped unless the product of
    // the two floats exceeds gate_cond (the blocked inversion's test of a pivot block's condition number)
    const int *gate = nullptr;
    float gate_cond = 0.f;
    const float *D = nullptr;    // kSubFrom
    long ldd = 0;
    bool wide_tiles = false;     // kStore: take the split-bf16 kernel whatever the depth and tile fill
};

enum GemmMode : int {
    kStore = 0,          // C[m][n] = acc
    kStoreT = 1,         // C[n][m] = acc   (ldc is the pitch of the transposed matrix)
    kSubLowerSkip = 2,   // C[m][n] -= acc for n <= m, m and n outside [p0, p1)
    kStoreDiv = 3,       // C[m][n] = acc / (rv[m] * cv[n] + gamma)   (the division of Eq. 13)
    kSubRect = 4,        // C[m][n] -= acc for n <= m + doff, n outside [p0, p1)   (a rectangle of a lower triangle)
    kAddRect = 5,        // the same entries, C[m][n] += acc
    kSubFrom = 6         // C[m][n] = D[m][n] - acc   (D a second matrix, row pitch ldd; block-tile kernel only)
};

// Symmetric eigen-decomposition M = Q diag(v) Q^T (eigenvectors in the columns of Q, order not sorted).
struct EigenJob {
    const float *M;  // [n, n], lower triangle read
    float *Q;        // [n, n]
    float *v;        // [n]
    int *info;       // 0, or 1 when the sweep budget ran out
    int n;
};

struct Im2colJob {
    const void *x;   // NCHW
    void *out;       // [B*Ho*Wo, ld]
    int dtype;
    int B, C, H, W, kh, kw, stride, pad_h, pad_w, Ho, Wo;
    int ld;
};

// ---- planners / launchers (each returns hipSuccess or the launch error) ----
size_t syrk_workspace_bytes(const FactorJob *jobs, int n);
hipError_t syrk_launch(const FactorJob *jobs, int n, void *work, size_t work_bytes, hipStream_t s);

size_t invert_workspace_bytes(const InvertJob *jobs, int n);
hipError_t invert_launch(const InvertJob *jobs, int n, void *work, size_t work_bytes, hipStream_t s);
// lam[2i] = pi sqrt(gamma), lam[2i+1] = sqrt(gamma) / pi for the factor pair (A_i, G_i), pi from the traces (Eq. 12)
hipError_t pi_damping_launch(const float *const *A, const float *const *G, const int *dA, const int *dG, int n,
                             float gamma, float *lam, hipStream_t s);

// `work` (optional): room for the K-slice partials of deep products, gemm_workspace_bytes(jobs, n) bytes; without
// it (or with less) every product is computed in one piece
hipError_t gemm_launch(const GemmJob *jobs, int n, hipStream_t s, void *work = nullptr, size_t work_bytes = 0);
size_t gemm_workspace_bytes(const GemmJob *jobs, int n);

hipError_t im2col_launch(const Im2colJob *jobs, int n, hipStream_t s);
// whether the patch kernel can stage one output row (Wo outputs) of its narrowest channel chunk in LDS
bool im2col_fits(int kh, int kw, int stride, int Wo, int esz);
size_t eigen_workspace_bytes(const EigenJob *jobs, int n);
hipError_t eigen_launch(const EigenJob *jobs, int n, void *work, size_t work_bytes, hipStream_t s);
hipError_t transpose_launch(const float *const *src, float *const *dst, const int *n, int count, hipStream_t s);

// output rows per stage of the fused 3x3 convolution factor kernel; 0 = image shape not supported
int conv3_rows(int h, int w);

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// development knobs (set through kfac_tune)
struct Tuning {
    long target_blocks = 512;        // blocks a grouped SYRK launch aims for
    long tile_max_splits = 256;      // cap on the K splits of a block-tile SYRK problem (serial chain of its reduction)
    long small_blocks_x = 1;         // multiple of target_blocks for the narrow-NCHW kernel (loads in flight, light blocks)
    long min_tiles_per_split = 16;   // K tiles (of 16 rows) per split at least
    long patch_chunk_bytes = 160l << 20;   // patch bytes materialised per chunk in the batched path
    long im2col_piece_elems = 128;   // patch extraction: elements of one output row a workgroup writes at least
    long im2col_block_bytes = 80 * 1024;  // output bytes per workgroup aimed for
    long im2col_lds_bytes = 20 * 1024;    // slab budget of a workgroup
    long im2col_min_blocks = 1024;   // shorter strips until a layer has this many workgroups
    long eigen_max_sweeps = 20;      // sweep budget of the block Jacobi eigen-decomposition (12-13 used at order 577)
    long eigen_inner_sweeps = 1;     // Jacobi sweeps over the 32 x 32 Gram matrix of a pair of blocks per round
    long bf16_rows_copy = 1;         // bf16 NCHW operands with an odd number of positions: row-major copy first
    long invert_panel_split = 1;     // blocked sweep: panel products on the split-bf16 kernel
    long invert_refine = 1;          // blocked sweep: refinement step of the panel products (see invert.hip) ...
    long invert_fused_refine_cond = 300;  // the same test for the 64 x 64 pivot blocks of the one-launch-per-step path
    long invert_refine_cond = 3000;  // ... of pivot blocks whose condition number (maximum norm) exceeds this
    long invert_outer_block = 256;   // outer pivot block of the two-level inversion (multiple of 32)
    long invert_border_refine = 2;   // ... its refinement step: 2 always, 1 only where the sweep met an ill-conditioned pivot block
    long invert_border = 1;          // orders 64 k + 1: last row and column by bordering instead of a one-row pivot block
    long invert_two_streams = 1;     // blocked sweep and smaller factors on the library's streams (look-ahead); 0: everything on the caller's stream
    long corr3_lds_kb = 72;          // LDS budget (both slabs) of the autocorrelation kernel
    long use_corr3 = 1;              // 3x3 convolution factors of 16 / 32 / 64 channels from input autocorrelations
    long invert_fused_max_n = 1280;  // orders up to this take the one-launch-per-step sweep
    long syrk_force_bm = 0;          // 0 = choose
    long use_wave_kernel = 1;        // wave-unit SYRK for aligned row-major fp32 operands
    long use_bf16_mfma = 1;          // row-major bf16 operands: bf16 MFMA kernel instead of widening to fp32
    long gemm_xcd_remap_min = 8;     // wave GEMM launches with at least this many problems renumber their tiles per XCD
    long use_wave_gemm = 1;          // wide A^T B products on the wave-unit GEMM
    long use_split_syrk = 1;         // wide fp32 factors as six bf16 MFMA products of the inputs' bf16 pieces
    long split_syrk_min_d = 192;     // narrowest factor the split-bf16 KF-GEMM takes
    long split_syrk_fill_rows = 60;  // ... row-major inputs: when the factor fills this percentage of its 256 x 128 tiles
    long split_syrk_fill_nchw = 40;  // ... NCHW inputs (tile fill x share of real positions in the K stages)
    long split_syrk_max_stages = 32; // ... K stages (of 16 rows) per slice at most: bounds the accumulation chain
    long use_split_gemm = 1;         // large A^T B products as six bf16 MFMA products of the operands' bf16 pieces
    long split_gemm_min_m = 192;     // ... from this many output rows on
    long split_gemm_min_k = 1024;     // ... and this depth (stores only)
    long split_gemm_min_fill = 60;   // ... when the product fills at least this percentage of its 256 x 128 tiles
    long gemm_kslice_stages = 75;    // ... deep stores of a call with few tiles: K slices of about this many stages (0 = never)
    long use_small_kernel = 1;       // direct MFMA kernel for narrow NCHW operands (d <= 64)
    long fuse_conv3 = 1;             // 3x3/s1/p1 fp32 convs: build A straight from the NCHW input
    long fuse_conv3_max_c = 64;      // ... up to this many input channels (wider ones: patch matrix + split-bf16 kernel)
    long update_bm = 64;             // block tile of the inverse's rank-64 update GEMM (0 = choose; 64 measured best)
    long gemm_bm = 0;                // block tile of the preconditioning GEMMs (0 = choose)
    long wave_debug = 0;             // measurement only: 1 = skip MFMAs, 2 = skip data loads (results are wrong)
};
Tuning &tuning();

// Optional per-launch HIP-event timing (see include/kfac_profile.h).
bool timing_active();
void timing_begin(int cls, hipStream_t s);
void timing_end(hipStream_t s);
// work of the launch recorded last: `work` in units of the definition (flops of the factor, inverse or product
// being computed, or bytes), `executed` the flops the kernel's own method spends on the MFMA units (negative:
// the same as `work`)
void timing_work(double work, double executed = -1.0);

// Launch wrapper: records the event pair when timing is enabled.
#define KFAC_LAUNCH(cls, stream, kernel, grid, block, smem, ...)               \
    do {                                                                       \
        ::kfac::timing_begin((cls), (stream));                                 \
        hipLaunchKernelGGL(kernel, grid, block, smem, stream, __VA_ARGS__);    \
        ::kfac::timing_end((stream));                                          \
    } while (0)

#if defined(__HIPCC__)
// Workgroups are dealt to the eight XCDs round-robin by the hardware (workgroup i runs on XCD i mod 8).
// This renumbering gives every XCD a contiguous range of logical block ids, so that neighbouring tiles,
// which share operand panels, meet in the same XCD's L2.
__device__ __forceinline__ int xcd_block_id()
{
    const int nb = gridDim.x, x = blockIdx.x & 7, idx = blockIdx.x >> 3;
    const int base = nb >> 3, rem = nb & 7;          // XCD y holds base + (y < rem) workgroups
    return x * base + (x < rem ? x : rem) + idx;
}
#endif

}  // namespace kfac

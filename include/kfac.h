/*
 * kfac.h - C ABI of the MI355X (gfx950) K-FAC second-order update library.
 *
 * The library computes, for one layer or a set of layers, the work DP-KFAC
 * (arXiv 2206.15143) assigns to the worker that owns those layers
 * (Algorithm 1, the per-layer body of the loop over assigned layers):
 *
 *   1. Kronecker factors        A = s_A * abar^T abar,  G = s_G * g^T g     (Eq. 4)
 *      with abar the layer input (im2col patches for a convolution, the
 *      footnote of section 3; homogeneous 1 appended last for the bias),
 *   2. running average          F <- decay * F + (1 - decay) * F_new        (Eqs. 10-11)
 *   3. damped inverses          (A + lambda_A I)^{-1}, (G + lambda_G I)^{-1} (section 5.2)
 *   4. preconditioned gradient  P = G_inv * grad * A_inv                     (Eq. 5, Eq. 12 rhs)
 *
 * Conventions
 *   - Every pointer whose name starts with d_ is a DEVICE pointer owned by the
 *     caller.  The library allocates no device memory: every intermediate lives in
 *     the caller's workspace (kfac_precondition_static: in a buffer that is part of
 *     the library image).  Arrays of descriptors / pointers / scalars passed to the
 *     *_batched calls are HOST arrays of length n, read before the call returns.
 *   - State the library keeps, all of it per process:
 *       * per device, created at the first inversion call that has a factor of order
 *         above 1280 and kept until the process ends: three HIP streams (non-blocking,
 *         default priority) and 322 events (timing disabled).  See kfac_invert.
 *       * a mutex that serialises the part of an inversion call that enqueues work on
 *         those streams: inversion calls from several host threads are safe, and
 *         their enqueueing is serialised for that part.
 *       * the address of the static scratch buffer of kfac_precondition_static, per device.
 *       * the planner knobs set through kfac_tune and the timing hooks of
 *         kfac_profile.h (development and measurement interfaces: process-wide, not
 *         synchronised; change them only while no other thread is inside the library,
 *         and not between a workspace query and the call it sizes).
 *     Nothing else persists from call to call: no cached plans, no device buffers.
 *   - All matrices are row-major.  Factors and inverses are d x d fp32 with
 *     leading dimension d.  Running factors: the LOWER triangle is read; both
 *     triangles are written (mirrored) on exit.  Inverses are written as full,
 *     bitwise symmetric matrices.
 *   - Activations: LINEAR [rows, d_in]; CONV2D NCHW [batch, d_in, h, w].
 *     Output gradients: LINEAR [rows, d_out]; CONV2D NCHW [batch, d_out, h_out, w_out].
 *     Element type given by in_dtype (fp32 or bfloat16 bit patterns).  Activation, output-gradient
 *     and patch buffers must be 16-byte aligned; fp32 matrices 4-byte aligned; workspaces 256-byte aligned.
 *   - Patch column order is (c, i, j), c slowest, i.e. the flattening of a
 *     [C_out, C_in, kh, kw] weight to [C_out, C_in*kh*kw]; the bias column is
 *     LAST.  Gradients and preconditioned gradients are [d_G, d_A] fp32 with the
 *     bias gradient in the last column.
 *   - `decay` is the weight on the OLD running factor.
 *   - Calls are asynchronous on `hip_stream` (a hipStream_t, may be NULL for
 *     the default stream); the caller synchronises.  Calls that share a
 *     workspace must be ordered on one stream.
 *   - Errors detectable on the host return a non-zero kfac_status before any
 *     kernel is launched and leave all buffers untouched.  A factor that is not
 *     positive definite after damping is reported through d_info (0 = ok,
 *     k > 0 = the k-th pivot was not positive, 1-based); the contents of that
 *     inverse are then unspecified (finite or not), other matrices are unaffected.
 *   - Results are run-to-run bitwise reproducible (fixed reduction order, no
 *     floating-point atomics).
 */
#ifndef KFAC_H
#define KFAC_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    KFAC_OK = 0,
    KFAC_ERR_NULL = 1,       /* a required pointer is NULL */
    KFAC_ERR_SHAPE = 2,      /* non-positive or inconsistent dimensions */
    KFAC_ERR_DTYPE = 3,      /* unknown in_dtype / kind */
    KFAC_ERR_WORKSPACE = 4,  /* workspace smaller than kfac_workspace_bytes says */
    KFAC_ERR_PARAM = 5,      /* decay outside [0,1], negative damping, scale <= 0 */
    KFAC_ERR_HIP = 6,        /* a HIP launch failed */
    KFAC_ERR_ALIGN = 7,      /* a device pointer is not aligned as required */
    KFAC_ERR_TOO_LARGE = 8   /* kfac_precondition_static: d_A * d_G * 4 exceeds KFAC_STATIC_SCRATCH_BYTES */
} kfac_status;

typedef enum { KFAC_F32 = 0, KFAC_BF16 = 1 } kfac_dtype;
typedef enum { KFAC_LINEAR = 0, KFAC_CONV2D = 1 } kfac_kind;

/* Plain data, copied by value. */
typedef struct {
    int kind;        /* kfac_kind */
    int d_in;        /* LINEAR: input features.  CONV2D: input channels C_in */
    int d_out;       /* LINEAR: output features. CONV2D: output channels C_out */
    int kh, kw;      /* CONV2D: kernel size (groups 1, dilation 1); LINEAR: ignored */
    int stride, pad; /* CONV2D only; pad: zero padding of both map dimensions */
    int has_bias;    /* 1: homogeneous column appended last, d_A = d_in*kh*kw + 1 */
    int in_dtype;    /* kfac_dtype of activations and output gradients */
    int pad_h, pad_w; /* CONV2D only, >= 0: FURTHER zero padding of the rows (top and bottom) / of the columns
                       * (left and right) on top of `pad`, for kernels padded differently in the two directions:
                       * a 1x7 "same" convolution is pad = 0, pad_h = 0, pad_w = 3.  A descriptor that leaves
                       * both at 0 means what it meant before these fields existed.
                       * h_out = (h + 2 (pad + pad_h) - kh) / stride + 1, w_out likewise with pad_w, kw. */
} kfac_layer_desc;

/* Order of the factors (section 3: A is d_{i-1} x d_{i-1}, G is d_i x d_i). */
int kfac_dim_A(const kfac_layer_desc *desc);
int kfac_dim_G(const kfac_layer_desc *desc);

/* Leading dimension (in elements) of the patch matrix kfac_im2col writes:
 * d_in*kh*kw rounded up to 16 bytes.  The bias column is not materialised. */
int kfac_patch_ld(const kfac_layer_desc *desc);

/* Bytes of workspace sufficient for any of the per-layer calls. */
size_t kfac_workspace_bytes(const kfac_layer_desc *desc, int batch, int h, int w);
/* Same for the batched calls over n layers (host arrays). */
size_t kfac_workspace_bytes_batched(int n, const kfac_layer_desc *descs, const int *batch, const int *h,
                                    const int *w);

/* Patch extraction alone (the first step of kfac_update_factors for CONV2D
 * layers with kh*kw > 1 or stride > 1): d_patches is row-major
 * [batch*h_out*w_out, kfac_patch_ld], row (n, oh, ow), column (c, i, j), zero
 * padding, pad columns zero; same element type as the input.
 * The kernel stages one output row of a few channels on chip: a map so wide that
 * (w_out - 1) * stride + kw elements times kh rows times 4 channels (8 for bf16, fewer when kh*kw shares a
 * factor with that) exceed 60 KB is rejected with KFAC_ERR_SHAPE by every call that would extract patches
 * (output rows of more than about 540 columns for a 7x7 kernel, 1270 for 3x3, stride 1, either dtype). */
kfac_status kfac_im2col(const kfac_layer_desc *desc, const void *d_act, int batch, int h, int w,
                        void *d_patches, void *hip_stream);

/* Factor construction + running average (Eq. 4, Eqs. 10-11).  LINEAR: rows =
 * batch, h = w = 1.  d_A_run [d_A, d_A], d_G_run [d_G, d_G] are updated in place. */
kfac_status kfac_update_factors(const kfac_layer_desc *desc, const void *d_act, const void *d_gout, int batch,
                                int h, int w, float scale_A, float scale_G, float decay, float *d_A_run,
                                float *d_G_run, void *d_work, size_t work_bytes, void *hip_stream);

/* Damped inverses (section 5.2, matrix-inversion variant with the damping of
 * each factor given explicitly).  d_info: 2 ints (A, G).
 * The inversion works in place in the output buffer: d_A_inv / d_G_inv must not alias the running factors, and
 * the inverse of a factor that is reported as not positive definite holds whatever the elimination had reached
 * (see Conventions); the running factor itself is never modified.
 * Accuracy: fp32 elimination, relative error of the order of a few hundredths of cond(M) * 2^-24.  The panel
 * products of ill-conditioned pivot blocks are refined once and the bordering step of orders 64 k + 1 corrected
 * to second order (both decided on the device from the condition number of the pivot block), which keeps the
 * result within a factor two of an fp32 LAPACK Cholesky inverse up to condition numbers of a few 1e5.
 * Streams: when a call has a factor of order above 1280, part of the work (the short dependent kernels of every
 * elimination step, and the factors of order up to 1280) runs on the three library streams named under
 * Conventions, forked from and joined back to hip_stream by events inside the call: ordering on hip_stream is
 * as if everything ran there, and the call may be captured into a HIP graph like any other. */
kfac_status kfac_invert(const kfac_layer_desc *desc, const float *d_A_run, const float *d_G_run,
                        float damping_A, float damping_G, float *d_A_inv, float *d_G_inv, int *d_info,
                        void *d_work, size_t work_bytes, void *hip_stream);

/* Damped inverses with the factored Tikhonov split of Eq. 12: from the running factors,
 *   pi = sqrt((tr A / d_A) / (tr G / d_G)),  lambda_A = pi sqrt(gamma),  lambda_G = sqrt(gamma) / pi,
 * computed on the device (no host synchronisation), then A_inv = (A + lambda_A I)^{-1},
 * G_inv = (G + lambda_G I)^{-1}.  A trace that is not positive leaves pi = 1.  d_damping may be NULL;
 * otherwise 2 floats receive (lambda_A, lambda_G).  gamma >= 0.  Everything else as kfac_invert. */
kfac_status kfac_invert_pi(const kfac_layer_desc *desc, const float *d_A_run, const float *d_G_run, float gamma,
                           float *d_A_inv, float *d_G_inv, int *d_info, float *d_damping, void *d_work,
                           size_t work_bytes, void *hip_stream);

/* P = G_inv * grad * A_inv (Eq. 5 / right-hand side of Eq. 12).  d_out may alias d_grad.  The workspace holds
 * the d_A x d_G intermediate of every layer; with the size kfac_workspace_bytes reports there is also room for
 * partial products, and a call of few, deep products (orders above about 1800) then computes each in K slices
 * that are summed in a fixed order (same result on every call; it differs in the last bits from the result of
 * a call whose workspace has room for the intermediates only, which computes every product in one piece). */
kfac_status kfac_precondition(const kfac_layer_desc *desc, const float *d_A_inv, const float *d_G_inv,
                              const float *d_grad, float *d_out, void *d_work, size_t work_bytes,
                              void *hip_stream);

/* kfac_precondition for callers that cannot allocate device memory or pass a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same two products, by the same kernels,
 * with the d_A x d_G intermediate in a buffer of KFAC_STATIC_SCRATCH_BYTES that is part of the library image
 * (one copy per GPU, held until the process ends).  Allocates nothing.  A layer with
 * d_A * d_G * 4 > KFAC_STATIC_SCRATCH_BYTES is rejected with KFAC_ERR_TOO_LARGE before any launch.  Every
 * call on a GPU shares that GPU's buffer: calls that may overlap on one GPU (different streams, different
 * host threads) race and must be ordered by the caller.  Nothing in the buffer needs clearing between calls
 * (the first product overwrites all of what the second reads).  Every product is computed in one piece (no K
 * slices): the result equals kfac_precondition's bit for bit for a layer that call does not slice, and to
 * rounding otherwise.  Arguments as kfac_precondition. */
#define KFAC_STATIC_SCRATCH_BYTES (32u << 20)
kfac_status kfac_precondition_static(const kfac_layer_desc *desc, const float *d_A_inv, const float *d_G_inv,
                                     const float *d_grad, float *d_out, void *hip_stream);

/* Eigen-decomposition variant of the preconditioner (section 5.2, Eq. 13).
 *
 * kfac_eigen: A_run = Q_A diag(v_A) Q_A^T and G_run = Q_G diag(v_G) Q_G^T.  d_Q_A [d_A, d_A], d_Q_G [d_G, d_G]
 * fp32 row-major with the eigenvectors in their COLUMNS; d_v_A [d_A], d_v_G [d_G] the eigenvalues, entry k
 * belonging to column k (no particular order).  The running factors are read (lower triangle) and not
 * modified; outputs must not alias them.  d_info: 2 ints (A, G): 0 = converged, 1 = the sweep budget of the
 * iteration ran out (the results are then the current iterate: still an orthogonal Q with W = Q^T M).
 *
 * kfac_precondition_eigen:  P = Q_G [ (Q_G^T grad Q_A) ./ (v_G v_A^T + gamma) ] Q_A^T, gamma >= 0.
 * Shapes of grad / out as in kfac_precondition; d_out may alias d_grad. */
kfac_status kfac_eigen(const kfac_layer_desc *desc, const float *d_A_run, const float *d_G_run, float *d_Q_A,
                       float *d_v_A, float *d_Q_G, float *d_v_G, int *d_info, void *d_work, size_t work_bytes,
                       void *hip_stream);
kfac_status kfac_precondition_eigen(const kfac_layer_desc *desc, const float *d_Q_A, const float *d_v_A,
                                    const float *d_Q_G, const float *d_v_G, float gamma, const float *d_grad,
                                    float *d_out, void *d_work, size_t work_bytes, void *hip_stream);

/* Grouped forms: the same three operations for n layers in one launch
 * sequence (layers of one size class share kernel launches).  Host arrays of
 * length n; d_info holds 2*n ints, (A, G) per layer. */
kfac_status kfac_update_factors_batched(int n, const kfac_layer_desc *descs, const void *const *d_act,
                                        const void *const *d_gout, const int *batch, const int *h,
                                        const int *w, const float *scale_A, const float *scale_G, float decay,
                                        float *const *d_A_run, float *const *d_G_run, void *d_work,
                                        size_t work_bytes, void *hip_stream);
kfac_status kfac_invert_batched(int n, const kfac_layer_desc *descs, const float *const *d_A_run,
                                const float *const *d_G_run, float damping_A, float damping_G,
                                float *const *d_A_inv, float *const *d_G_inv, int *d_info, void *d_work,
                                size_t work_bytes, void *hip_stream);
/* d_damping: NULL or 2*n floats, (lambda_A, lambda_G) per layer. */
kfac_status kfac_invert_pi_batched(int n, const kfac_layer_desc *descs, const float *const *d_A_run,
                                   const float *const *d_G_run, float gamma, float *const *d_A_inv,
                                   float *const *d_G_inv, int *d_info, float *d_damping, void *d_work,
                                   size_t work_bytes, void *hip_stream);
kfac_status kfac_precondition_batched(int n, const kfac_layer_desc *descs, const float *const *d_A_inv,
                                      const float *const *d_G_inv, const float *const *d_grad,
                                      float *const *d_out, void *d_work, size_t work_bytes, void *hip_stream);

kfac_status kfac_eigen_batched(int n, const kfac_layer_desc *descs, const float *const *d_A_run,
                               const float *const *d_G_run, float *const *d_Q_A, float *const *d_v_A,
                               float *const *d_Q_G, float *const *d_v_G, int *d_info, void *d_work,
                               size_t work_bytes, void *hip_stream);
kfac_status kfac_precondition_eigen_batched(int n, const kfac_layer_desc *descs, const float *const *d_Q_A,
                                            const float *const *d_v_A, const float *const *d_Q_G,
                                            const float *const *d_v_G, float gamma, const float *const *d_grad,
                                            float *const *d_out, void *d_work, size_t work_bytes,
                                            void *hip_stream);

const char *kfac_status_string(kfac_status s);
int kfac_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KFAC_H */

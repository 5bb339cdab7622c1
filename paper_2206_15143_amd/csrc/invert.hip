// Damped inverse of the Kronecker factors, (M + damping I)^{-1} (section 5.2 of
// the DP-KFAC paper, matrix-inversion variant).
//
// Method: blocked symmetric Gauss-Jordan ("sweep") on the lower triangle,
// batched over matrices.  Sweeping the pivot block K of a symmetric matrix does
//     P      = M_KK^{-1}
//     M_iK  <- M_iK P                      (i != K)
//     M_ij  <- M_ij - M_iK P M_Kj          (i, j != K)
//     M_KK  <- -P
// and after all blocks have been swept the matrix holds -M^{-1}.  The pivots met
// on the way are the pivots of the Cholesky / LDL^T factorisation (the
// technique section 5.2 names), so "pivot k not positive" is the same
// positive-definiteness test; unlike potrf + trtri + lauum there is a single
// pass of n/nb steps, every step is one rank-nb MFMA update of the whole
// triangle (n^3 flops in total) and the result appears in place.
//
// Two forms, chosen per matrix by its order:
//   - up to invert_fused_max_n (1280): 64-row blocks, ONE launch per step for all
//     matrices (invert_fused.hpp): panel product, update and the inversion of
//     the next pivot block fused;
//   - above: two-level blocking with 256-row outer blocks (BlockedRun below): the
//     pivot block is inverted by the first form, the panel product W = P V, its
//     gated refinement and the rank-256 update run on the split-bf16 GEMM
//     (gemm_split.hpp), small kernels gather the old panel K-major and scatter
//     the new one; with the library's streams the short dependent launches of
//     step K+1 run beside the update of step K (look-ahead).
// kfac_invert_pi computes the two damping terms of Eq. 12 on the device first
// (pi_damping_kernel) and the kernels above read them through a device pointer.
#include "invert_fused.hpp"

#include <algorithm>
#include <mutex>
#include <vector>

namespace kfac {

constexpr int NB = 64;   // pivot block order

__device__ __forceinline__ long lmin(long a, long b) { return a < b ? a : b; }

struct InvProb {
    const float *M;
    float *W;        // working matrix = output buffer [n, n]
    float *P;        // [NB, NB] pivot-block inverse
    float *Vt;       // [NB, ldv]
    float *Wt;       // [NB, ldv]
    int *info;
    int n;
    int ldv;         // n rounded up to 4 (16-byte aligned rows)
    float damping;
    int blk_start;
    const float *dptr;   // device-side damping (overrides `damping` when not null)
    int *gate;           // null, or the two gate words of the blocked sweep, cleared with info
};

struct InvTable {
    int count;
    int step;
    InvProb p[kMaxProblems];
};

// W(lower) = M(lower) + damping I
__global__ __launch_bounds__(256) void sweep_init_kernel(const InvTable tab)
{
    int pi = 0;
    while (pi + 1 < tab.count && (int)blockIdx.x >= tab.p[pi + 1].blk_start) ++pi;
    const InvProb &pr = tab.p[pi];
    const int local = blockIdx.x - pr.blk_start;
    const long total = (long)pr.n * pr.n;
    const float damping = pr.dptr ? *pr.dptr : pr.damping;
    if (local == 0 && threadIdx.x == 0) {
        *pr.info = 0;
        if (pr.gate) { pr.gate[0] = 0; pr.gate[1] = 0; }
    }
    for (long e = (long)local * 4096 + threadIdx.x; e < lmin(total, (long)(local + 1) * 4096); e += 256) {
        const int i = (int)(e / pr.n), j = (int)(e - (long)i * pr.n);
        if (j <= i) pr.W[e] = pr.M[e] + (i == j ? damping : 0.f);
    }
}

// ---- two-level blocked sweep for the large factors -------------------------------------------
// Outer pivot blocks of PB rows (invert_outer_block, 256; a multiple of the 32-wide gather / scatter tiles, at
// most 512).  Per outer step: the pivot block is inverted by the one-launch-per-step sweep above (a PB x PB
// problem), the old panel is gathered K-major into V, W = V P (refined once where the pivot block is
// ill-conditioned) and the rank-PB update of the rest of the triangle run on the split-bf16 GEMM, and the new panel
// and -P are scattered back in place.  512 is 12 % faster on the workloads with many large factors, but the error
// of the inverse grows with the order of the explicitly inverted pivot block (measured at order 2305:
// 2.8e-5 / 6.2e-5 for 256 / 512), so 256 stays.
inline int outer_block() { return (int)std::min(512l, std::max(64l, tuning().invert_outer_block / 32 * 32)); }

struct BlkProb {
    float *W;          // working matrix [n, n]
    float *Vt;         // [PB, ldv]
    float *Wt;         // [PB, ldv]
    float *S;          // [PB, pb] the pivot block before its inversion, both triangles, or null
    int *gate;         // two words: bit patterns of the maximum norms of S and of P (see blk_cond_kernel)
    float gate_cond;   // the refinement runs when their product exceeds this
    const float *P;    // [PB, PB] inverse of the pivot block
    int *info;
    const int *ninfo;  // status of the pivot block inversion (0 or 1-based pivot index inside the block)
    int n, ldv, p0, bs;
    int pb;            // row pitch of P
    int blk_start;
};

struct BlkTable {
    int count;
    BlkProb p[32];
};

// Does the refinement of the panel product pay for this pivot block?  The condition number of the block in the
// maximum norm, ||S|| ||P|| with the largest absolute row sums (S from the lower triangle of the working matrix,
// P from the nested inversion).  A workgroup per 32 rows forms the sums of its rows and folds their largest into
// gate[0] (S) and gate[1] (P) with an integer atomic maximum on the bit patterns (the values are not negative:
// the order is the same and the result does not depend on the order of arrival).  The gather kernel and the two
// refinement products compare the product of the two with the threshold; the scatter kernel at the end of the
// step clears both words for the next one.  (A comparison with a NaN is false: a block whose inversion failed
// is left alone, its matrix is already flagged.)
__device__ __forceinline__ bool blk_gate_open(const int *gate, float cond)
{
    return __int_as_float(gate[0]) * __int_as_float(gate[1]) > cond;
}

__global__ __launch_bounds__(256) void blk_cond_kernel(const BlkTable tab)
{
    __shared__ float part[3][8][33];
    __shared__ float rowpart[32];
    int pi = 0;
    while (pi + 1 < tab.count && (int)blockIdx.x >= tab.p[pi + 1].blk_start) ++pi;
    const BlkProb &pr = tab.p[pi];
    const int i0 = ((int)blockIdx.x - pr.blk_start) * 32;
    const long n = pr.n;
    const int p0 = pr.p0, bs = pr.bs;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int c = i0 + tx;
    // rows i0 .. i0 + 31 left of the diagonal: lanes along the row, four rows per group of 32 threads
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int r = i0 + ty + 8 * j;
        float a = 0.f;
        if (r < bs) {
#pragma unroll 8
            for (int b = tx; b < r; b += 32) a += fabsf(pr.W[(p0 + r) * n + p0 + b]);
        }
#pragma unroll
        for (int off = 16; off > 0; off >>= 1) a += __shfl_xor(a, off, 32);
        if (tx == 0) rowpart[ty + 8 * j] = a;
    }
    // the rest of row c is column c from the diagonal down; P is full: its column c
    float as = 0.f, ap = 0.f;
    if (c < bs) {
#pragma unroll 8
        for (int b = i0 + ty; b < bs; b += 8)
            if (b >= c) as += fabsf(pr.W[(p0 + b) * n + p0 + c]);
#pragma unroll 8
        for (int b = ty; b < bs; b += 8) ap += fabsf(pr.P[(long)b * pr.pb + c]);
    }
    part[0][ty][tx] = as;
    part[1][ty][tx] = ap;
    __syncthreads();
    if (ty == 0) {
        float ss = rowpart[tx], ps = 0.f;
#pragma unroll
        for (int k = 0; k < 8; ++k) { ss += part[0][k][tx]; ps += part[1][k][tx]; }
#pragma unroll
        for (int off = 16; off > 0; off >>= 1) {
            ss = fmaxf(ss, __shfl_xor(ss, off, 32));
            ps = fmaxf(ps, __shfl_xor(ps, off, 32));
        }
        if (tx == 0) {
            // NaN sums (a failed nested inversion) must not look like large numbers to the integer maximum
            atomicMax(pr.gate, ss >= 0.f ? __float_as_int(ss) : 0);
            atomicMax(pr.gate + 1, ps >= 0.f ? __float_as_int(ps) : 0);
        }
    }
}

// V[kk][gi] = old panel, K-major: row panel (gi < p0) copied, column panel (gi >= p0 + bs) transposed
// through LDS, pivot columns zero.  One workgroup per 32 x 32 tile.  With the refinement of the panel product
// on, the pivot block itself, mirrored to both triangles, goes to S (whether or not the gate will open: the test of
// the pivot block runs beside this kernel on another stream).
__global__ __launch_bounds__(256) void blk_gather_kernel(const BlkTable tab)
{
    __shared__ float t[32][33];
    int pi = 0;
    while (pi + 1 < tab.count && (int)blockIdx.x >= tab.p[pi + 1].blk_start) ++pi;
    const BlkProb &pr = tab.p[pi];
    const int local = blockIdx.x - pr.blk_start;
    const int kt = (pr.bs + 31) / 32;
    const int gt = local / kt, kq = local - gt * kt;
    const int g0 = gt * 32, k0 = kq * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const long n = pr.n;
    const int p0 = pr.p0, p1 = pr.p0 + pr.bs;
    float *S = pr.S;      // null unless the refinement is on
    // p0 and p1 are multiples of 32 (or p1 = n): a tile lies wholly in one of the three regions
    if (g0 < p0) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int kk = k0 + ty + 8 * r, gi = g0 + tx;
            if (kk < pr.bs && gi < pr.n) {
                const float v = pr.W[(p0 + kk) * n + gi];
                pr.Vt[(long)kk * pr.ldv + gi] = v;
            }
        }
    } else if (g0 >= p1) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int gi = g0 + ty + 8 * r, kk = k0 + tx;
            t[ty + 8 * r][tx] = (gi < pr.n && kk < pr.bs) ? pr.W[gi * n + p0 + kk] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int kk = k0 + ty + 8 * r, gi = g0 + tx;
            if (kk < pr.bs && gi < pr.n) {
                pr.Vt[(long)kk * pr.ldv + gi] = t[tx][ty + 8 * r];
            }
        }
    } else {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int kk = k0 + ty + 8 * r, gi = g0 + tx;
            if (kk < pr.bs && gi < pr.n) {
                pr.Vt[(long)kk * pr.ldv + gi] = 0.f;
                if (S) {   // entry (kk, gi - p0) of the pivot block, from its lower triangle
                    const int b = gi - p0, hi = kk > b ? kk : b, lo = kk > b ? b : kk;
                    S[(long)kk * pr.pb + b] = pr.W[(p0 + hi) * n + p0 + lo];
                }
            }
        }
    }
}

// New panel W = V P back in place (row panel copied, column panel transposed), pivot block <- -P,
// and the pivot-block status folded into the matrix's info.
__global__ __launch_bounds__(256) void blk_scatter_kernel(const BlkTable tab)
{
    __shared__ float t[32][33];
    int pi = 0;
    while (pi + 1 < tab.count && (int)blockIdx.x >= tab.p[pi + 1].blk_start) ++pi;
    const BlkProb &pr = tab.p[pi];
    const int local = blockIdx.x - pr.blk_start;
    const int kt = (pr.bs + 31) / 32;
    const int gt = local / kt, kq = local - gt * kt;
    const int g0 = gt * 32, k0 = kq * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const long n = pr.n;
    const int p0 = pr.p0, p1 = pr.p0 + pr.bs;
    if (local == 0 && threadIdx.x == 0) {
        const int f = *pr.ninfo;
        if (f != 0 && *pr.info == 0) *pr.info = p0 + f;
        if (pr.gate) { pr.gate[0] = 0; pr.gate[1] = 0; }   // for the next step's blk_cond_kernel
    }
    if (g0 < p0) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int kk = k0 + ty + 8 * r, gi = g0 + tx;
            if (kk < pr.bs && gi < pr.n) pr.W[(p0 + kk) * n + gi] = pr.Wt[(long)kk * pr.ldv + gi];
        }
    } else if (g0 >= p1) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int kk = k0 + ty + 8 * r, gi = g0 + tx;
            t[ty + 8 * r][tx] = (kk < pr.bs && gi < pr.n) ? pr.Wt[(long)kk * pr.ldv + gi] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int gi = g0 + ty + 8 * r, kk = k0 + tx;
            if (gi < pr.n && kk < pr.bs) pr.W[gi * n + p0 + kk] = t[tx][ty + 8 * r];
        }
    } else {
        // pivot block: rows g0.., columns k0..; lower part <- -P
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int a = g0 - p0 + ty + 8 * r, b = k0 + tx;
            if (a < pr.bs && b <= a) pr.W[(p0 + a) * n + p0 + b] = -pr.P[a * pr.pb + b];
        }
    }
}

// out = -W mirrored to both triangles (in place).  One workgroup per 32 x 32 tile of the lower
// triangle; the mirror image goes through LDS so that both stores are along rows.
__global__ __launch_bounds__(256) void sweep_finish_kernel(const InvTable tab)
{
    __shared__ float t[32][33];
    int pi = 0;
    while (pi + 1 < tab.count && (int)blockIdx.x >= tab.p[pi + 1].blk_start) ++pi;
    const InvProb &pr = tab.p[pi];
    int bi, bj;
    tri_decode(blockIdx.x - pr.blk_start, bi, bj);
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const long n = pr.n;
    const int i0 = bi * 32, j0 = bj * 32;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int i = i0 + ty + 8 * r, j = j0 + tx;
        float v = 0.f;
        if (i < pr.n && j <= i) {
            v = -pr.W[i * n + j];
            pr.W[i * n + j] = v;
        }
        t[ty + 8 * r][tx] = v;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        // element (j, i) of the upper triangle, j from this tile's columns, i from its rows
        const int j = j0 + ty + 8 * r, i = i0 + tx;
        if (i < pr.n && j < i) pr.W[j * n + i] = t[tx][ty + 8 * r];
    }
}

namespace {
bool takes_fused(int n) { return n <= tuning().invert_fused_max_n; }
size_t fused_ws_floats(int n) { return 4 * (size_t)NB * NB + 2 * (size_t)NB * ((n + 3) / 4 * 4) + 16; }
// large matrices: two sets of V, W panels, P, the workspace of the nested pivot-block inversion, its status word
size_t job_ws_floats(int n)
{
    if (takes_fused(n)) return fused_ws_floats(n);
    const size_t PB = (size_t)outer_block();
    return 5 * PB * ((n + 3) / 4 * 4) + 2 * PB * PB + fused_ws_floats((int)PB) + 64;
}
// the three flags at the end of a matrix's one-launch-per-step workspace: gate of either step parity, sticky flag
int *fused_gate_ptr(float *ws, int n)
{
    return reinterpret_cast<int *>(ws + 4 * (size_t)NB * NB + 2 * (size_t)NB * ((n + 3) / 4 * 4));
}
size_t table_bytes(int n) { return align_up((size_t)2 * n * sizeof(InvProbF), 256); }

// One-launch-per-step sweep for the matrices listed in `idx` (sorted by order, largest first).
hipError_t fused_launch(const InvertJob *jobs, const std::vector<int> &idx, const std::vector<size_t> &offs,
                        void *work, InvProbF *dtab, hipStream_t s)
{
    const int total = (int)idx.size();
    // descriptors -> device table
    for (int g0 = 0; g0 < total; g0 += kInvUploadMax) {
        InvUpload u;
        u.dst = dtab + g0;
        u.count = std::min(kInvUploadMax, total - g0);
        for (int k = 0; k < u.count; ++k) {
            const InvertJob &j = jobs[idx[g0 + k]];
            InvProbF &p = u.p[k];
            float *ws = reinterpret_cast<float *>(static_cast<char *>(work) + offs[idx[g0 + k]]);
            p.M = j.M; p.W = j.Minv; p.info = j.info; p.n = j.n; p.damping = j.damping; p.dptr = j.damping_dev;
            p.ldv = (j.n + 3) / 4 * 4;
            p.nblk = (j.n + FNB - 1) / FNB;
            p.ldm = j.ldm > 0 ? j.ldm : j.n;
            p.ldw = j.ldo > 0 ? j.ldo : j.n;
            p.P = ws;
            p.Vt = ws + 2 * FNB * FNB;
            p.S = p.Vt + 2 * (size_t)FNB * p.ldv;
            p.gate = fused_gate_ptr(ws, j.n);
        }
        KFAC_LAUNCH(KFAC_K_INV_INIT, s, inv_upload_kernel, dim3((u.count + 15) / 16), dim3(64), 0, u);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    // classes of equal order, in sequences of at most kMaxInvClasses
    int c0 = 0;
    while (c0 < total) {
        InvSeq q;
        q.tab = dtab;
        q.nclass = 0;
        q.step = 0;
        q.refine_cond = tuning().invert_refine ? (float)tuning().invert_fused_refine_cond : -1.f;
        int c = c0;
        while (c < total && q.nclass < kMaxInvClasses) {
            int e = c;
            while (e < total && jobs[idx[e]].n == jobs[idx[c]].n) ++e;
            InvClass &k = q.c[q.nclass++];
            k.first = c; k.count = e - c; k.n = jobs[idx[c]].n; k.nblk = (k.n + FNB - 1) / FNB;
            k.per = 0; k.blk_start = 0;
            c = e;
        }
        c0 = c;
        auto lay_out = [&](InvSeq &t, int nclass, auto per_fn) {
            long blocks = 0;
            t.nclass = nclass;
            for (int k = 0; k < nclass; ++k) {
                t.c[k].per = per_fn(t.c[k]);
                t.c[k].blk_start = (int)blocks;
                blocks += (long)t.c[k].per * seq_slots(t.c[k].count);
            }
            return blocks;
        };
        const int nclass = q.nclass;
        long blocks = 0;
        hipError_t e = hipSuccess;
        blocks = lay_out(q, nclass, [](const InvClass &k) { return k.nblk; });
        KFAC_LAUNCH(KFAC_K_INV_PIVOT, s, fsweep_pivot0_kernel, dim3((unsigned)blocks), dim3(256), 0, q);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        const int steps = q.c[0].nblk;   // classes are sorted: the first is the largest
        for (int st = 0; st < steps && steps > 1; ++st) {
            int active = 0;
            while (active < nclass && q.c[active].nblk > st && q.c[active].nblk > 1) ++active;
            if (active == 0) break;
            q.step = st;
            blocks = lay_out(q, active, [](const InvClass &k) { return k.nblk * (k.nblk + 1) / 2; });
            if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
            KFAC_LAUNCH(KFAC_K_INV_STEP, s, fsweep_step_kernel, dim3((unsigned)blocks), dim3(256), 0, q);
            {   // a rank-64 update of the triangle, n^2 * 64 flops per matrix; every tile also forms its own W = V P
                double fl = 0.0;
                for (int k = 0; k < active; ++k) fl += (double)q.c[k].count * q.c[k].n * q.c[k].n * FNB;
                timing_work(fl, 2.0 * fl);
            }
            e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}
// Two-level blocked sweep of the matrices listed in `idx` (sorted by order, largest first).  An outer step K is
// cut into a *chain* (inverse of pivot block K, gather of the old panel, panel product, scatter: short dependent
// launches) and a *bulk* rank-PB update of everything outside the pivot rows and columns.  With look-ahead the
// chain of step K+1 runs on a second stream beside the bulk update of step K: the bulk update then leaves out
// the rows and columns of pivot block K+1 as well, and the chain of step K+1 first applies update K to just
// that band (two rectangular products), so that its pivot block and panel are ready without waiting for the
// bulk.  Panels are double buffered (the bulk of step K reads panels K while the chain writes panels K+1).
struct BlockedRun {
    struct Big { float *Vt[2], *Wt[2], *Rt, *S, *P, *nws; int *ninfo; int ldv; };
    bool refine = false;
    const InvertJob *jobs = nullptr;
    std::vector<int> idx;
    const std::vector<size_t> *offs = nullptr;
    void *work = nullptr;
    InvProbF *dtab = nullptr;
    std::vector<Big> big;
    int total = 0, PB = 0, steps = 0;
    std::vector<InvertJob> nested;
    std::vector<int> nidx;
    std::vector<size_t> noffs;
    std::vector<GemmJob> gj;

    int active(int st) const
    {
        int a = 0;
        while (a < total && jobs[idx[a]].n > st * PB) ++a;
        return a;
    }
    hipError_t start(hipStream_t s);
    hipError_t look(int st, int part, hipStream_t s);   // update st applied to the band of pivot block st + 1
    hipError_t chain(int st, hipStream_t sn, hipStream_t sc, hipEvent_t before_gather, hipEvent_t ev_nest,
                     hipEvent_t ev_cond);
    hipError_t bulk(int st, bool skip_next, hipStream_t s);
    hipError_t finish(hipStream_t s);
    hipError_t copy_kernel(int what, int st, int act, hipStream_t s);    // 0 gather, 1 scatter, 2 condition test
};

hipError_t BlockedRun::start(hipStream_t s)
{
    total = (int)idx.size();
    PB = outer_block();
    refine = tuning().invert_refine != 0;
    big.assign(total, Big());
    for (int k = 0; k < total; ++k) {
        const InvertJob &j = jobs[idx[k]];
        float *ws = reinterpret_cast<float *>(static_cast<char *>(work) + (*offs)[idx[k]]);
        Big &b = big[k];
        b.ldv = (j.n + 3) / 4 * 4;
        const size_t panel = (size_t)PB * b.ldv;
        b.Vt[0] = ws;
        b.Wt[0] = ws + panel;
        b.Vt[1] = ws + 2 * panel;
        b.Wt[1] = ws + 3 * panel;
        b.Rt = ws + 4 * panel;
        b.S = ws + 5 * panel;
        b.P = b.S + (size_t)PB * PB;
        b.nws = b.P + (size_t)PB * PB;
        b.ninfo = reinterpret_cast<int *>(b.nws + fused_ws_floats(PB));
    }
    // W = M + damping I (lower), info = 0
    for (int g0 = 0; g0 < total; g0 += kMaxProblems) {
        InvTable tab;
        tab.count = std::min(kMaxProblems, total - g0);
        tab.step = 0;
        int blocks = 0;
        for (int k = 0; k < tab.count; ++k) {
            const InvertJob &j = jobs[idx[g0 + k]];
            InvProb &p = tab.p[k];
            p.M = j.M; p.W = j.Minv; p.info = j.info; p.n = j.n; p.damping = j.damping; p.dptr = j.damping_dev;
            p.ldv = big[g0 + k].ldv; p.P = nullptr; p.Vt = nullptr; p.Wt = nullptr;
            p.gate = big[g0 + k].ninfo + 1;
            p.blk_start = blocks;
            blocks += (int)(((long)j.n * j.n + 4095) / 4096);
        }
        KFAC_LAUNCH(KFAC_K_INV_INIT, s, sweep_init_kernel, dim3(blocks), dim3(256), 0, tab);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    steps = total > 0 ? (jobs[idx[0]].n + PB - 1) / PB : 0;
    return hipSuccess;
}

hipError_t BlockedRun::copy_kernel(int what, int st, int act, hipStream_t s)
{
    const bool scatter = what == 1;
    const int p0 = st * PB;
    for (int g0 = 0; g0 < act; g0 += 32) {
        BlkTable tab;
        tab.count = std::min(32, act - g0);
        int blocks = 0;
        for (int k = 0; k < tab.count; ++k) {
            const InvertJob &j = jobs[idx[g0 + k]];
            BlkProb &p = tab.p[k];
            p.W = j.Minv; p.Vt = big[g0 + k].Vt[st & 1]; p.Wt = big[g0 + k].Wt[st & 1]; p.P = big[g0 + k].P;
            p.S = (refine && !scatter) ? big[g0 + k].S : nullptr;   // the condition test reads the matrix itself
            p.gate = refine ? big[g0 + k].ninfo + 1 : nullptr;
            p.gate_cond = (float)tuning().invert_refine_cond;
            p.info = j.info; p.ninfo = big[g0 + k].ninfo;
            p.n = j.n; p.ldv = big[g0 + k].ldv; p.p0 = p0; p.bs = std::min(PB, j.n - p0); p.pb = PB;
            p.blk_start = blocks;
            blocks += ((j.n + 31) / 32) * ((p.bs + 31) / 32);
        }
        if (what == 1) {
            KFAC_LAUNCH(KFAC_K_INV_PANEL, s, blk_scatter_kernel, dim3(blocks), dim3(256), 0, tab);
        } else if (what == 2) {
            int cb = 0;
            for (int k = 0; k < tab.count; ++k) {
                tab.p[k].blk_start = cb;
                cb += (tab.p[k].bs + 31) / 32;
            }
            KFAC_LAUNCH(KFAC_K_INV_PANEL, s, blk_cond_kernel, dim3(cb), dim3(256), 0, tab);
        } else {
            KFAC_LAUNCH(KFAC_K_INV_PANEL, s, blk_gather_kernel, dim3(blocks), dim3(256), 0, tab);
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// Update st restricted to the band of pivot block st + 1, leaving out the columns of pivot block st, which the
// scatter of step st owns.  part 0: the diagonal block of the band alone (all the nested inversion of step st + 1
// needs); part 1: the rest, i.e. the rows q0..q1 left of pivot block st and the columns q0..q1 below the diagonal
// block (what the gather of step st + 1 needs as well).
hipError_t BlockedRun::look(int st, int part, hipStream_t s)
{
    const int p0 = st * PB, q0 = p0 + PB;
    const int act = active(st + 1);
    gj.clear();
    for (int k = 0; k < act; ++k) {
        const InvertJob &j = jobs[idx[k]];
        const int q1 = std::min(q0 + PB, j.n);
        const Big &b = big[k];
        const float *Wt = b.Wt[st & 1], *Vt = b.Vt[st & 1];
        if (part == 0) {
            GemmJob d{};   // rows and columns q0..q1, on and below the diagonal
            d.A = Wt + q0; d.B = Vt + q0; d.C = j.Minv + (size_t)q0 * j.n + q0;
            d.M = q1 - q0; d.N = q1 - q0; d.K = PB; d.lda = b.ldv; d.ldb = b.ldv; d.ldc = j.n;
            d.mode = kSubRect; d.p0 = d.p1 = 0; d.doff = 0;
            gj.push_back(d);
            continue;
        }
        if (p0 > 0) {
            GemmJob r{};   // rows q0..q1, columns left of pivot block st
            r.A = Wt + q0; r.B = Vt; r.C = j.Minv + (size_t)q0 * j.n;
            r.M = q1 - q0; r.N = p0; r.K = PB; r.lda = b.ldv; r.ldb = b.ldv; r.ldc = j.n;
            r.mode = kSubRect; r.p0 = r.p1 = 0; r.doff = 1l << 30;
            gj.push_back(r);
        }
        if (j.n > q1) {
            GemmJob c{};   // rows below q1, columns q0..q1
            c.A = Wt + q1; c.B = Vt + q0; c.C = j.Minv + (size_t)q1 * j.n + q0;
            c.M = j.n - q1; c.N = q1 - q0; c.K = PB; c.lda = b.ldv; c.ldb = b.ldv; c.ldc = j.n;
            c.mode = kSubRect; c.p0 = c.p1 = 0; c.doff = 1l << 30;
            gj.push_back(c);
        }
    }
    return gj.empty() ? hipSuccess : gemm_launch(gj.data(), (int)gj.size(), s);
}

// The chain of step st.  The nested inversion of the pivot block and the test of its condition number go to
// stream sn, the gather, the panel product, its refinement and the scatter to stream sc: the gather needs the band
// of the pivot block (before_gather: null, or the event after which it is up to date) but not the inverse, so
// with two streams it runs beside the nested inversion, the longest link of the chain; ev_nest and ev_cond (used
// when the streams differ) order the panel product after the inversion and the refinement after the test.
hipError_t BlockedRun::chain(int st, hipStream_t sn, hipStream_t sc, hipEvent_t before_gather, hipEvent_t ev_nest,
                             hipEvent_t ev_cond)
{
    const bool two = sn != sc;
    const int p0 = st * PB;
    const int act = active(st);
    // 1. inverse of the pivot blocks (in their current, updated state) -> P
    nested.assign(act, InvertJob());
    nidx.resize(act);
    noffs.resize(act);
    for (int k = 0; k < act; ++k) {
        const InvertJob &j = jobs[idx[k]];
        InvertJob &q = nested[k];
        q.M = j.Minv + (size_t)p0 * j.n + p0;
        q.Minv = big[k].P;
        q.n = std::min(PB, j.n - p0);
        q.damping = 0.f;
        q.info = big[k].ninfo;
        q.ldm = j.n;
        q.ldo = PB;
        nidx[k] = k;
        noffs[k] = (size_t)(reinterpret_cast<char *>(big[k].nws) - static_cast<char *>(work));
    }
    // nested problems are grouped by order (all PB except possibly the last block of a matrix)
    std::stable_sort(nidx.begin(), nidx.end(), [&](int a, int b) { return nested[a].n > nested[b].n; });
    hipError_t e = fused_launch(nested.data(), nidx, noffs, work, dtab, sn);
    if (e != hipSuccess) return e;
    if (two && hipEventRecord(ev_nest, sn) != hipSuccess) return hipErrorUnknown;
    if (refine) {
        e = copy_kernel(2, st, act, sn);
        if (e != hipSuccess) return e;
        if (two && hipEventRecord(ev_cond, sn) != hipSuccess) return hipErrorUnknown;
    }
    hipStream_t s = sc;
    if (before_gather && hipStreamWaitEvent(s, before_gather, 0) != hipSuccess) return hipErrorUnknown;
    // 2. gather V, 3. W^T = P V^T, 4. scatter
    e = copy_kernel(0, st, act, s);
    if (e != hipSuccess) return e;
    if (two && hipStreamWaitEvent(s, ev_nest, 0) != hipSuccess) return hipErrorUnknown;
    gj.assign(act, GemmJob());
    for (int k = 0; k < act; ++k) {
        const InvertJob &j = jobs[idx[k]];
        const int bs = std::min(PB, j.n - p0);
        GemmJob &a = gj[k];
        a.A = big[k].P; a.B = big[k].Vt[st & 1]; a.C = big[k].Wt[st & 1];
        a.M = bs; a.N = j.n; a.K = bs; a.lda = PB; a.ldb = big[k].ldv; a.ldc = big[k].ldv;
        a.mode = kStore; a.p0 = a.p1 = 0;
        a.wide_tiles = tuning().invert_panel_split != 0;
    }
    e = gemm_launch(gj.data(), act, s);
    if (e != hipSuccess) return e;
    if (refine) {
        // One step of iterative refinement of the panel product.  W = V P with an explicitly inverted pivot block
        // S carries an error of eps |V| |P|, which for an ill-conditioned S is far above eps |W|; the residual
        // V - W S is made of small terms and comes out accurately, and W += (V - W S) P removes most of that error
        // (the inverse of a factor with condition number 1e5 goes from useless to the accuracy of an fp32
        // Cholesky inverse).  K-major: R^T = V^T - S W^T, W^T += P R^T.
        if (two && hipStreamWaitEvent(s, ev_cond, 0) != hipSuccess) return hipErrorUnknown;
        for (int pass = 0; pass < 2; ++pass) {
            for (int k = 0; k < act; ++k) {
                const InvertJob &j = jobs[idx[k]];
                const int bs = std::min(PB, j.n - p0);
                GemmJob &a = gj[k];
                a = GemmJob();
                a.A = pass == 0 ? big[k].S : big[k].P;
                a.B = pass == 0 ? big[k].Wt[st & 1] : big[k].Rt;
                a.C = pass == 0 ? big[k].Rt : big[k].Wt[st & 1];
                a.M = bs; a.N = j.n; a.K = bs; a.lda = PB; a.ldb = big[k].ldv; a.ldc = big[k].ldv;
                a.mode = pass == 0 ? kSubFrom : kAddRect; a.p0 = a.p1 = 0; a.doff = 1l << 30;
                if (pass == 0) { a.D = big[k].Vt[st & 1]; a.ldd = big[k].ldv; }
                a.gate = big[k].ninfo + 1;
                a.gate_cond = (float)tuning().invert_refine_cond;
            }
            e = gemm_launch(gj.data(), act, s);
            if (e != hipSuccess) return e;
        }
    }
    return copy_kernel(1, st, act, s);
}

hipError_t BlockedRun::bulk(int st, bool skip_next, hipStream_t s)
{
    const int p0 = st * PB;
    const int act = active(st);
    gj.clear();
    for (int k = 0; k < act; ++k) {
        const InvertJob &j = jobs[idx[k]];
        const int bs = std::min(PB, j.n - p0);
        const int p1 = std::min(j.n, p0 + bs + (skip_next ? PB : 0));
        if (p1 - p0 >= j.n) continue;      // nothing outside the bands
        GemmJob u{};
        u.A = big[k].Wt[st & 1]; u.B = big[k].Vt[st & 1]; u.C = j.Minv;
        u.M = j.n; u.N = j.n; u.K = bs; u.lda = big[k].ldv; u.ldb = big[k].ldv; u.ldc = j.n;
        u.mode = kSubLowerSkip; u.p0 = p0; u.p1 = p1;
        gj.push_back(u);
    }
    return gemm_launch(gj.data(), (int)gj.size(), s);
}

hipError_t BlockedRun::finish(hipStream_t s)
{
    // negate and mirror
    for (int g0 = 0; g0 < total; g0 += kMaxProblems) {
        InvTable tab;
        tab.count = std::min(kMaxProblems, total - g0);
        tab.step = 0;
        int blocks = 0;
        for (int k = 0; k < tab.count; ++k) {
            const InvertJob &j = jobs[idx[g0 + k]];
            InvProb &p = tab.p[k];
            p.M = j.M; p.W = j.Minv; p.info = j.info; p.n = j.n; p.damping = j.damping; p.dptr = j.damping_dev;
            p.ldv = big[g0 + k].ldv; p.P = nullptr; p.Vt = nullptr; p.Wt = nullptr;
            p.gate = nullptr;
            p.blk_start = blocks;
            const int nb32 = (j.n + 31) / 32;
            blocks += nb32 * (nb32 + 1) / 2;
        }
        KFAC_LAUNCH(KFAC_K_INV_FINISH, s, sweep_finish_kernel, dim3(blocks), dim3(256), 0, tab);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// Streams and events of the library, per device, created at the first call that needs them (default priority).
struct AuxStreams {
    static constexpr int kEvents = 64;
    hipStream_t chain = nullptr, nest = nullptr, side = nullptr;
    hipEvent_t fork = nullptr, side_done = nullptr;
    hipEvent_t ev_chain[kEvents] = {}, ev_bulk[kEvents] = {}, ev_look[kEvents] = {}, ev_nest[kEvents] = {},
               ev_cond[kEvents] = {};
    bool ok = false;
};

std::mutex &aux_mutex()
{
    static std::mutex m;
    return m;
}

// call with aux_mutex() held
AuxStreams *aux_streams()
{
    static AuxStreams per_dev[16];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) return nullptr;
    AuxStreams &a = per_dev[dev];
    if (a.ok) return &a;
    if (a.chain) return nullptr;     // an earlier attempt failed half way: stay on one stream
    bool good = hipStreamCreateWithFlags(&a.chain, hipStreamNonBlocking) == hipSuccess &&
                hipStreamCreateWithFlags(&a.nest, hipStreamNonBlocking) == hipSuccess &&
                hipStreamCreateWithFlags(&a.side, hipStreamNonBlocking) == hipSuccess &&
                hipEventCreateWithFlags(&a.fork, hipEventDisableTiming) == hipSuccess &&
                hipEventCreateWithFlags(&a.side_done, hipEventDisableTiming) == hipSuccess;
    for (int i = 0; good && i < AuxStreams::kEvents; ++i)
        good = hipEventCreateWithFlags(&a.ev_chain[i], hipEventDisableTiming) == hipSuccess &&
               hipEventCreateWithFlags(&a.ev_bulk[i], hipEventDisableTiming) == hipSuccess &&
               hipEventCreateWithFlags(&a.ev_look[i], hipEventDisableTiming) == hipSuccess &&
               hipEventCreateWithFlags(&a.ev_nest[i], hipEventDisableTiming) == hipSuccess &&
               hipEventCreateWithFlags(&a.ev_cond[i], hipEventDisableTiming) == hipSuccess;
    if (!good) {
        if (!a.chain) a.chain = reinterpret_cast<hipStream_t>(1);   // marks the failed attempt
        return nullptr;
    }
    a.ok = true;
    return &a;
}

// One stream: chain and bulk of every step in a row.
hipError_t blocked_serial(BlockedRun &run, hipStream_t s)
{
    hipError_t e = run.start(s);
    for (int st = 0; st < run.steps && e == hipSuccess; ++st) {
        e = run.chain(st, s, s, nullptr, nullptr, nullptr);
        if (e == hipSuccess) e = run.bulk(st, false, s);
    }
    return e == hipSuccess ? run.finish(s) : e;
}

// Look-ahead on three streams: updates on the caller's stream `s`, nested inversions on `aux->nest`, the rest of
// the chains on `aux->chain`.
//   update stream: wait chain(st); look(st, 0) [update st on the diagonal block of band st + 1]; record A;
//                  look(st, 1) [the rest of the band]; record B; bulk(st) without that band
//   nest stream:   wait A(st - 1); nested inversion of pivot block st; record N; condition test; record C
//   chain stream:  wait B(st - 1); gather; wait N; panel product; wait C; refinement; scatter; record
// The nested inversion, the longest link of the chain, only needs the diagonal block, a product of two tiles per
// matrix; it runs beside the rest of the band product, the gather and the bulk update.  Panels st (buffer st mod 2)
// are not overwritten before bulk(st) is done: the gather of step st + 2 waits for B(st + 1), which follows
// bulk(st) on its stream.  The inverse of pivot block st - 1 is not overwritten before scatter(st - 1) is done:
// A(st - 1) follows chain(st - 1).
hipError_t blocked_lookahead(BlockedRun &run, AuxStreams *aux, hipStream_t s)
{
    hipError_t e = run.start(s);
    if (e != hipSuccess) return e;
    hipStream_t c = aux->chain, nn = aux->nest;
    if (hipEventRecord(aux->fork, s) != hipSuccess || hipStreamWaitEvent(c, aux->fork, 0) != hipSuccess ||
        hipStreamWaitEvent(nn, aux->fork, 0) != hipSuccess)
        return hipErrorUnknown;
    bool joined = false;
    for (int st = 0; st < run.steps && e == hipSuccess; ++st) {
        joined = false;
        e = run.chain(st, nn, c, st > 0 ? aux->ev_bulk[st - 1] : nullptr, aux->ev_nest[st], aux->ev_cond[st]);
        if (e == hipSuccess && hipEventRecord(aux->ev_chain[st], c) != hipSuccess) e = hipErrorUnknown;
        if (e == hipSuccess && hipStreamWaitEvent(s, aux->ev_chain[st], 0) != hipSuccess) e = hipErrorUnknown;
        if (e != hipSuccess) break;
        joined = true;            // everything the other two streams hold so far is ordered before what follows on `s`
        const bool more = st + 1 < run.steps;
        if (more) {
            e = run.look(st, 0, s);
            if (e == hipSuccess && hipEventRecord(aux->ev_look[st], s) != hipSuccess) e = hipErrorUnknown;
            if (e == hipSuccess && hipStreamWaitEvent(nn, aux->ev_look[st], 0) != hipSuccess) e = hipErrorUnknown;
            if (e == hipSuccess) e = run.look(st, 1, s);
            if (e == hipSuccess && hipEventRecord(aux->ev_bulk[st], s) != hipSuccess) e = hipErrorUnknown;
        }
        if (e == hipSuccess) e = run.bulk(st, more, s);
    }
    if (!joined) {
        // after an error the caller's stream must still not run ahead of what the other two streams hold
        if (hipEventRecord(aux->ev_chain[0], c) == hipSuccess) (void)hipStreamWaitEvent(s, aux->ev_chain[0], 0);
        if (hipEventRecord(aux->ev_nest[0], nn) == hipSuccess) (void)hipStreamWaitEvent(s, aux->ev_nest[0], 0);
    }
    return e == hipSuccess ? run.finish(s) : e;
}

hipError_t blocked_launch(const InvertJob *jobs, const std::vector<int> &idx, const std::vector<size_t> &offs,
                          void *work, InvProbF *dtab, AuxStreams *aux, hipStream_t s)
{
    BlockedRun run;
    run.jobs = jobs; run.idx = idx; run.offs = &offs; run.work = work; run.dtab = dtab;
    if (!aux) return blocked_serial(run, s);
    return blocked_lookahead(run, aux, s);
}

// ---- orders 64 k + 1: the last row and column by bordering ---------------------------------
// A factor with a bias column has order 9 C + 1 or d + 1: with C or d a multiple of 64 the last pivot block of
// the sweep would be a single row, a whole step (and a block row of tiles in every other step) for a rank-1
// update.  Instead the sweep inverts the leading block, X = (M_11 + damping I)^-1, and with b the last row of M
// and c its corner,  y = X b,  s = c + damping - b^T y,
//     M^-1 = [ X + y y^T / s   -y / s ]
//            [   -y^T / s       1 / s ],
// which is the last pivot step of the same sweep (s is its pivot: not positive -> flagged as pivot n).
// On an ill-conditioned factor b^T y cancels c almost entirely and the error of the computed X makes s useless (a
// relative error of 0.2 to 1.5 in s at condition numbers of 1e5, emulated and measured), and at condition numbers of
// a few thousand the bordered inverse still carries ten times the error of X (3e-5 to 1e-4 against 4e-6 at order 577,
// condition 6e3, measured).  So the residual r = b - (M_11 + damping I) y is formed and
//     s = c + damping - b^T y - y^T r        (b^T M_11^-1 b to second order in the error of y)
//     y <- y + X r
// which brings the bordered inverse back to the accuracy of X itself: two more passes over an n x n matrix.  With
// invert_border_refine = 1 this is done only where the sweep found an ill-conditioned pivot block (the sticky flag
// of its gate): elsewhere the two extra kernels return at once.
struct BorderProb {
    const float *M;
    float *W;
    float *y;          // workspace: y, then r, then X r, each n - 1 floats rounded up to 64
    const int *sticky; // the sweep's flag: some pivot block of this matrix was ill-conditioned (null: refinement off)
    int always;        // refine whatever the flag says
    int *info;
    const float *dptr;
    float damping;
    int n, ldm, ldw;
    int blk_start;
    int rblk_start;    // first block of the residual kernel (one per 64 rows)
};

struct BorderTable {
    int count;
    BorderProb p[kMaxProblems];
};

constexpr int kBorderRows = 16;   // rows per workgroup: four per wavefront, their loads in flight together

__device__ __forceinline__ const BorderProb &border_locate(const BorderTable &tab, int &chunk)
{
    int pi = 0;
    while (pi + 1 < tab.count && (int)blockIdx.x >= tab.p[pi + 1].blk_start) ++pi;
    chunk = blockIdx.x - tab.p[pi].blk_start;
    return tab.p[pi];
}

__device__ __forceinline__ int border_vec_len(int n) { return (n - 1 + 63) / 64 * 64; }

// y = X b (second = 0) or z = X r for the refinement (second = 1: only where the sticky flag is set): a wavefront
// per row, lanes along the row
template <int second>
__global__ __launch_bounds__(256) void border_matvec_kernel(const BorderTable tab)
{
    __shared__ float bs[1280 + 64];
    int chunk;
    const BorderProb &pr = border_locate(tab, chunk);
    if (second && (!pr.sticky || (!pr.always && *pr.sticky == 0))) return;
    const int m = pr.n - 1, lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const float *vin = second ? pr.y + border_vec_len(pr.n) : pr.M + (long)m * pr.ldm;
    float *vout = second ? pr.y + 2 * border_vec_len(pr.n) : pr.y;
    for (int j = threadIdx.x; j < m; j += 256) bs[j] = vin[j];
    __syncthreads();
    // rows 4 w .. 4 w + 3 of the chunk: rows past the end repeat the last one and are not stored
    const int i0 = chunk * kBorderRows + 4 * w;
    const float *row[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) row[q] = pr.W + (long)min(i0 + q, m - 1) * pr.ldw;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    int j = lane;
    for (; j + 64 < m; j += 128) {              // two columns per lane and trip: eight loads in flight
        float v0[4], v1[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) { v0[q] = row[q][j]; v1[q] = row[q][j + 64]; }
        const float b0 = bs[j], b1 = bs[j + 64];
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[q] = __builtin_fmaf(v1[q], b1, __builtin_fmaf(v0[q], b0, acc[q]));
    }
    for (; j < m; j += 64) {
        const float b0 = bs[j];
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[q] = __builtin_fmaf(row[q][j], b0, acc[q]);
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        float a = acc[q];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) a += __shfl_xor(a, o);
        if (lane == 0 && i0 + q < m) vout[i0 + q] = a;
    }
}

// r = b - (M_11 + damping I) y from the lower triangle of M (the part the inversion may read), where the sticky flag
// is set.  One workgroup per 64 rows (the order of M_11 is a multiple of 64); the 64 x 64 tiles left of the diagonal
// are read as they are, those right of it from their mirror images, transposed through LDS.
__global__ __launch_bounds__(256) void border_resid_kernel(const BorderTable tab)
{
    __shared__ float L[64][65];
    __shared__ float ysh[1280 + 64];
    __shared__ float part[4][64];
    int pi = 0;
    while (pi + 1 < tab.count && (int)blockIdx.x >= tab.p[pi + 1].rblk_start) ++pi;
    const BorderProb &pr = tab.p[pi];
    if (!pr.sticky || (!pr.always && *pr.sticky == 0)) return;
    const int i0 = ((int)blockIdx.x - pr.rblk_start) * 64;
    const int m = pr.n - 1, t = threadIdx.x;
    for (int j = t; j < m; j += 256) ysh[j] = pr.y[j];
    const int r = t & 63, q = t >> 6;
    float acc = 0.f;
    for (int j0 = 0; j0 < m; j0 += 64) {
        const int R0 = j0 > i0 ? j0 : i0, C0 = j0 > i0 ? i0 : j0;
        __syncthreads();                       // the last tile has been consumed (and, first trip, ysh is complete)
        for (int e = t; e < 64 * 64; e += 256) {
            const int a = e >> 6, b = e & 63;
            L[a][b] = pr.M[(long)(R0 + a) * pr.ldm + C0 + b];
        }
        __syncthreads();
#pragma unroll 4
        for (int c = 16 * q; c < 16 * q + 16; ++c) {
            float v;
            if (j0 < i0) v = L[r][c];
            else if (j0 > i0) v = L[c][r];
            else v = c <= r ? L[r][c] : L[c][r];
            acc = __builtin_fmaf(v, ysh[j0 + c], acc);
        }
    }
    part[q][r] = acc;
    __syncthreads();
    if (t < 64) {
        const float damping = pr.dptr ? *pr.dptr : pr.damping;
        const float My = part[0][t] + part[1][t] + part[2][t] + part[3][t] + damping * ysh[i0 + t];
        pr.y[border_vec_len(pr.n) + i0 + t] = pr.M[(long)m * pr.ldm + i0 + t] - My;
    }
}

// the rank-1 update of X and the last row and column
__global__ __launch_bounds__(256) void border_update_kernel(const BorderTable tab)
{
    __shared__ float ys[1280 + 64];
    __shared__ float red[256];
    int chunk;
    const BorderProb &pr = border_locate(tab, chunk);
    const int m = pr.n - 1, t = threadIdx.x, lane = t & 63, w = t >> 6;
    const bool fix = pr.sticky && (pr.always || *pr.sticky != 0);          // uniform over the workgroup
    const float *rv = pr.y + border_vec_len(pr.n), *zv = rv + border_vec_len(pr.n);
    float part = 0.f;
    for (int j = t; j < m; j += 256) {
        const float yj = pr.y[j];
        float term = pr.M[(long)m * pr.ldm + j];
        if (fix) term += rv[j];                 // b^T y + y^T r
        ys[j] = fix ? yj + zv[j] : yj;
        part += term * yj;
    }
    red[t] = part;
    __syncthreads();
    for (int h = 128; h > 0; h >>= 1) {
        if (t < h) red[t] += red[t + h];
        __syncthreads();
    }
    const float damping = pr.dptr ? *pr.dptr : pr.damping;
    const float sp = pr.M[(long)m * pr.ldm + m] + damping - red[0];      // the same in every workgroup
    const float is = 1.0f / sp;
    if (chunk == 0) {
        if (t == 0) {
            if (!(sp > 0.f) && *pr.info == 0) *pr.info = pr.n;
            pr.W[(long)m * pr.ldw + m] = is;
        }
        for (int j = t; j < m; j += 256) pr.W[(long)m * pr.ldw + j] = -ys[j] * is;
    }
    // rows 4 w .. 4 w + 3 of the chunk (rows past the end repeat the last one and are not stored), three
    // column pieces per trip: twelve loads in flight before the first store
    const int i0 = chunk * kBorderRows + 4 * w;
    float *row[4];
    float yi[4];
    bool live[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        live[q] = i0 + q < m;
        const int i = min(i0 + q, m - 1);
        row[q] = pr.W + (long)i * pr.ldw;
        yi[q] = ys[i];
    }
    for (int j0 = lane; j0 < m; j0 += 192) {
        float v[3][4];
#pragma unroll
        for (int c = 0; c < 3; ++c)
#pragma unroll
            for (int q = 0; q < 4; ++q) v[c][q] = row[q][min(j0 + 64 * c, m - 1)];
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            const int j = j0 + 64 * c;
            if (j < m) {
                const float yj = ys[j];
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (live[q]) row[q][j] = v[c][q] + (yi[q] * yj) * is;   // y_i y_j first: the same value at (i, j) and (j, i)
            }
        }
    }
    if (lane == 0) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (live[q]) row[q][m] = -yi[q] * is;
    }
}

hipError_t border_launch(const InvertJob *jobs, const std::vector<int> &idx, const std::vector<float *> &ybuf,
                         const std::vector<const int *> &sticky, hipStream_t s)
{
    for (size_t g0 = 0; g0 < idx.size(); g0 += kMaxProblems) {
        BorderTable tab;
        tab.count = (int)std::min<size_t>(kMaxProblems, idx.size() - g0);
        int blocks = 0, rblocks = 0;
        for (int k = 0; k < tab.count; ++k) {
            const InvertJob &j = jobs[idx[g0 + k]];
            BorderProb &p = tab.p[k];
            p.M = j.M; p.W = j.Minv; p.y = ybuf[g0 + k]; p.info = j.info; p.dptr = j.damping_dev; p.damping = j.damping;
            p.sticky = tuning().invert_refine ? sticky[g0 + k] : nullptr;    // not maintained with the refinement off
            p.always = tuning().invert_border_refine >= 2;
            p.n = j.n;
            p.ldm = j.ldm > 0 ? j.ldm : j.n;
            p.ldw = j.ldo > 0 ? j.ldo : j.n;
            p.blk_start = blocks;
            blocks += (j.n - 1 + kBorderRows - 1) / kBorderRows;
            p.rblk_start = rblocks;
            rblocks += (j.n - 1) / 64;
        }
        KFAC_LAUNCH(KFAC_K_INV_FINISH, s, border_matvec_kernel<0>, dim3(blocks), dim3(256), 0, tab);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        if (tuning().invert_refine) {
            KFAC_LAUNCH(KFAC_K_INV_FINISH, s, border_resid_kernel, dim3(rblocks), dim3(256), 0, tab);
            e = hipGetLastError();
            if (e != hipSuccess) return e;
            KFAC_LAUNCH(KFAC_K_INV_FINISH, s, border_matvec_kernel<1>, dim3(blocks), dim3(256), 0, tab);
            e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
        KFAC_LAUNCH(KFAC_K_INV_FINISH, s, border_update_kernel, dim3(blocks), dim3(256), 0, tab);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// orders the sweep hands to the bordering: 64 k + 1 inside the range of the one-launch-per-step path
bool takes_border(int n)
{
    return tuning().invert_border && n > 64 && n % 64 == 1 && takes_fused(n - 1) && n - 1 <= 1280;   // 1280: the LDS vectors of the two kernels
}
size_t border_ws_floats(int n) { return takes_border(n) ? 3 * (size_t)((n - 1 + 63) / 64 * 64) : 0; }
}  // namespace

size_t invert_workspace_bytes(const InvertJob *jobs, int n)
{
    size_t total = table_bytes(n);
    for (int i = 0; i < n; ++i)
        total += align_up((job_ws_floats(jobs[i].n) + border_ws_floats(jobs[i].n)) * sizeof(float), 256);
    return total;
}

hipError_t invert_launch(const InvertJob *jobs_in, int n_all, void *work, size_t work_bytes, hipStream_t s)
{
    if (invert_workspace_bytes(jobs_in, n_all) > work_bytes) return hipErrorInvalidValue;
    std::vector<size_t> offs(n_all);
    size_t off = table_bytes(n_all);
    // bordered orders: the sweep sees the leading block (same storage, same pitches), the last row and column
    // follow at the end
    std::vector<InvertJob> inner(jobs_in, jobs_in + n_all);
    std::vector<int> bordered;
    std::vector<float *> ybuf;
    std::vector<const int *> sticky;
    for (int i = 0; i < n_all; ++i) {
        offs[i] = off;
        const int n = jobs_in[i].n;
        if (takes_border(n)) {
            inner[i].n = n - 1;
            inner[i].ldm = jobs_in[i].ldm > 0 ? jobs_in[i].ldm : n;
            inner[i].ldo = jobs_in[i].ldo > 0 ? jobs_in[i].ldo : n;
            bordered.push_back(i);
            ybuf.push_back(reinterpret_cast<float *>(static_cast<char *>(work) + off) + job_ws_floats(n));
            sticky.push_back(fused_gate_ptr(reinterpret_cast<float *>(static_cast<char *>(work) + off), n - 1) + 2);
        }
        off += align_up((job_ws_floats(n) + border_ws_floats(n)) * sizeof(float), 256);
    }
    const InvertJob *jobs = inner.data();
    // largest matrices first so that the matrices still active at a step form a prefix
    std::vector<int> large, fused;
    for (int i = 0; i < n_all; ++i) (takes_fused(jobs[i].n) ? fused : large).push_back(i);
    auto by_size = [&](int a, int b) { return jobs[a].n > jobs[b].n; };
    std::stable_sort(large.begin(), large.end(), by_size);
    std::stable_sort(fused.begin(), fused.end(), by_size);
    InvProbF *dtab = static_cast<InvProbF *>(work);
    // The library's own streams: the chains of the blocked sweep on one, and, when there are large matrices too,
    // the one-launch-per-step class on the other (independent matrices: the two classes run side by side).
    std::unique_lock<std::mutex> lock(aux_mutex(), std::defer_lock);
    AuxStreams *aux = nullptr;
    // (with the per-launch event timing on, everything stays on the caller's stream: an event pair around a kernel
    // that waits for another stream's kernel to leave the chip would time the wait as well)
    if (!large.empty() && tuning().invert_two_streams && !timing_active()) {
        lock.lock();       // the events are shared by all calls on a device: one call enqueues at a time
        aux = aux_streams();
        if (!aux) lock.unlock();
    }
    // With the library's streams the large matrices are enqueued first: their lock-step sequence of launches is the
    // critical path of the call, and the hundred-odd launches of the other class take the host half a millisecond
    // to enqueue, which would otherwise pass before the first kernel of the long sequence starts.
    hipStream_t fs = s;
    if (aux && !fused.empty()) {
        fs = aux->side;
        if (hipEventRecord(aux->fork, s) != hipSuccess || hipStreamWaitEvent(fs, aux->fork, 0) != hipSuccess)
            return hipErrorUnknown;
    }
    const bool side_open = fs != s;
    hipError_t e = hipSuccess;
    auto run_large = [&]() -> hipError_t {
        if (large.empty()) return hipSuccess;
        // the nested pivot-block inversions use the second half of the descriptor table
        const int steps = (jobs[large[0]].n + outer_block() - 1) / outer_block();
        return blocked_launch(jobs, large, offs, work, dtab + n_all, steps <= AuxStreams::kEvents ? aux : nullptr, s);
    };
    if (side_open) e = run_large();
    if (e == hipSuccess && !fused.empty()) e = fused_launch(jobs, fused, offs, work, dtab, fs);
    // bordered orders of the fused class finish on the same stream
    if (e == hipSuccess && !bordered.empty()) e = border_launch(jobs_in, bordered, ybuf, sticky, fs);
    if (side_open && hipEventRecord(aux->side_done, fs) != hipSuccess) return hipErrorUnknown;
    if (!side_open && e == hipSuccess) e = run_large();
    // always join the side stream, also after an error
    if (side_open && hipStreamWaitEvent(s, aux->side_done, 0) != hipSuccess) return hipErrorUnknown;
    return e;
}

// ---- factored Tikhonov damping (Eq. 12) ----------------------------------------------------
struct PiTable {
    int count;
    float gamma;
    float *lam;
    const float *A[kMaxProblems];
    const float *G[kMaxProblems];
    int dA[kMaxProblems], dG[kMaxProblems];
    int first;
};

// One workgroup per layer: traces of A and G (fixed-order tree sums), pi = sqrt((tr A / d_A) / (tr G / d_G)),
// lam[2l] = pi sqrt(gamma), lam[2l+1] = sqrt(gamma) / pi.  A trace that is not positive leaves pi = 1.
__global__ __launch_bounds__(256) void pi_damping_kernel(const PiTable tab)
{
    __shared__ float red[2][256];
    const int l = blockIdx.x, t = threadIdx.x;
    const float *A = tab.A[l], *G = tab.G[l];
    const int dA = tab.dA[l], dG = tab.dG[l];
    float sa = 0.f, sg = 0.f;
    for (int i = t; i < dA; i += 256) sa += A[(long)i * dA + i];
    for (int i = t; i < dG; i += 256) sg += G[(long)i * dG + i];
    red[0][t] = sa;
    red[1][t] = sg;
    __syncthreads();
    for (int h = 128; h > 0; h >>= 1) {
        if (t < h) {
            red[0][t] += red[0][t + h];
            red[1][t] += red[1][t + h];
        }
        __syncthreads();
    }
    if (t == 0) {
        const float trA = red[0][0], trG = red[1][0];
        float pi = 1.f;
        if (trA > 0.f && trG > 0.f) pi = sqrtf((trA / (float)dA) / (trG / (float)dG));
        const float sq = sqrtf(tab.gamma);
        tab.lam[2 * (tab.first + l)] = pi * sq;
        tab.lam[2 * (tab.first + l) + 1] = sq / pi;
    }
}

hipError_t pi_damping_launch(const float *const *A, const float *const *G, const int *dA, const int *dG, int n,
                             float gamma, float *lam, hipStream_t s)
{
    for (int g0 = 0; g0 < n; g0 += kMaxProblems) {
        PiTable tab;
        tab.count = std::min(kMaxProblems, n - g0);
        tab.gamma = gamma;
        tab.lam = lam;
        tab.first = g0;
        for (int k = 0; k < tab.count; ++k) {
            tab.A[k] = A[g0 + k]; tab.G[k] = G[g0 + k];
            tab.dA[k] = dA[g0 + k]; tab.dG[k] = dG[g0 + k];
        }
        KFAC_LAUNCH(KFAC_K_INV_INIT, s, pi_damping_kernel, dim3(tab.count), dim3(256), 0, tab);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace kfac

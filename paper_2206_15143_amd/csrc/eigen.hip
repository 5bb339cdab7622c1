// Batched symmetric eigen-decomposition of the Kronecker factors, M = Q diag(v) Q^T: the Q_A, v_A,
// Q_G, v_G that the eigen-decomposition variant of the preconditioner uses (Eq. 13 of the DP-KFAC
// paper, section 5.2).
//
// Method: one-sided block Jacobi on rows.  The working pair (W, V) starts as (M, I) and every step
// applies the same orthogonal transform to both from the left, so W = V M holds throughout; when the
// rows of W are mutually orthogonal, row i of V is an eigenvector and <v_i, w_i> its eigenvalue.
// Rows are grouped into blocks of 16.  One round pairs all blocks off (round-robin tournament: every
// two blocks meet once per sweep) and is ONE launch with one workgroup per pair of every matrix:
//   1. the 32 x 32 Gram matrix S = X X^T of the pair's 32 rows of W on the MFMA units (K = n);
//   2. one sweep of two-sided cyclic Jacobi over S in LDS (16 disjoint rotations per inner round,
//      31 inner rounds) gives the 32 x 32 orthogonal R (more inner sweeps per round did not save
//      outer sweeps);
//   3. the rows of W and of V are replaced by R^T X on the MFMA units.
// A pair whose Gram matrix is already diagonal to rounding does nothing; a matrix none of whose
// pairs did anything for a whole sweep has converged and its workgroups return at once (the
// per-matrix round stamp lives in device memory, so the host never synchronises).  The launch
// sequence has a fixed length (a sweep budget); `info` reports a matrix that used it up.
// Rows past n (padding of the last block, and the bye of an odd number of blocks) are zero rows:
// their Gram entries vanish and no rotation touches them.
#include "common.hpp"

#include <algorithm>
#include <cmath>
#include <vector>

namespace kfac {

constexpr int EB = 16;              // rows per block (32 halves the rounds and the traffic, but the in-LDS sweep over
                                    // the then 64 x 64 Gram matrix costs 8x more and the rounds become slower: measured)
constexpr int kMaxEigClasses = 16;  // distinct orders per launch sequence

struct EigProb {                    // init / final kernels: one entry per matrix
    const float *M;
    float *Q;
    float *v;
    int *info;
    float *Wt, *Vt;
    float *scale;                   // [nb * EB] reciprocal row norms of V (final pass)
    int *stamp;
    int n, ld, nb;
    int blk_start;
    int rounds_total, m;
};

struct EigTable {
    int count;
    EigProb p[kMaxProblems];
};

struct EigClass {                   // round kernel: matrices of one order, stored back to back
    float *Wt, *Vt;                 // first matrix; the next ones follow at `stride` floats
    int *stamp;                     // per matrix: 1 + index of the last round in which a pair rotated
    long stride;
    int n, ld, nb, m;               // order, row pitch, blocks, blocks rounded up to even
    int count;
    int blk_start;
    float tol;
};

struct EigSeq {
    int nclass;
    int t;                          // global round index
    int inner_sweeps;
    EigClass c[kMaxEigClasses];
};

__global__ __launch_bounds__(256) void eig_init_kernel(const EigTable tab)
{
    int pi = 0;
    while (pi + 1 < tab.count && (int)blockIdx.x >= tab.p[pi + 1].blk_start) ++pi;
    const EigProb &pr = tab.p[pi];
    const long total = (long)pr.nb * EB * pr.ld;
    const long e0 = ((long)(blockIdx.x - pr.blk_start) * 256 + threadIdx.x) * 4;
    if (blockIdx.x == pr.blk_start && threadIdx.x == 0) {
        *pr.stamp = 0;
        *pr.info = 0;
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const long e = e0 + q;
        if (e >= total) return;
        const int i = (int)(e / pr.ld), j = (int)(e - (long)i * pr.ld);
        float w = 0.f;
        if (i < pr.n && j < pr.n) w = pr.M[(long)max(i, j) * pr.n + min(i, j)];   // lower triangle is authoritative
        pr.Wt[e] = w;
        pr.Vt[e] = (i == j && i < pr.n) ? 1.f : 0.f;
    }
}

// Pair k of round r of a round-robin tournament over m (even) players.
__device__ __forceinline__ void rr_pair(int m, int r, int k, int &a, int &b)
{
    if (k == 0) {
        a = m - 1;
        b = r;
    } else {
        a = (r + k) % (m - 1);
        b = (r - k + (m - 1)) % (m - 1);
    }
}

__global__ __launch_bounds__(256) void eig_round_kernel(const EigSeq q)
{
    constexpr int PR = 2 * EB;               // rows of a pair of blocks
    constexpr int NG = PR / 16;              // 16-row groups of a pair
    __shared__ float S[PR][PR + 1];
    __shared__ float R[PR][PR + 1];

    int ci = 0;
    while (ci + 1 < q.nclass && (int)blockIdx.x >= q.c[ci + 1].blk_start) ++ci;
    const EigClass &c = q.c[ci];
    const int local = blockIdx.x - c.blk_start;
    const int half = c.m / 2;
    const int mat = local / half, pk = local - mat * half;
    if (mat >= c.count) return;
    // converged: a whole sweep (m - 1 rounds) without a rotation
    const int stamp = c.stamp[mat];
    if (q.t - stamp >= c.m - 1) return;

    int I, J;
    rr_pair(c.m, q.t % (c.m - 1), pk, I, J);
    if (I > J) { const int t = I; I = J; J = t; }
    if (I >= c.nb) return;                      // cannot happen for m <= nb + 1; keeps the indexing safe
    const bool hasJ = J < c.nb;                 // the bye block of an odd count is all zero rows
    const int tid = threadIdx.x;
    const int lane = tid & 63, w = tid >> 6;
    const int r = lane & 15, kk = lane >> 4;
    const long ld = c.ld;
    float *Wt = c.Wt + (long)mat * c.stride;
    float *Vt = c.Vt + (long)mat * c.stride;
    // row of the pair -> row of the matrix: the first EB rows are block I, the rest block J
    auto pair_row = [&](int pr) { return pr < EB ? I * EB + pr : J * EB + (pr - EB); };

    // ---- 1. Gram matrix of the pair's rows: wavefront w takes the 16-column chunks w, w + 4, ...;
    //         16 x 16 tiles of the lower triangle of the grid of row groups ----
    {
        floatx4 acc[NG * (NG + 1) / 2];
#pragma unroll
        for (int t = 0; t < NG * (NG + 1) / 2; ++t) acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
        const float *rowp[NG];
#pragma unroll
        for (int g = 0; g < NG; ++g) rowp[g] = Wt + (long)pair_row(16 * g + r) * ld + 4 * kk;
#pragma unroll 2
        for (int k0 = 16 * w; k0 < c.ld; k0 += 64) {
            floatx4 x[NG];
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                x[g] = floatx4{0.f, 0.f, 0.f, 0.f};
                if (g < NG / 2 || hasJ) x[g] = *reinterpret_cast<const floatx4 *>(rowp[g] + k0);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                int t = 0;
#pragma unroll
                for (int gi = 0; gi < NG; ++gi)
#pragma unroll
                    for (int gj = 0; gj <= gi; ++gj, ++t)
                        acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[gi][e], x[gj][e], acc[t], 0, 0, 0);
            }
        }
        // the four wavefronts add their parts one after the other: a fixed order, no scratch tiles
#pragma unroll 1
        for (int ww = 0; ww < 4; ++ww) {
            if (w == ww) {
                int t = 0;
#pragma unroll
                for (int gi = 0; gi < NG; ++gi)
#pragma unroll
                    for (int gj = 0; gj <= gi; ++gj, ++t)
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            const int row = 16 * gi + 4 * kk + v, col = 16 * gj + r;
                            const float val = (ww == 0 ? 0.f : S[row][col]) + acc[t][v];
                            S[row][col] = val;
                        }
            }
            __syncthreads();
        }
    }
    // mirror the strictly lower tiles, R = I
    for (int e = tid; e < PR * PR; e += 256) {
        const int row = e / PR, col = e - row * PR;
        if ((col >> 4) > (row >> 4)) S[row][col] = S[col][row];
        R[row][col] = (row == col) ? 1.f : 0.f;
    }
    __syncthreads();

    // ---- 2. two-sided cyclic Jacobi on S; thread (pair = tid % EB, part = tid / EB) moves PE elements ----
    const int pr_ = tid & (PR / 2 - 1), part = tid / (PR / 2);
    constexpr int PE = PR / (256 / (PR / 2));   // elements per thread and phase
    bool active = false;
    for (int sw = 0; sw < q.inner_sweeps; ++sw) {
        bool any = false;
#pragma unroll 1
        for (int rd = 0; rd < PR - 1; ++rd) {
            int p, qq;
            rr_pair(PR, rd, pr_, p, qq);
            if (p > qq) { const int t = p; p = qq; qq = t; }
            const float app = S[p][p], aqq = S[qq][qq], apq = S[p][qq];
            float cs = 1.f, sn = 0.f;
            const bool rot = fabsf(apq) > c.tol * __builtin_amdgcn_sqrtf(fabsf(app * aqq)) && apq != 0.f;
            if (rot) {
                // tangent of the rotation that annihilates S[p][q]: the smaller root of t^2 + 2 tau t - 1 = 0.
                // Hardware reciprocal / square root (1 ulp): the angle only has to be nearly right, and
                // cs^2 + sn^2 = 1 holds to rounding whatever tt is.
                const float tau = (aqq - app) * __builtin_amdgcn_rcpf(2.f * apq);
                const float tt = (tau >= 0.f ? 1.f : -1.f) *
                                 __builtin_amdgcn_rcpf(fabsf(tau) + __builtin_amdgcn_sqrtf(1.f + tau * tau));
                cs = __builtin_amdgcn_rsqf(1.f + tt * tt);
                sn = tt * cs;
            }
            any = any || rot;
            __syncthreads();                    // every thread has read its pivots before anything moves
            // columns p, q of S and of R:  S <- S J,  R <- R J   (all loads first: they pipeline)
            {
                float sp[PE], sq[PE], rp[PE], rq[PE];
#pragma unroll
                for (int e = 0; e < PE; ++e) {
                    const int i = part * PE + e;
                    sp[e] = S[i][p]; sq[e] = S[i][qq];
                    rp[e] = R[i][p]; rq[e] = R[i][qq];
                }
#pragma unroll
                for (int e = 0; e < PE; ++e) {
                    const int i = part * PE + e;
                    S[i][p] = cs * sp[e] - sn * sq[e];
                    S[i][qq] = sn * sp[e] + cs * sq[e];
                    R[i][p] = cs * rp[e] - sn * rq[e];
                    R[i][qq] = sn * rp[e] + cs * rq[e];
                }
            }
            __syncthreads();
            // rows p, q of S:  S <- J^T S
            {
                float sp[PE], sq[PE];
#pragma unroll
                for (int e = 0; e < PE; ++e) {
                    const int j = part * PE + e;
                    sp[e] = S[p][j]; sq[e] = S[qq][j];
                }
#pragma unroll
                for (int e = 0; e < PE; ++e) {
                    const int j = part * PE + e;
                    S[p][j] = cs * sp[e] - sn * sq[e];
                    S[qq][j] = sn * sp[e] + cs * sq[e];
                }
            }
            __syncthreads();
        }
        if (!__syncthreads_or(any ? 1 : 0)) break;
        active = true;
    }
    if (!active) return;                        // R is the identity: nothing to apply
    if (tid == 0) atomicMax(c.stamp + mat, q.t + 1);

    // ---- 3. rows <- R^T rows, for W and V; wavefront w takes the 32-column groups w, w + 4, ... ----
    float a[NG][PR / 4];
#pragma unroll
    for (int it = 0; it < NG; ++it)
#pragma unroll
        for (int s = 0; s < PR / 4; ++s) a[it][s] = R[4 * s + kk][16 * it + r];
#pragma unroll 1
    for (int which = 0; which < 2; ++which) {
        float *X = which == 0 ? Wt : Vt;
        // two 16-column chunks at a time: 32 loads in flight, then the products, then the stores
        for (int k0 = 32 * w; k0 < c.ld; k0 += 128) {
            float b[2][PR / 4];
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                const int kc = k0 + 16 * g + r;
                const bool in = k0 + 16 * g < c.ld;
#pragma unroll
                for (int s = 0; s < PR / 4; ++s) {
                    const int pr = 4 * s + kk;
                    b[g][s] = (in && (pr < EB || hasJ)) ? X[(long)pair_row(pr) * ld + kc] : 0.f;
                }
            }
            floatx4 d[2][NG];
#pragma unroll
            for (int g = 0; g < 2; ++g)
#pragma unroll
                for (int it = 0; it < NG; ++it) {
                    d[g][it] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int s = 0; s < PR / 4; ++s)
                        d[g][it] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[it][s], b[g][s], d[g][it], 0, 0, 0);
                }
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                if (k0 + 16 * g >= c.ld) break;
                const int kc = k0 + 16 * g + r;
#pragma unroll
                for (int it = 0; it < NG; ++it)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int pr = 16 * it + 4 * kk + v;
                        if (pr < EB || hasJ) X[(long)pair_row(pr) * ld + kc] = d[g][it][v];
                    }
            }
        }
    }
}

// Row norms and eigenvalues.  A rotation whose tangent t is below sqrt(eps) has cosine 1 in fp32, so it
// scales its two rows by sqrt(1 + t^2) instead of leaving their norms alone; over the thousands of small
// rotations near convergence the rows of V (and of W, which sees the same transforms) grow by ~1e-4, all
// by nearly the same factor, while staying orthogonal.  Hence v[i] = <V_i, W_i> / |V_i|^2 and the
// eigenvector is V_i / |V_i|; scale[i] = 1 / |V_i|.  32 rows per workgroup, 8 lanes per row.
// info = 1 if the sweep budget ran out before a quiet sweep.
__global__ __launch_bounds__(256) void eig_values_kernel(const EigTable tab)
{
    int pi = 0;
    while (pi + 1 < tab.count && (int)blockIdx.x >= tab.p[pi + 1].blk_start) ++pi;
    const EigProb &pr = tab.p[pi];
    const int local = blockIdx.x - pr.blk_start;
    if (local == 0 && threadIdx.x == 0) *pr.info = (pr.rounds_total - *pr.stamp >= pr.m - 1) ? 0 : 1;
    const int row = local * 32 + (threadIdx.x >> 3), l8 = threadIdx.x & 7;
    float vw = 0.f, vv = 0.f;
    if (row < pr.n) {
        const float *vr = pr.Vt + (long)row * pr.ld, *wr = pr.Wt + (long)row * pr.ld;
        for (int j = l8; j < pr.n; j += 8) {
            vw += vr[j] * wr[j];
            vv += vr[j] * vr[j];
        }
    }
#pragma unroll
    for (int h = 1; h < 8; h <<= 1) {
        vw += __shfl_xor(vw, h);
        vv += __shfl_xor(vv, h);
    }
    if (row < pr.n && l8 == 0) {
        pr.v[row] = vw / vv;
        pr.scale[row] = 1.f / sqrtf(vv);
    }
}

// Q[j][i] = V[i][j] * scale[i] (eigenvectors in the columns of Q).  One workgroup per 32 x 32 tile of V.
__global__ __launch_bounds__(256) void eig_final_kernel(const EigTable tab)
{
    __shared__ float t[32][33];
    int pi = 0;
    while (pi + 1 < tab.count && (int)blockIdx.x >= tab.p[pi + 1].blk_start) ++pi;
    const EigProb &pr = tab.p[pi];
    const int local = blockIdx.x - pr.blk_start;
    const int nt = (pr.n + 31) / 32;
    const int ti = local / nt, tj = local - ti * nt;       // tile (rows ti of V, columns tj)
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
        const int i = ti * 32 + ty + 8 * rr, j = tj * 32 + tx;
        t[ty + 8 * rr][tx] = (i < pr.n && j < pr.n) ? pr.Vt[(long)i * pr.ld + j] * pr.scale[i] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
        const int j = tj * 32 + ty + 8 * rr, i = ti * 32 + tx;
        if (i < pr.n && j < pr.n) pr.Q[(long)j * pr.n + i] = t[tx][ty + 8 * rr];
    }
}

struct TrProb {
    const float *src;
    float *dst;
    int n;
    int blk_start;
};

struct TrTable {
    int count;
    TrProb p[kMaxProblems];
};

// dst = src^T for square matrices, 32 x 32 tiles through LDS.
__global__ __launch_bounds__(256) void transpose_kernel(const TrTable tab)
{
    __shared__ float t[32][33];
    int pi = 0;
    while (pi + 1 < tab.count && (int)blockIdx.x >= tab.p[pi + 1].blk_start) ++pi;
    const TrProb &pr = tab.p[pi];
    const int local = blockIdx.x - pr.blk_start;
    const int nt = (pr.n + 31) / 32;
    const int ti = local / nt, tj = local - ti * nt;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
        const int i = ti * 32 + ty + 8 * rr, j = tj * 32 + tx;
        t[ty + 8 * rr][tx] = (i < pr.n && j < pr.n) ? pr.src[(long)i * pr.n + j] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
        const int j = tj * 32 + ty + 8 * rr, i = ti * 32 + tx;
        if (i < pr.n && j < pr.n) pr.dst[(long)j * pr.n + i] = t[tx][ty + 8 * rr];
    }
}

hipError_t transpose_launch(const float *const *src, float *const *dst, const int *n, int count, hipStream_t s)
{
    for (int g0 = 0; g0 < count; g0 += kMaxProblems) {
        TrTable tab;
        tab.count = std::min(kMaxProblems, count - g0);
        int blocks = 0;
        for (int k = 0; k < tab.count; ++k) {
            TrProb &p = tab.p[k];
            p.src = src[g0 + k]; p.dst = dst[g0 + k]; p.n = n[g0 + k];
            p.blk_start = blocks;
            const int nt = (p.n + 31) / 32;
            blocks += nt * nt;
        }
        KFAC_LAUNCH(KFAC_K_EIG_FINAL, s, transpose_kernel, dim3(blocks), dim3(256), 0, tab);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

namespace {

struct EigLayout {
    int ld, nb, m;
    size_t floats;      // W or V of one matrix
    size_t total;       // floats of one matrix in the workspace
};

EigLayout eig_layout(int n)
{
    EigLayout L;
    L.ld = (n + 15) / 16 * 16;
    L.nb = (n + EB - 1) / EB;
    L.m = L.nb + (L.nb & 1);
    if (L.m < 2) L.m = 2;
    L.floats = (size_t)L.nb * EB * L.ld;
    L.total = 2 * L.floats + (size_t)L.nb * EB;   // W, V, scale
    return L;
}

}  // namespace

size_t eigen_workspace_bytes(const EigenJob *jobs, int n)
{
    size_t total = 0;
    for (int i = 0; i < n; ++i) total += align_up(eig_layout(jobs[i].n).total * sizeof(float), 256);
    return total + align_up((size_t)n * sizeof(int), 256);
}

hipError_t eigen_launch(const EigenJob *jobs, int n, void *work, size_t work_bytes, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    if (eigen_workspace_bytes(jobs, n) > work_bytes) return hipErrorInvalidValue;
    // matrices of one order back to back (largest first), W and V of a matrix adjacent
    std::vector<int> order(n);
    for (int i = 0; i < n; ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return jobs[a].n > jobs[b].n; });
    int *stamps = reinterpret_cast<int *>(work);
    char *base = static_cast<char *>(work) + align_up((size_t)n * sizeof(int), 256);
    std::vector<EigProb> probs(n);
    size_t off = 0;
    const int sweeps = (int)std::max(1l, tuning().eigen_max_sweeps);
    for (int k = 0; k < n; ++k) {
        const EigenJob &j = jobs[order[k]];
        const EigLayout L = eig_layout(j.n);
        EigProb &p = probs[k];
        p.M = j.M; p.Q = j.Q; p.v = j.v; p.info = j.info;
        p.Wt = reinterpret_cast<float *>(base + off);
        p.Vt = p.Wt + L.floats;
        p.scale = p.Vt + L.floats;
        off += align_up(L.total * sizeof(float), 256);
        p.stamp = stamps + k;
        p.n = j.n; p.ld = L.ld; p.nb = L.nb; p.m = L.m;
        p.rounds_total = 0;
    }
    // launch sequences of at most kMaxEigClasses distinct orders
    int k0 = 0;
    while (k0 < n) {
        EigSeq q;
        q.nclass = 0;
        q.inner_sweeps = (int)std::max(1l, tuning().eigen_inner_sweeps);
        int blocks = 0, k1 = k0, mmax = 2;
        while (k1 < n) {
            const int nn = probs[k1].n;
            int k2 = k1;
            while (k2 < n && probs[k2].n == nn) ++k2;
            if (q.nclass == kMaxEigClasses) break;
            EigClass &c = q.c[q.nclass++];
            const EigLayout L = eig_layout(nn);
            c.Wt = probs[k1].Wt; c.Vt = probs[k1].Vt; c.stamp = probs[k1].stamp;
            c.stride = (long)(align_up(L.total * sizeof(float), 256) / sizeof(float));
            c.n = nn; c.ld = L.ld; c.nb = L.nb; c.m = L.m;
            c.count = k2 - k1;
            c.blk_start = blocks;
            c.tol = std::max(5e-7f, 1.2e-7f * std::sqrt((float)nn));
            blocks += c.count * (L.m / 2);
            mmax = std::max(mmax, L.m);
            k1 = k2;
        }
        const int rounds = sweeps * (mmax - 1);
        for (int k = k0; k < k1; ++k) probs[k].rounds_total = rounds;
        // init
        for (int g0 = k0; g0 < k1; g0 += kMaxProblems) {
            EigTable tab;
            tab.count = std::min(kMaxProblems, k1 - g0);
            int ib = 0;
            for (int k = 0; k < tab.count; ++k) {
                tab.p[k] = probs[g0 + k];
                tab.p[k].blk_start = ib;
                ib += (int)(((long)tab.p[k].nb * EB * tab.p[k].ld + 1023) / 1024);
            }
            KFAC_LAUNCH(KFAC_K_EIG_INIT, s, eig_init_kernel, dim3(ib), dim3(256), 0, tab);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
        for (int t = 0; t < rounds; ++t) {
            q.t = t;
            KFAC_LAUNCH(KFAC_K_EIG_ROUND, s, eig_round_kernel, dim3(blocks), dim3(256), 0, q);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
        for (int g0 = k0; g0 < k1; g0 += kMaxProblems) {
            EigTable tab;
            tab.count = std::min(kMaxProblems, k1 - g0);
            int vb = 0;
            for (int k = 0; k < tab.count; ++k) {
                tab.p[k] = probs[g0 + k];
                tab.p[k].blk_start = vb;
                vb += (tab.p[k].n + 31) / 32;
            }
            KFAC_LAUNCH(KFAC_K_EIG_FINAL, s, eig_values_kernel, dim3(vb), dim3(256), 0, tab);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
            int fb = 0;
            for (int k = 0; k < tab.count; ++k) {
                tab.p[k].blk_start = fb;
                const int nt = (tab.p[k].n + 31) / 32;
                fb += nt * nt;
            }
            KFAC_LAUNCH(KFAC_K_EIG_FINAL, s, eig_final_kernel, dim3(fb), dim3(256), 0, tab);
            e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
        k0 = k1;
    }
    return hipSuccess;
}

}  // namespace kfac

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
// Per step: sweep_pivot_kernel (one workgroup per matrix inverts the nb x nb
// pivot block in LDS), sweep_panel_kernel (V = old panel, W = V P, both stored
// K-major for the MFMA update; new panel written in place), then the rank-nb
// update through the A^T B GEMM (gemm.hip, mode kSubLowerSkip).
#include "invert_fused.hpp"

#include <algorithm>
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
    if (local == 0 && threadIdx.x == 0) *pr.info = 0;
    for (long e = (long)local * 4096 + threadIdx.x; e < lmin(total, (long)(local + 1) * 4096); e += 256) {
        const int i = (int)(e / pr.n), j = (int)(e - (long)i * pr.n);
        if (j <= i) pr.W[e] = pr.M[e] + (i == j ? pr.damping : 0.f);
    }
}

// Inverts the pivot block of step `tab.step` by an unblocked sweep.  The 64 x 64 block lives in
// registers (thread (i, jq) holds S[i][jq + 4m], m = 0..15); per elimination step only the pivot
// row and column travel through LDS (double buffered), so a step costs one barrier, 17 LDS reads
// and 16 FMAs per thread.
__global__ __launch_bounds__(256) void sweep_pivot_kernel(const InvTable tab)
{
    __shared__ float colb[2][NB];
    __shared__ float rowb[2][NB];
    const InvProb &pr = tab.p[blockIdx.x];
    const int p0 = tab.step * NB;
    if (p0 >= pr.n) return;
    const int bs = min(NB, pr.n - p0);
    const int tid = threadIdx.x;
    const int i = tid >> 2, jq = tid & 3;
    const long n = pr.n;

    float s[NB / 4];
#pragma unroll
    for (int m = 0; m < NB / 4; ++m) {
        const int j = jq + 4 * m;
        float v = (i == j) ? 1.f : 0.f;      // identity padding keeps the tail block well defined
        if (i < bs && j < bs) v = (j <= i) ? pr.W[(p0 + i) * n + p0 + j] : pr.W[(p0 + j) * n + p0 + i];
        s[m] = v;
    }
    if (jq == 0) colb[0][i] = s[0];
    if (i == 0) {
#pragma unroll
        for (int m = 0; m < NB / 4; ++m) rowb[0][jq + 4 * m] = s[m];
    }
    __syncthreads();

    int fail = 0;
    for (int k = 0; k < bs; ++k) {
        const int b = k & 1;
        const float p = rowb[b][k];
        if (!(p > 0.f) && fail == 0) fail = p0 + k + 1;
        const float ip = __builtin_amdgcn_rcpf(p);   // 1 ulp reciprocal: far below the fp32 error of the sweep
        const float ci = colb[b][i];
        const bool prow = (i == k);
        const float cip = ci * ip;
        // selects instead of branches: the four cases (pivot, pivot row, pivot column, rest) differ per element
#pragma unroll
        for (int m = 0; m < NB / 4; ++m) {
            const int j = jq + 4 * m;
            const float rk = rowb[b][j];
            const bool pcol = (j == k);
            const float rest = s[m] - (ci * rk) * ip;
            const float on_row = pcol ? -ip : rk * ip;
            const float off_row = pcol ? cip : rest;
            s[m] = prow ? on_row : off_row;
        }
        // publish the next pivot column and row
        const int kn = k + 1;
        float cv = s[0];
#pragma unroll
        for (int m = 1; m < NB / 4; ++m) cv = (m == (kn >> 2)) ? s[m] : cv;
        if (jq == (kn & 3)) colb[b ^ 1][i] = cv;
        if (i == kn) {
#pragma unroll
            for (int m = 0; m < NB / 4; ++m) rowb[b ^ 1][jq + 4 * m] = s[m];
        }
        __syncthreads();
    }
#pragma unroll
    for (int m = 0; m < NB / 4; ++m) {
        const int j = jq + 4 * m;
        const bool in = (i < bs && j < bs);
        pr.P[i * NB + j] = in ? -s[m] : 0.f;
        if (in && j <= i) pr.W[(p0 + i) * n + p0 + j] = s[m];
    }
    if (fail != 0 && tid == 0 && *pr.info == 0) *pr.info = fail;
}

// One workgroup per 64 rows of the panel of step `tab.step`: V = old panel rows (transposed to
// K-major), W^T = P V^T on the MFMA units (P is symmetric, so it is its own K-major operand), then
// V^T and W^T go to the workspace for the rank-64 update and W replaces the panel in place.
__global__ __launch_bounds__(256) void sweep_panel_kernel(const InvTable tab)
{
    typedef Tile<2, 2> T;                          // 64 x 64 output, four waves of 32 x 32
    constexpr int PITCH = T::PITCH;                // 80: conflict-free K-major operand reads
    __shared__ float Ps[NB * PITCH];               // [k][m]
    __shared__ float Vs[NB * PITCH];               // [k][i]
    int pi = 0;
    while (pi + 1 < tab.count && (int)blockIdx.x >= tab.p[pi + 1].blk_start) ++pi;
    const InvProb &pr = tab.p[pi];
    const int chunk = blockIdx.x - pr.blk_start;
    const int p0 = tab.step * NB;
    if (p0 >= pr.n) return;
    const int bs = min(NB, pr.n - p0);
    const int i0 = chunk * NB;
    const int tid = threadIdx.x;
    const int n = pr.n;

    if (i0 == p0) {   // the pivot rows themselves: zero columns in V and W
        for (int e = tid; e < NB * NB; e += 256) {
            const int kk = e / NB, i = e % NB;
            if (i0 + i < n) {
                pr.Vt[(long)kk * pr.ldv + i0 + i] = 0.f;
                pr.Wt[(long)kk * pr.ldv + i0 + i] = 0.f;
            }
        }
        return;
    }
    for (int e = tid; e < NB * NB; e += 256) Ps[(e / NB) * PITCH + (e % NB)] = pr.P[e];
    if (i0 > p0) {    // column panel: M[gi][p0 + kk], contiguous in kk
        for (int e = tid; e < NB * NB; e += 256) {
            const int i = e / NB, kk = e % NB;
            const int gi = i0 + i;
            Vs[kk * PITCH + i] = (gi < n && kk < bs) ? pr.W[(long)gi * n + p0 + kk] : 0.f;
        }
    } else {          // row panel: M[p0 + kk][gi], contiguous in gi
        for (int e = tid; e < NB * NB; e += 256) {
            const int kk = e / NB, i = e % NB;
            const int gi = i0 + i;
            Vs[kk * PITCH + i] = (gi < n && kk < bs) ? pr.W[(long)(p0 + kk) * n + gi] : 0.f;
        }
    }
    __syncthreads();

    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    floatx4 acc[T::WT][T::WT];
#pragma unroll
    for (int a = 0; a < T::WT; ++a)
#pragma unroll
        for (int b = 0; b < T::WT; ++b) acc[a][b] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int q = 0; q < NB / T::KT; ++q)
        mma_stage<T, kRows, kRows, false>(Ps + q * T::KT * PITCH, Vs + q * T::KT * PITCH, wm, wn, lane, acc);

    // acc[ti][tj][v] = W^T[m][i], m = (wm*2+ti)*16 + 4*lk + v, i = (wn*2+tj)*16 + lr
    const int lr = lane & 15, lk = lane >> 4;
#pragma unroll
    for (int ti = 0; ti < T::WT; ++ti)
#pragma unroll
        for (int tj = 0; tj < T::WT; ++tj) {
            const int i = (wn * T::WT + tj) * 16 + lr;
            const int gi = i0 + i;
            if (gi >= n) continue;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int m = (wm * T::WT + ti) * 16 + 4 * lk + v;
                const float w = acc[ti][tj][v];
                pr.Vt[(long)m * pr.ldv + gi] = Vs[m * PITCH + i];
                pr.Wt[(long)m * pr.ldv + gi] = w;
                if (m < bs) {
                    if (i0 > p0)
                        pr.W[(long)gi * n + p0 + m] = w;
                    else
                        pr.W[(long)(p0 + m) * n + gi] = w;
                }
            }
        }
}

// out = -W mirrored to both triangles (in place)
__global__ __launch_bounds__(256) void sweep_finish_kernel(const InvTable tab)
{
    int pi = 0;
    while (pi + 1 < tab.count && (int)blockIdx.x >= tab.p[pi + 1].blk_start) ++pi;
    const InvProb &pr = tab.p[pi];
    const int local = blockIdx.x - pr.blk_start;
    const long total = (long)pr.n * pr.n;
    for (long e = (long)local * 4096 + threadIdx.x; e < lmin(total, (long)(local + 1) * 4096); e += 256) {
        const int i = (int)(e / pr.n), j = (int)(e - (long)i * pr.n);
        if (j <= i) {
            const float v = -pr.W[e];
            pr.W[e] = v;
            pr.W[(long)j * pr.n + i] = v;
        }
    }
}

namespace {
size_t job_ws_floats(int n) { return 2 * (size_t)NB * NB + 2 * (size_t)NB * ((n + 3) / 4 * 4); }
size_t table_bytes(int n) { return align_up((size_t)n * sizeof(InvProbF), 256); }

// One-launch-per-step sweep for the matrices listed in `idx` (sorted by order, largest first).
hipError_t fused_launch(const InvertJob *jobs, const std::vector<int> &idx, const std::vector<size_t> &offs,
                        void *work, InvProbF *dtab, hipStream_t s)
{
    const int total = (int)idx.size();
    // descriptors -> device table, 64 per upload launch
    for (int g0 = 0; g0 < total; g0 += 64) {
        InvUpload u;
        u.dst = dtab + g0;
        u.count = std::min(64, total - g0);
        for (int k = 0; k < u.count; ++k) {
            const InvertJob &j = jobs[idx[g0 + k]];
            InvProbF &p = u.p[k];
            float *ws = reinterpret_cast<float *>(static_cast<char *>(work) + offs[idx[g0 + k]]);
            p.M = j.M; p.W = j.Minv; p.info = j.info; p.n = j.n; p.damping = j.damping;
            p.ldv = (j.n + 3) / 4 * 4;
            p.nblk = (j.n + FNB - 1) / FNB;
            p.P = ws;
            p.Vt = ws + 2 * FNB * FNB;
        }
        KFAC_LAUNCH(KFAC_K_INV_INIT, s, inv_upload_kernel, dim3(1), dim3(64), 0, u);
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
                blocks += (long)t.c[k].per * t.c[k].count;
            }
            return blocks;
        };
        const int nclass = q.nclass;
        long blocks = 0;
        hipError_t e = hipSuccess;
        blocks = lay_out(q, nclass, [](const InvClass &) { return 1; });
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
            e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}
}  // namespace

size_t invert_workspace_bytes(const InvertJob *jobs, int n)
{
    size_t total = table_bytes(n);
    for (int i = 0; i < n; ++i) total += align_up(job_ws_floats(jobs[i].n) * sizeof(float), 256);
    return total;
}

hipError_t invert_launch(const InvertJob *jobs, int n_all, void *work, size_t work_bytes, hipStream_t s)
{
    if (invert_workspace_bytes(jobs, n_all) > work_bytes) return hipErrorInvalidValue;
    std::vector<size_t> offs(n_all);
    size_t off = table_bytes(n_all);
    for (int i = 0; i < n_all; ++i) {
        offs[i] = off;
        off += align_up(job_ws_floats(jobs[i].n) * sizeof(float), 256);
    }
    // largest matrices first so that one launch group holds similar step counts
    std::vector<int> order, fused;
    for (int i = 0; i < n_all; ++i) (jobs[i].n <= tuning().invert_fused_max_n ? fused : order).push_back(i);
    auto by_size = [&](int a, int b) { return jobs[a].n > jobs[b].n; };
    std::stable_sort(order.begin(), order.end(), by_size);
    std::stable_sort(fused.begin(), fused.end(), by_size);
    const int n = (int)order.size();

    for (int g0 = 0; g0 < n; g0 += kMaxProblems) {
        const int cnt = std::min(kMaxProblems, n - g0);
        InvTable tab;
        tab.count = cnt;
        tab.step = 0;
        int nmax = 0;
        for (int k = 0; k < cnt; ++k) {
            const InvertJob &j = jobs[order[g0 + k]];
            InvProb &p = tab.p[k];
            float *ws = reinterpret_cast<float *>(static_cast<char *>(work) + offs[order[g0 + k]]);
            p.M = j.M; p.W = j.Minv; p.info = j.info; p.n = j.n; p.damping = j.damping;
            p.ldv = (j.n + 3) / 4 * 4;
            p.P = ws;
            p.Vt = ws + NB * NB;
            p.Wt = p.Vt + (size_t)NB * p.ldv;
            nmax = std::max(nmax, j.n);
        }
        // element-wise kernels: 4096 elements per block
        int blocks = 0;
        for (int k = 0; k < cnt; ++k) {
            tab.p[k].blk_start = blocks;
            blocks += (int)(((long)tab.p[k].n * tab.p[k].n + 4095) / 4096);
        }
        const int ew_blocks = blocks;
        KFAC_LAUNCH(KFAC_K_INV_INIT, s, sweep_init_kernel, dim3(ew_blocks), dim3(256), 0, tab);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;

        const int steps = (nmax + NB - 1) / NB;
        for (int st = 0; st < steps; ++st) {
            tab.step = st;
            const int p0 = st * NB;
            // matrices are sorted by size: those still active form a prefix
            int active = 0;
            while (active < cnt && tab.p[active].n > p0) ++active;
            InvTable t2 = tab;
            t2.count = active;
            KFAC_LAUNCH(KFAC_K_INV_PIVOT, s, sweep_pivot_kernel, dim3(active), dim3(256), 0, t2);
            e = hipGetLastError();
            if (e != hipSuccess) return e;
            // panel + update only where something lies outside the pivot block
            int act2 = 0;
            while (act2 < active && tab.p[act2].n > NB) ++act2;
            if (act2 == 0) continue;
            t2.count = act2;
            blocks = 0;
            for (int k = 0; k < act2; ++k) {
                t2.p[k].blk_start = blocks;
                blocks += (t2.p[k].n + NB - 1) / NB;
            }
            KFAC_LAUNCH(KFAC_K_INV_PANEL, s, sweep_panel_kernel, dim3(blocks), dim3(256), 0, t2);
            e = hipGetLastError();
            if (e != hipSuccess) return e;
            std::vector<GemmJob> gj(act2);
            for (int k = 0; k < act2; ++k) {
                const InvProb &p = t2.p[k];
                GemmJob &g = gj[k];
                g.A = p.Wt; g.B = p.Vt; g.C = p.W;
                g.M = p.n; g.N = p.n; g.K = NB;
                g.lda = p.ldv; g.ldb = p.ldv; g.ldc = p.n;
                g.mode = kSubLowerSkip;
                g.p0 = p0;
                g.p1 = std::min(p.n, p0 + NB);
            }
            e = gemm_launch(gj.data(), act2, s);
            if (e != hipSuccess) return e;
        }
        blocks = 0;
        for (int k = 0; k < cnt; ++k) {
            tab.p[k].blk_start = blocks;
            blocks += (int)(((long)tab.p[k].n * tab.p[k].n + 4095) / 4096);
        }
        KFAC_LAUNCH(KFAC_K_INV_FINISH, s, sweep_finish_kernel, dim3(blocks), dim3(256), 0, tab);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (!fused.empty())
        return fused_launch(jobs, fused, offs, work, static_cast<InvProbF *>(work), s);
    return hipSuccess;
}

}  // namespace kfac

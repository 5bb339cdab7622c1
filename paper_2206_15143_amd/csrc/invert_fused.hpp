// One-launch-per-step form of the blocked symmetric sweep (see invert.hip for
// the method), for the small and medium factors where the three-kernel step
// (pivot, panel, update) is bound by launch latency and by the serial pivot
// block inversion rather than by flops.
//
// Step K of the sweep is ONE launch over all lower-triangular 64 x 64 tiles of
// all matrices that are still active:
//   - a tile in the pivot row/column (panel tile) computes W = V P and stores
//     it in place;
//   - any other tile (i, j) loads V_i and V_j, forms W_i = V_i P on the MFMA
//     units again (cheaper than a launch that would share it) and applies
//     M_ij -= W_i V_j^T;
//   - tiles in row/column K+1 also store their new values K-major into the
//     side buffer V' that step K+1 reads (so the panel is never read from the
//     matrix while panel tiles overwrite it);
//   - the workgroup of tile (K+1, K+1) goes on to invert that block, which is
//     final for step K+1 once updated: P' and the in-place block are ready
//     when the launch ends.  That tile gets block index 0 of its matrix so
//     that it starts first.
// Step 0 reads the input factor (plus damping) instead of the working matrix and
// the last step of a matrix stores the negated result to both triangles, so
// there is no initialisation or finishing pass.
// P and V are double buffered by step parity.  Problem descriptors live in
// device memory (uploaded by a small kernel from kernel arguments), so one
// launch covers any number of matrices; the launch argument only carries the
// table of distinct sizes.
#pragma once

#include "tn_engine.hpp"

namespace kfac {

constexpr int FNB = 64;            // pivot block order
constexpr int kMaxInvClasses = 24; // distinct matrix orders per launch sequence

struct InvProbF {
    const float *M;   // input factor [n, n], lower triangle read
    float *W;         // working matrix = output [n, n]
    float *P;         // 2 x [64, 64] pivot-block inverses (step parity)
    float *Vt;        // 2 x [64, ldv] K-major panels (step parity)
    float *S;         // 2 x [64, 64] pivot blocks before their inversion, both triangles (step parity)
    int *gate;        // 2 flags (step parity): the pivot block is ill-conditioned, refine the panel product;
                      // a third that stays set once either was (read by the bordering of orders 64 k + 1)
    int *info;
    int n;
    int ldv;          // n rounded up to 4
    float damping;
    int nblk;
    int ldm, ldw;     // row pitches of M and W
    const float *dptr; // device-side damping (overrides `damping` when not null)
};

constexpr int kInvUploadMax = 224;   // descriptors per upload launch (a 20 KB kernel argument)

struct InvUpload {
    InvProbF *dst;
    int count;
    InvProbF p[kInvUploadMax];
};

struct InvClass {
    int first;       // index of the first problem of this class in the device table
    int count;       // problems in the class
    int n, nblk;
    int per;         // blocks per problem in this launch
    int blk_start;   // first block of the class in this launch (a multiple of 8)
};

struct InvSeq {
    const InvProbF *tab;
    int nclass;
    int step;
    float refine_cond;   // panel products of pivot blocks whose condition number exceeds this are refined (< 0: never)
    InvClass c[kMaxInvClasses];
};

__global__ __launch_bounds__(64) void inv_upload_kernel(const InvUpload u)
{
    // plain vector stores of the descriptors into the device table
    const int words = (int)(sizeof(InvProbF) / 4);
    const unsigned *src = reinterpret_cast<const unsigned *>(u.p);
    unsigned *dst = reinterpret_cast<unsigned *>(u.dst);
    for (int e = threadIdx.x + blockIdx.x * 64; e < u.count * words; e += 64 * gridDim.x) dst[e] = src[e];
}

// Block -> (matrix, block of that matrix).  Inside a class the blocks are dealt block-major: block `local` of
// every matrix before block `local + 1` of any, with the matrix count rounded up to a multiple of 8 (the slots
// past the last matrix are empty).  Two things follow: workgroup i runs on XCD i mod 8, so every block of a
// matrix runs on the same XCD and its panels and pivot inverse are fetched into one L2 instead of eight; and
// block 0 of every matrix (the one that goes on to invert the next pivot block) is dispatched first.
__host__ __device__ __forceinline__ int seq_slots(int count) { return (count + 7) & ~7; }

__device__ __forceinline__ bool seq_locate(const InvSeq &q, int blk, int &prob, int &local, int &ci)
{
    ci = 0;
    while (ci + 1 < q.nclass && blk >= q.c[ci + 1].blk_start) ++ci;
    const InvClass &c = q.c[ci];
    const int off = blk - c.blk_start;
    const int slots = seq_slots(c.count);
    local = off / slots;
    const int pl = off - local * slots;
    if (pl >= c.count || local >= c.per) return false;
    prob = c.first + pl;
    return true;
}

// One pivot of the in-register 16 x 16 sweep (see sweep64_blocked): lane (lr, lk) holds D[lr][4lk..4lk+3].
template <int K>
__device__ __forceinline__ void sweep16_pivot(float (&d)[4], int lr, int lk, int c0, int &fail)
{
    float rk[4];
#pragma unroll
    for (int m = 0; m < 4; ++m)
        rk[m] = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(d[m]), 0x150 + K, 0xf, 0xf, false));
    // the pivot D[K][K] sits in lane K + 16*(K>>2), register K & 3
    const float p = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(d[K & 3]), K + 16 * (K >> 2)));
    if (!(p > 0.f) && fail == 0) fail = c0 + K + 1;
    const float ip = __builtin_amdgcn_rcpf(p);   // 1 ulp reciprocal: far below the fp32 error of the sweep
    // column element D[i][K] = D[K][i]: element i of the row, held by lane i + 16*(i>>2) in register i & 3
    float mine = rk[0];
    mine = (lr & 3) == 1 ? rk[1] : mine;
    mine = (lr & 3) == 2 ? rk[2] : mine;
    mine = (lr & 3) == 3 ? rk[3] : mine;
    const float ci = __int_as_float(__builtin_amdgcn_ds_bpermute((lr + 16 * (lr >> 2)) * 4, __float_as_int(mine)));
    const float cip = ci * ip;
    const bool prow = (lr == K);
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        const float upd = __builtin_fmaf(-cip, rk[m], d[m]);
        const float onr = rk[m] * ip;
        float v = prow ? onr : upd;
        if (m == (K & 3)) v = (lk == (K >> 2)) ? (prow ? -ip : cip) : v;
        d[m] = v;
    }
}

// Sweep of a 64 x 64 pivot block held in LDS (full symmetric storage, row pitch
// SW_PITCH; blocks smaller than 64 are padded with the identity by the caller).  Four sub-steps of 16
// pivots.  Per sub-step: wavefront 0 sweeps the 16 x 16 pivot block inside its registers (lane (i, q)
// holds D[i][4q..4q+3]; the pivot row reaches the lanes by DPP row broadcast, the pivot column, equal to
// the row by symmetry, by one ds_bpermute: no barrier inside the 16 pivots); then all four wavefronts
// form W = V P and the rank-16 update of the other blocks on the MFMA units and write the new panel.
// On exit S holds the swept block (-inverse).  Pb: [16][17], Wb: [64][17] scratch.
// Returns 0 or the 1-based index (within the block) of the first non-positive pivot (valid in wave 0).
constexpr int SW_PITCH = 68;

__device__ __forceinline__ int sweep64_blocked(float *S, float *Pb, float *Wb, int tid)
{
    const int lane = tid & 63, w = tid >> 6;
    const int lr = lane & 15, lk = lane >> 4;
    int fail = 0;
#pragma unroll 1
    for (int kb = 0; kb < 4; ++kb) {
        const int c0 = kb * 16;
        if (w == 0) {
            // ---- the 16 x 16 pivot block, in registers ----
            float d[4];
            {
                const floatx4 v = *reinterpret_cast<const floatx4 *>(S + (c0 + lr) * SW_PITCH + c0 + 4 * lk);
                d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
            }
            sweep16_pivot<0>(d, lr, lk, c0, fail);
            sweep16_pivot<1>(d, lr, lk, c0, fail);
            sweep16_pivot<2>(d, lr, lk, c0, fail);
            sweep16_pivot<3>(d, lr, lk, c0, fail);
            sweep16_pivot<4>(d, lr, lk, c0, fail);
            sweep16_pivot<5>(d, lr, lk, c0, fail);
            sweep16_pivot<6>(d, lr, lk, c0, fail);
            sweep16_pivot<7>(d, lr, lk, c0, fail);
            sweep16_pivot<8>(d, lr, lk, c0, fail);
            sweep16_pivot<9>(d, lr, lk, c0, fail);
            sweep16_pivot<10>(d, lr, lk, c0, fail);
            sweep16_pivot<11>(d, lr, lk, c0, fail);
            sweep16_pivot<12>(d, lr, lk, c0, fail);
            sweep16_pivot<13>(d, lr, lk, c0, fail);
            sweep16_pivot<14>(d, lr, lk, c0, fail);
            sweep16_pivot<15>(d, lr, lk, c0, fail);
            // P = -swept block
#pragma unroll
            for (int m = 0; m < 4; ++m) Pb[lr * 17 + 4 * lk + m] = -d[m];
        }
        __syncthreads();
        // ---- W = V P for the row tile of this wavefront (rows 16w..16w+15) ----
        if (w != kb) {
            floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) {
                const float a = S[(16 * w + lr) * SW_PITCH + c0 + 4 * s4 + lk];
                const float b = Pb[(4 * s4 + lk) * 17 + lr];
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc, 0, 0, 0);
            }
#pragma unroll
            for (int v = 0; v < 4; ++v) Wb[(16 * w + 4 * lk + v) * 17 + lr] = acc[v];
        }
        __syncthreads();
        // ---- S_ij -= W_i V_j^T for the nine blocks outside the pivot row and column ----
        for (int t = w; t < 9; t += 4) {
            const int r3 = t / 3, c3 = t - 3 * r3;
            const int bi = r3 + (r3 >= kb ? 1 : 0), bj = c3 + (c3 >= kb ? 1 : 0);
            floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) {
                const float a = Wb[(16 * bi + lr) * 17 + 4 * s4 + lk];
                const float b = S[(16 * bj + lr) * SW_PITCH + c0 + 4 * s4 + lk];
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc, 0, 0, 0);
            }
#pragma unroll
            for (int v = 0; v < 4; ++v) S[(16 * bi + 4 * lk + v) * SW_PITCH + 16 * bj + lr] -= acc[v];
        }
        __syncthreads();
        // ---- new panel (both triangles) and pivot block ----
        for (int e = tid; e < 64 * 16; e += 256) {
            const int i = e >> 4, c = e & 15;
            if ((i >> 4) != kb) {
                const float wv = Wb[i * 17 + c];
                S[i * SW_PITCH + c0 + c] = wv;
                S[(c0 + c) * SW_PITCH + i] = wv;
            } else {
                S[i * SW_PITCH + c0 + c] = -Pb[(i - c0) * 17 + c];
            }
        }
        __syncthreads();
    }
    return fail;
}

// The condition test of a pivot block (largest absolute row sums of the block and of its inverse) rides on the loops
// that load the block and store its inverse: in those loops thread t visits column t mod 64 in the rows t / 64 + 4 k,
// so it sums the absolute values it sees (both matrices are symmetric: column sums are row sums), leaves its part
// in nrm[(t / 64) * 64 + column], and after the next barrier one wavefront folds the four parts of every column and
// takes the largest.  nrm: 4 * 64 + 2 floats of LDS; the result goes to nrm[256 + slot], read after a later barrier.
__device__ __forceinline__ void norm_fold(float *nrm, int slot, int lane)
{
    float a = nrm[lane] + nrm[64 + lane] + nrm[128 + lane] + nrm[192 + lane];
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) a = fmaxf(a, __shfl_xor(a, off));
    if (lane == 0) nrm[256 + slot] = a;
}

// Workgroup 0 of a matrix inverts the first pivot block; workgroup r >= 1 copies block r of the first
// column panel K-major into V[0] (transposed through LDS), so that step 0 stages its panels like any
// other step.
__global__ __launch_bounds__(256) void fsweep_pivot0_kernel(const InvSeq q)
{
    __shared__ __attribute__((aligned(16))) float sbuf[64 * SW_PITCH];
    __shared__ __attribute__((aligned(16))) float pw[16 * 17 + 64 * 17];
    __shared__ float nrm[4 * 64 + 2];
    float (*tile)[65] = reinterpret_cast<float (*)[65]>(sbuf);
    int prob, local, ci;
    if (!seq_locate(q, blockIdx.x, prob, local, ci)) return;
    const InvProbF pr = q.tab[prob];
    const int tid = threadIdx.x;
    if (local > 0) {
        const int g0 = local * FNB;
        for (int e = tid; e < FNB * FNB; e += 256) {
            const int c = e >> 6, k = e & 63;
            tile[c][k] = (g0 + c < pr.n) ? pr.M[(long)(g0 + c) * pr.ldm + k] : 0.f;
        }
        __syncthreads();
        for (int e = tid; e < FNB * FNB; e += 256) {
            const int k = e >> 6, c = e & 63;
            if (g0 + c < pr.n) pr.Vt[(long)k * pr.ldv + g0 + c] = tile[c][k];
        }
        return;
    }
    const int bs = min(FNB, pr.n);
    const long ldm = pr.ldm, ldw = pr.ldw;
    const float damping = pr.dptr ? *pr.dptr : pr.damping;
    const bool test = q.refine_cond >= 0.f;
    float colsum = 0.f;
    for (int e = tid; e < FNB * FNB; e += 256) {
        const int i = e >> 6, j = e & 63;
        float v = (i == j) ? 1.f : 0.f;
        const bool in = i < bs && j < bs;
        if (in) {
            const int a = max(i, j), b = min(i, j);
            v = pr.M[a * ldm + b] + (a == b ? damping : 0.f);
            colsum += fabsf(v);
        }
        sbuf[i * SW_PITCH + j] = v;
        if (test) pr.S[i * FNB + j] = in ? v : 0.f;
    }
    nrm[tid] = colsum;
    __syncthreads();
    if (test && (tid >> 6) == 1) norm_fold(nrm, 0, tid & 63);       // beside the first in-register sweep of wavefront 0
    const int fail = sweep64_blocked(sbuf, pw, pw + 16 * 17, tid);   // valid in wavefront 0
    const bool whole = pr.nblk == 1;   // the block is the matrix: store the result itself, both triangles
    colsum = 0.f;
    for (int e = tid; e < FNB * FNB; e += 256) {
        const int i = e >> 6, j = e & 63;
        const bool in = (i < bs && j < bs);
        const float v = sbuf[i * SW_PITCH + j];
        if (in) colsum += fabsf(v);
        pr.P[i * FNB + j] = in ? -v : 0.f;
        if (in && j <= i) {
            pr.W[i * ldw + j] = whole ? -v : v;
            if (whole) pr.W[j * ldw + i] = -v;
        }
    }
    if (tid == 0) *pr.info = (fail <= bs) ? fail : 0;
    if (!test) return;
    nrm[tid] = colsum;
    __syncthreads();
    if ((tid >> 6) == 0) {
        norm_fold(nrm, 1, tid);
        if (tid == 0) {
            // (a failed inversion leaves a NaN here: the comparison is false and the block is left alone)
            const int open = nrm[256] * nrm[257] > q.refine_cond ? 1 : 0;
            pr.gate[0] = open;
            pr.gate[2] = open;
        }
    }
}

// One step of the sweep for every tile of every active matrix (see the header of this file).
__global__ __launch_bounds__(256) void fsweep_step_kernel(const InvSeq q)
{
    typedef Tile<2, 2> T;
    constexpr int PITCH = T::PITCH;   // 80
    // two operand buffers (40 KB: three workgroups per CU; the pivot-block sweep reuses them).  P is
    // not staged: every lane keeps its 32 operand values of P in registers.
    __shared__ __attribute__((aligned(16))) float Va[FNB * PITCH];   // V of the tile's row block (or the panel block)
    __shared__ __attribute__((aligned(16))) float Vb[FNB * PITCH];   // V of the tile's column block, or W^T
    __shared__ float nrm[4 * 64 + 2];                                // the condition test of the next pivot block

    int prob, t, ci;
    if (!seq_locate(q, blockIdx.x, prob, t, ci)) return;
    const InvProbF pr = q.tab[prob];
    const int K = q.step, K1 = K + 1;
    const int nblk = pr.nblk;
    if (K >= nblk) return;
    int bi, bj;
    tri_decode(t, bi, bj);
    if (K1 < nblk) {   // the next pivot tile takes block 0 and gives tile (0, 0) its own slot
        const int tp = K1 * (K1 + 1) / 2 + K1;
        if (t == 0) { bi = K1; bj = K1; }
        else if (t == tp) { bi = 0; bj = 0; }
    }
    const int tid = threadIdx.x;
    const int n = pr.n, ldv = pr.ldv;
    const long ldm = pr.ldm, ldw = pr.ldw;
    const bool first = (K == 0), last = (K1 == nblk);
    const float damping = (first && pr.dptr) ? *pr.dptr : pr.damping;
    if (bi == K && bj == K) {
        // the pivot block itself was finished by the previous launch; on the last step it still has to
        // be negated and mirrored like everything else
        if (last) {
            const int p0 = K * FNB, bs = n - p0;
            for (int e = tid; e < FNB * FNB; e += 256) {
                const int i = e >> 6, j = e & 63;
                if (i < bs && j <= i) {
                    const float v = -pr.W[(long)(p0 + i) * ldw + p0 + j];
                    pr.W[(long)(p0 + i) * ldw + p0 + j] = v;
                    pr.W[(long)(p0 + j) * ldw + p0 + i] = v;
                }
            }
        }
        return;
    }

    const int p0 = K * FNB, p1 = K1 * FNB;
    const int bs = min(FNB, n - p0);
    const int bs1 = min(FNB, n - p1);              // <= 0 when there is no next block
    const float *Pk = pr.P + (K & 1) * FNB * FNB;
    const float *Vk = pr.Vt + (long)(K & 1) * FNB * ldv;
    float *Pn = pr.P + (K1 & 1) * FNB * FNB;
    float *Sn = pr.S + (K1 & 1) * FNB * FNB;
    const float *Sk = pr.S + (K & 1) * FNB * FNB;
    const bool refine = q.refine_cond >= 0.f && pr.gate[K & 1] != 0;      // uniform over the workgroup
    float *Vn = pr.Vt + (long)(K1 & 1) * FNB * ldv;
    const bool panel = (bi == K) != (bj == K);
    const int ra = panel ? (bi == K ? bj : bi) : bi;   // block whose V goes to Va
    const int rb = bj;

    // the tile's current values: fetched now, needed after the two products
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int lr = lane & 15, lk = lane >> 4;
    const bool diag = (bi == bj);
    float oldc[T::WT][T::WT][4];
    if (!panel) {
#pragma unroll
        for (int ti = 0; ti < T::WT; ++ti)
#pragma unroll
            for (int tj = 0; tj < T::WT; ++tj) {
                const int gb = bj * FNB + (wn * T::WT + tj) * 16 + lr;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int ga = bi * FNB + (wm * T::WT + ti) * 16 + 4 * lk + v;
                    const bool ok = (ga < n && gb < n && (!diag || gb <= ga));
                    float o = 0.f;
                    if (ok)
                        o = first ? pr.M[(long)ga * ldm + gb] + (ga == gb ? damping : 0.f)
                                  : pr.W[(long)ga * ldw + gb];
                    oldc[ti][tj][v] = o;
                }
            }
    }

    // ---- P operand values of this lane: P[k = 4s + lk][m = (wm*2 + t)*16 + lr] ----
    float pa[FNB / 4][T::WT];
#pragma unroll
    for (int s4 = 0; s4 < FNB / 4; ++s4)
#pragma unroll
        for (int t2 = 0; t2 < T::WT; ++t2) pa[s4][t2] = Pk[(4 * s4 + lk) * FNB + (wm * T::WT + t2) * 16 + lr];

    // ---- stage V_a (and V_b) ----
    for (int e = tid; e < FNB * FNB / 4; e += 256) {
        const int k = e >> 4, c4 = (e & 15) * 4;
        const int ga = ra * FNB + c4;
        floatx4 va = {0.f, 0.f, 0.f, 0.f};
        if (ga < ldv && k < bs) {
            va = *reinterpret_cast<const floatx4 *>(Vk + (long)k * ldv + ga);
            if (ga + 1 >= n) va.y = 0.f;
            if (ga + 2 >= n) va.z = 0.f;
            if (ga + 3 >= n) va.w = 0.f;
        }
        *reinterpret_cast<floatx4 *>(Va + k * PITCH + c4) = va;
        if (!panel && rb != ra) {
            const int gb = rb * FNB + c4;
            floatx4 vb = {0.f, 0.f, 0.f, 0.f};
            if (gb < ldv && k < bs) {
                vb = *reinterpret_cast<const floatx4 *>(Vk + (long)k * ldv + gb);
                if (gb + 1 >= n) vb.y = 0.f;
                if (gb + 2 >= n) vb.z = 0.f;
                if (gb + 3 >= n) vb.w = 0.f;
            }
            *reinterpret_cast<floatx4 *>(Vb + k * PITCH + c4) = vb;
        }
    }
    __syncthreads();

    floatx4 acc[T::WT][T::WT];
#pragma unroll
    for (int a = 0; a < T::WT; ++a)
#pragma unroll
        for (int b = 0; b < T::WT; ++b) acc[a][b] = floatx4{0.f, 0.f, 0.f, 0.f};
    // acc = W^T[m][c] = sum_k P[k][m] V_a[k][c]   (P symmetric)
#pragma unroll
    for (int s4 = 0; s4 < FNB / 4; ++s4) {
        float b[T::WT];
#pragma unroll
        for (int t2 = 0; t2 < T::WT; ++t2) b[t2] = Va[(4 * s4 + lk) * PITCH + (wn * T::WT + t2) * 16 + lr];
#pragma unroll
        for (int ti = 0; ti < T::WT; ++ti)
#pragma unroll
            for (int tj = 0; tj < T::WT; ++tj)
                acc[ti][tj] = __builtin_amdgcn_mfma_f32_16x16x4f32(pa[s4][ti], b[tj], acc[ti][tj], 0, 0, 0);
    }

    if (refine) {
        // One step of iterative refinement of W = V P for an ill-conditioned pivot block S (see the blocked sweep in
        // invert.hip for the reason): R^T = V^T - S W^T, W^T += P R^T, two more 64 x 64 x 64 products.  W^T and R^T
        // pass through the LDS buffer this kind of tile does not need at this point.
        float vt[T::WT][T::WT][4];      // V^T in the layout of the accumulators
#pragma unroll
        for (int ti = 0; ti < T::WT; ++ti)
#pragma unroll
            for (int tj = 0; tj < T::WT; ++tj)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    vt[ti][tj][v] = Va[((wm * T::WT + ti) * 16 + 4 * lk + v) * PITCH + (wn * T::WT + tj) * 16 + lr];
        float *X = (panel || diag) ? Vb : Va;
        __syncthreads();   // every wave is done reading V_a
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
#pragma unroll
            for (int ti = 0; ti < T::WT; ++ti)
#pragma unroll
                for (int tj = 0; tj < T::WT; ++tj)
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        X[((wm * T::WT + ti) * 16 + 4 * lk + v) * PITCH + (wn * T::WT + tj) * 16 + lr] =
                            pass == 0 ? acc[ti][tj][v] : vt[ti][tj][v];
            __syncthreads();
            floatx4 r2[T::WT][T::WT];
#pragma unroll
            for (int a = 0; a < T::WT; ++a)
#pragma unroll
                for (int b = 0; b < T::WT; ++b) r2[a][b] = pass == 0 ? floatx4{0.f, 0.f, 0.f, 0.f} : acc[a][b];
#pragma unroll
            for (int s4 = 0; s4 < FNB / 4; ++s4) {
                float b[T::WT], sop[T::WT];     // the operand values of S are read as they are used: this path is rare
#pragma unroll
                for (int t2 = 0; t2 < T::WT; ++t2) {
                    b[t2] = X[(4 * s4 + lk) * PITCH + (wn * T::WT + t2) * 16 + lr];
                    sop[t2] = pass == 0 ? Sk[(4 * s4 + lk) * FNB + (wm * T::WT + t2) * 16 + lr] : 0.f;
                }
#pragma unroll
                for (int ti = 0; ti < T::WT; ++ti)
#pragma unroll
                    for (int tj = 0; tj < T::WT; ++tj)
                        r2[ti][tj] = __builtin_amdgcn_mfma_f32_16x16x4f32(pass == 0 ? sop[ti] : pa[s4][ti], b[tj],
                                                                          r2[ti][tj], 0, 0, 0);
            }
            __syncthreads();   // every wave is done reading X
            if (pass == 0) {
                // R^T = V^T - S W^T takes the place of V^T
#pragma unroll
                for (int ti = 0; ti < T::WT; ++ti)
#pragma unroll
                    for (int tj = 0; tj < T::WT; ++tj)
#pragma unroll
                        for (int v = 0; v < 4; ++v) vt[ti][tj][v] -= r2[ti][tj][v];
            } else {
#pragma unroll
                for (int a = 0; a < T::WT; ++a)
#pragma unroll
                    for (int b = 0; b < T::WT; ++b) acc[a][b] = r2[a][b];
            }
        }
        // off-diagonal tiles: V_a now holds R^T, which nothing reads again (W^T goes there next)
    }

    if (panel) {
        // new panel values in place; tile (K+1, K) also feeds the next step's V'
        const bool below = ra > K;
        const bool next = (ra == K1);
#pragma unroll
        for (int ti = 0; ti < T::WT; ++ti)
#pragma unroll
            for (int tj = 0; tj < T::WT; ++tj) {
                const int c = (wn * T::WT + tj) * 16 + lr;
                const int gc = ra * FNB + c;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int m = (wm * T::WT + ti) * 16 + 4 * lk + v;
                    const float w = acc[ti][tj][v];
                    const bool ok = (gc < n && m < bs);
                    if (ok) {
                        if (below) pr.W[(long)gc * ldw + p0 + m] = w;
                        else if (!last) pr.W[(long)(p0 + m) * ldw + gc] = w;
                        else {   // last step: the row panel is final
                            pr.W[(long)(p0 + m) * ldw + gc] = -w;
                            pr.W[(long)gc * ldw + p0 + m] = -w;
                        }
                    }
                    // V'[kk = c][column p0 + m] = M[p1 + c][p0 + m]; rows kk >= bs1 are zero
                    if (next && m < bs) Vn[(long)c * ldv + p0 + m] = ok ? w : 0.f;
                }
            }
        return;
    }

    // ---- W^T to LDS, then C = M_ij - W_i V_j^T ----
    // off-diagonal tiles: V_a is dead after the first product and takes W^T; diagonal tiles still need
    // V_a as V_j and put W^T into the unused second buffer
    float *Ws = diag ? Vb : Va;
    const float *Vj = diag ? Va : Vb;
    __syncthreads();   // every wave is done reading V_a
#pragma unroll
    for (int ti = 0; ti < T::WT; ++ti)
#pragma unroll
        for (int tj = 0; tj < T::WT; ++tj) {
            const int c = (wn * T::WT + tj) * 16 + lr;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int m = (wm * T::WT + ti) * 16 + 4 * lk + v;
                Ws[m * PITCH + c] = acc[ti][tj][v];
            }
        }
    __syncthreads();
#pragma unroll
    for (int a = 0; a < T::WT; ++a)
#pragma unroll
        for (int b = 0; b < T::WT; ++b) acc[a][b] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s4 = 0; s4 < FNB / T::KT; ++s4)
        mma_stage<T, kRows, kRows, false>(Ws + s4 * T::KT * PITCH, Vj + s4 * T::KT * PITCH, wm, wn, lane, acc);

    // acc[ti][tj][v] = (W_i V_j^T)[a][b], a = (wm*2+ti)*16 + 4*lk + v, b = (wn*2+tj)*16 + lr
    const bool next_col = (bj == K1 && bi > K1);    // column panel of the next pivot: V'[b][ga]
    const bool next_row = (bi == K1 && bj < K1);    // row panel of the next pivot: V'[a][gb]
    const bool next_piv = (bi == K1 && bj == K1);
    __syncthreads();   // Va is reused below when this tile is the next pivot
#pragma unroll
    for (int ti = 0; ti < T::WT; ++ti)
#pragma unroll
        for (int tj = 0; tj < T::WT; ++tj) {
            const int b = (wn * T::WT + tj) * 16 + lr;
            const int gb = bj * FNB + b;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int a = (wm * T::WT + ti) * 16 + 4 * lk + v;
                const int ga = bi * FNB + a;
                const bool ok = (ga < n && gb < n && (!diag || gb <= ga));
                float c = 0.f;
                if (ok) {
                    c = oldc[ti][tj][v] - acc[ti][tj][v];
                    if (last) {
                        pr.W[(long)ga * ldw + gb] = -c;
                        pr.W[(long)gb * ldw + ga] = -c;
                    } else if (!next_piv) {
                        pr.W[(long)ga * ldw + gb] = c;
                    }
                }
                if (next_col && ga < n) Vn[(long)b * ldv + ga] = ok ? c : 0.f;
                if (next_row && gb < n) Vn[(long)a * ldv + gb] = ok ? c : 0.f;
                if (next_piv) Va[a * PITCH + b] = c;
            }
        }
    if (!next_piv) return;

    // ---- this workgroup holds the next pivot block: invert it now ----
    __syncthreads();
    {
        const bool test = q.refine_cond >= 0.f;
        float colsum = 0.f;
        for (int e = tid; e < FNB * FNB; e += 256) {
            const int i = e >> 6, j = e & 63;
            float v = (i == j) ? 1.f : 0.f;
            const bool in = i < bs1 && j < bs1;
            if (in) {
                v = (j <= i) ? Va[i * PITCH + j] : Va[j * PITCH + i];
                colsum += fabsf(v);
            }
            Vb[i * SW_PITCH + j] = v;
            if (test) Sn[i * FNB + j] = in ? v : 0.f;
        }
        nrm[tid] = colsum;
        __syncthreads();
        if (test && (tid >> 6) == 1) norm_fold(nrm, 0, tid & 63);   // beside the first in-register sweep of wavefront 0
        const int fail = sweep64_blocked(Vb, Va, Va + 16 * 17, tid);
        colsum = 0.f;
        for (int e = tid; e < FNB * FNB; e += 256) {
            const int i = e >> 6, j = e & 63;
            const bool in = (i < bs1 && j < bs1);
            const float v = Vb[i * SW_PITCH + j];
            if (in) colsum += fabsf(v);
            Pn[i * FNB + j] = in ? -v : 0.f;
            if (in && j <= i) pr.W[(long)(p1 + i) * ldw + p1 + j] = v;
        }
        // launches of one sequence are ordered, so the first failing pivot wins
        if (fail != 0 && fail <= bs1 && tid == 0 && *pr.info == 0) *pr.info = p1 + fail;
        if (!test) return;
        nrm[tid] = colsum;
        __syncthreads();
        if ((tid >> 6) == 0) {
            norm_fold(nrm, 1, tid);
            if (tid == 0) {
                const int open = nrm[256] * nrm[257] > q.refine_cond ? 1 : 0;
                pr.gate[K1 & 1] = open;
                if (open) pr.gate[2] = 1;
            }
        }
    }
}

}  // namespace kfac

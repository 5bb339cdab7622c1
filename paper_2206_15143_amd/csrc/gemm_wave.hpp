// C = A^T B (both operands K-major fp32) with the wave-unit tiling of the factor
// kernel (syrk_wave.hpp): a workgroup owns one 144-wide macro row of A's columns
// and two adjacent 144-wide macro columns of B's columns; the 81 MFMA tiles
// (v_mfma_f32_16x16x4_f32) of a macro tile are cut into units of 40 and 41 for
// two wavefronts (column tiles 0-3 plus the top four tiles of column 4, and
// the rest), so the four wavefronts of a workgroup carry equal work; each
// keeps its accumulators for the whole K range.  Panels [16 k][144 columns] are copied from global
// memory straight into LDS by buffer_load_dwordx4 ... lds, double buffered: the
// two stage buffers take 55 KB, so two workgroups share a CU and the prologue
// and the read-modify-write epilogue of one overlap the MFMA loop of the other.
// Used for the large preconditioning products
// (Eq. 5 of the DP-KFAC paper) and for the rank-k updates and panel products of
// the two-level blocked inversion.
//
// Columns past M (or N) of an operand panel may hold neighbouring data (a
// 16-byte piece is not split); they only feed outputs that are never stored.
// Rows past K are outside the buffer range and arrive as zeros.
#pragma once

#include "wave_common.hpp"

namespace kfac {

struct GemmWProb {
    const float *A;
    const float *B;
    float *C;
    int lda, ldb, ldc;
    int M, N, K;
    int mI;          // macro rows (over M)
    int nJ2;         // macro column pairs (over N)
    int blk_start;
    int mode;        // kStore or kSubLowerSkip
    int p0, p1;
};

struct GemmWTable {
    int count;
    int xcd_remap;   // 1: give every XCD a contiguous range of tiles (pays when the launch spans many problems)
    GemmWProb p[kMaxProblems];
};

struct GemmWCtx {
    int4v rsrcA, rsrcB;
    unsigned vo[W_SLOTS][3];
    unsigned tileA, tileB;     // bytes per K stage
    unsigned lds_base;
    int nstages, w;
};

constexpr int GW_NSTAGE = 2;
constexpr int GW_LDS_FLOATS = GW_NSTAGE * W_STAGE + 256;   // + 1 KB landing zone for the padding loads

__device__ __forceinline__ void gemmw_issue(const GemmWCtx &c, int g)
{
    const unsigned buf = c.lds_base + (unsigned)((g & (GW_NSTAGE - 1)) * W_STAGE * 4);
    const unsigned dummy = c.lds_base + (unsigned)(GW_NSTAGE * W_STAGE * 4);
    const bool live = g < c.nstages;
#pragma unroll
    for (int s = 0; s < W_SLOTS; ++s) {
        const unsigned so = live ? (unsigned)g * (s == 0 ? c.tileA : c.tileB) : 0u;
#pragma unroll
        for (int qi = 0; qi < 3; ++qi) {
            const int q = c.w + 4 * qi;
            const bool piece = q < W_NT;
            const unsigned v = (live && piece) ? c.vo[s][qi] : W_OOB;
            const unsigned dst = piece ? buf + (unsigned)((s * W_PANEL + q * 256) * 4) : dummy;
            if (s == 0) dma16(dst, v, c.rsrcA, so);
            else dma16(dst, v, c.rsrcB, so);
        }
    }
}

// Tile (ti, tj) of a unit's 9 x 5 grid (tj counts from the unit's first column tile: 0 for part 0,
// 4 for part 1).  Part 0 owns columns 0-3 and rows 0-3 of column 4; part 1 owns rows 4-8 of column 4
// (its local column 0) and columns 5-8.
template <int PART>
__device__ __forceinline__ constexpr bool gemmw_owns(int ti, int tj)
{
    return PART == 0 ? (tj < 4 || ti < 4) : (tj > 0 || ti >= 4);
}

template <int PART>
__device__ __forceinline__ void gemmw_unit(const float *Pr, const float *Pc, int kk, int lane, floatx4 (&acc)[45])
{
    const int lr = lane & 15, lk = lane >> 4;
    const float *sr = Pr + (kk + lk) * W_MT + lr;
    const float *sc = Pc + (kk + lk) * W_MT + lr;     // Pc already points at the unit's first column tile
    float a[W_NT], b[5];
#pragma unroll
    for (int t = 0; t < W_NT; ++t) a[t] = sr[t * 16];
#pragma unroll
    for (int t = 0; t < 5; ++t) b[t] = sc[t * 16];
#pragma unroll
    for (int ti = 0; ti < W_NT; ++ti)
#pragma unroll
        for (int tj = 0; tj < 5; ++tj)
            if (gemmw_owns<PART>(ti, tj))
                acc[ti * 5 + tj] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[ti], b[tj], acc[ti * 5 + tj], 0, 0, 0);
}

template <int NC>
__device__ __forceinline__ void gemmw_loop(const GemmWCtx &c, const float *lds, int cslot, int ctile0, int lane,
                                           floatx4 (&acc)[45])
{
    gemmw_issue(c, 0);
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    for (int g = 0; g < c.nstages; ++g) {
        gemmw_issue(c, g + 1);   // into the buffer every wave left at the last barrier
        const float *buf = lds + (g & (GW_NSTAGE - 1)) * W_STAGE;
        const float *Pr = buf;
        const float *Pc = buf + cslot * W_PANEL + ctile0 * 16;
#pragma unroll
        for (int st = 0; st < 4; ++st) gemmw_unit<NC>(Pr, Pc, 4 * st, lane, acc);
        asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    }
}

__global__ __launch_bounds__(256, 2) void gemm_wave_kernel(const GemmWTable tab)
{
    __shared__ float lds[GW_LDS_FLOATS];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);

    const int bid = tab.xcd_remap ? xcd_block_id() : (int)blockIdx.x;
    int pi = 0;
    while (pi + 1 < tab.count && bid >= tab.p[pi + 1].blk_start) ++pi;
    const GemmWProb &pr = tab.p[pi];
    int local = bid - pr.blk_start;
    int I, jp;
    if (pr.mode == kSubLowerSkip) {
        // macro row I holds the column pairs with first column 2*jp <= I
        I = 0;
        while (local >= I / 2 + 1) { local -= I / 2 + 1; ++I; }
        jp = local;
    } else {
        I = local / pr.nJ2;
        jp = local - I * pr.nJ2;
    }
    const int J0 = 2 * jp;
    const int Jw = J0 + (w >> 1);          // macro column of this wave
    const int part = w & 1;
    const int ctile0 = part ? 4 : 0;

    if (pr.mode == kSubLowerSkip) {
        // macro tiles inside the pivot rows / columns are left untouched (p0 and p1 are multiples of 144)
        const int q0 = pr.p0 / W_MT, q1 = (pr.p1 + W_MT - 1) / W_MT;
        const bool row_skip = I >= q0 && I < q1;
        const bool both_cols_skip = (J0 >= q0 && J0 < q1) && (J0 + 1 >= q0 && J0 + 1 < q1);
        if (row_skip || both_cols_skip) return;
    }

    GemmWCtx c;
    c.w = w;
    c.lds_base = (unsigned)(unsigned long)(__attribute__((address_space(3))) float *)lds;
    c.nstages = (pr.K + W_KT - 1) / W_KT;
    {
        const unsigned long ba = (unsigned long)pr.A, bb = (unsigned long)pr.B;
        const long na = (long)pr.K * pr.lda * 4, nb = (long)pr.K * pr.ldb * 4;
        c.rsrcA.x = (int)(unsigned)ba; c.rsrcA.y = (int)(unsigned)(ba >> 32);
        c.rsrcA.z = na > 0x7fffffffl ? 0x7fffffff : (int)na; c.rsrcA.w = 0x00020000;
        c.rsrcB.x = (int)(unsigned)bb; c.rsrcB.y = (int)(unsigned)(bb >> 32);
        c.rsrcB.z = nb > 0x7fffffffl ? 0x7fffffff : (int)nb; c.rsrcB.w = 0x00020000;
    }
    c.tileA = (unsigned)(W_KT * pr.lda * 4);
    c.tileB = (unsigned)(W_KT * pr.ldb * 4);
#pragma unroll
    for (int qi = 0; qi < 3; ++qi) {
        const int q = w + 4 * qi;
        const int f = 256 * q + 4 * lane;
        const int k = f / W_MT;
        const int col = f - k * W_MT;
        const bool qok = q < W_NT;
        const int ga = I * W_MT + col, gb0 = J0 * W_MT + col, gb1 = (J0 + 1) * W_MT + col;
        c.vo[0][qi] = (qok && ga < pr.M) ? (unsigned)((k * pr.lda + ga) * 4) : W_OOB;
        c.vo[1][qi] = (qok && gb0 < pr.N) ? (unsigned)((k * pr.ldb + gb0) * 4) : W_OOB;
        c.vo[2][qi] = (qok && gb1 < pr.N) ? (unsigned)((k * pr.ldb + gb1) * 4) : W_OOB;
    }

    floatx4 acc[45];
#pragma unroll
    for (int i = 0; i < 45; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};

    if (part) gemmw_loop<1>(c, lds, 1 + (w >> 1), ctile0, lane, acc);
    else gemmw_loop<0>(c, lds, 1 + (w >> 1), ctile0, lane, acc);

    // ---- epilogue: acc[ti*5 + tj][v] = C[I*144 + ti*16 + 4*lk + v][Jw*144 + (ctile0 + tj)*16 + lr] ----
    const int lr = lane & 15, lk = lane >> 4;
    const bool lower = pr.mode == kSubLowerSkip;
    if (lower) {
        const int q0 = pr.p0 / W_MT, q1 = (pr.p1 + W_MT - 1) / W_MT;
        if (Jw > I || (Jw >= q0 && Jw < q1)) return;
    }
    if (!lower) {
#pragma unroll
        for (int ti = 0; ti < W_NT; ++ti)
#pragma unroll
            for (int tj = 0; tj < 5; ++tj) {
                if (!(part ? gemmw_owns<1>(ti, tj) : gemmw_owns<0>(ti, tj))) continue;
                const int n = Jw * W_MT + (ctile0 + tj) * 16 + lr;
                if (n >= pr.N) continue;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int m = I * W_MT + ti * 16 + 4 * lk + v;
                    if (m < pr.M) pr.C[(long)m * pr.ldc + n] = acc[ti * 5 + tj][v];
                }
            }
        return;
    }
    // read-modify-write of the lower triangle: the 20 loads of a tile row are issued together, and the loads
    // of the next tile row go out before the stores of the current one, so the nine round trips overlap
    auto load_row = [&](int ti, float (&old)[5][4]) {
#pragma unroll
        for (int tj = 0; tj < 5; ++tj) {
            const int n = Jw * W_MT + (ctile0 + tj) * 16 + lr;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int m = I * W_MT + ti * 16 + 4 * lk + v;
                const bool ok = (part ? gemmw_owns<1>(ti, tj) : gemmw_owns<0>(ti, tj)) && n < pr.N && m < pr.M && n <= m;
                old[tj][v] = ok ? pr.C[(long)m * pr.ldc + n] : 0.f;
            }
        }
    };
    auto store_row = [&](int ti, const float (&old)[5][4]) {
#pragma unroll
        for (int tj = 0; tj < 5; ++tj) {
            const int n = Jw * W_MT + (ctile0 + tj) * 16 + lr;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int m = I * W_MT + ti * 16 + 4 * lk + v;
                const bool ok = (part ? gemmw_owns<1>(ti, tj) : gemmw_owns<0>(ti, tj)) && n < pr.N && m < pr.M && n <= m;
                if (ok) pr.C[(long)m * pr.ldc + n] = old[tj][v] - acc[ti * 5 + tj][v];
            }
        }
    };
    float oa[5][4], ob[5][4];
    load_row(0, oa);
#pragma unroll
    for (int ti = 0; ti < W_NT; ti += 2) {
        if (ti + 1 < W_NT) load_row(ti + 1, ob);
        store_row(ti, oa);
        if (ti + 2 < W_NT) load_row(ti + 2, oa);
        if (ti + 1 < W_NT) store_row(ti + 1, ob);
    }
}

}  // namespace kfac

// C = A^T B for fp32 operands (both K-major) on the bf16 MFMA units, at fp32 accuracy.
//
// MI355X multiplies bf16 matrices sixteen times faster than fp32 ones (2.5 PFLOP/s against 157 TFLOP/s),
// so an fp32 product is cheaper as several bf16 products.  Every fp32 operand element is cut into three bf16
// pieces, x = x1 + x2 + x3 (x1 = bf16(x), x2 = bf16(x - x1), x3 = bf16(x - x1 - x2): 3 x 8 significant bits,
// the sum is exact), and the product keeps the six piece products down to 2^-16 of the leading one,
//     a b  ~  a1 b1 + a1 b2 + a2 b1 + a1 b3 + a3 b1 + a2 b2,
// each exact in the fp32 accumulator of v_mfma_f32_32x32x16_bf16.  The terms left out (a2 b3, a3 b2, a3 b3)
// are below 2^-24 |a b|, the size of the rounding of an fp32 product: the result is as accurate as an fp32
// MFMA product, for 6/16 of its MFMA time.
//
// Used for the preconditioning products (Eq. 5 of the DP-KFAC paper) and for the rank-k updates and panel
// products of the blocked inversion (section 5.2).
//
// A workgroup of four wavefronts owns a 256 x 128 tile of C (256 columns of A, 128 of B); wave (wm, wn) owns
// 128 x 64 of it: 4 x 2 MFMA tiles, 128 accumulator registers.  K is walked in stages of 16 rows = one MFMA
// step.  The fp32 panels [16 k][256 | 128 columns] are copied from global memory straight into LDS by
// buffer_load_dwordx4 ... lds (no staging registers) in a ring of three stage buffers, two stages in flight:
// a stage waits for loads issued two stages earlier, which is what hides the latency of the loads behind the
// 48 MFMAs of a stage (with the panels fetched through registers one stage ahead, the kernel spent three
// quarters of its time waiting for them).  A lane reads the eight k of its row of an operand tile from the
// panel (lanes along the columns: conflict-free), cuts them into the three pieces in registers and feeds the
// MFMAs; the conversions (5.5 VALU operations per element) are issued in the shadow of the MFMAs.  Three stage
// buffers take 72 KB: two workgroups share a CU, so the epilogue of one runs beside the MFMAs of the other.
//
// Rows past K lie outside the buffer range and arrive as zeros.  Columns past M (or N) may hold neighbouring
// data (a 16-byte piece is not split); they only feed outputs that are never stored.
#pragma once

#include "split_common.hpp"

namespace kfac {

struct GemmSProb {
    const float *A;
    const float *B;
    float *C;
    int lda, ldb, ldc;
    int M, N, K;
    int tI, tJ;      // tiles over M (256 rows) and N (128 columns)
    int blk_start;
    int mode;        // kStore, kSubLowerSkip, kSubRect or kAddRect
    int p0, p1;
    int doff;        // the subtracting modes touch n <= m + doff (0 for kSubLowerSkip)
    const int *gate; // null, or two float bit patterns: leave C alone unless their product exceeds gate_cond
    float gate_cond;
};

struct GemmSTable {
    int count;
    int debug;       // measurement only (results are wrong): 8 no epilogue
    GemmSProb p[kMaxProblems];
};

// column tiles of tile row i: all of them, or those that reach the line n = m + doff
__host__ __device__ inline int split_row_len(int mode, int tJ, int doff, int i)
{
    if (mode == kStore) return tJ;
    const long last = ((long)i * S_BM + S_BM - 1 + doff) / S_BN + 1;
    return (int)(last < tJ ? last : tJ);
}

__global__ __launch_bounds__(256, 2) void gemm_split_kernel(const GemmSTable tab)
{
    __shared__ __attribute__((aligned(16))) float lds[S_LDS_FLOATS];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = w >> 1, wn = w & 1;

    // Every XCD takes a contiguous range of tile numbers (its L2 then sees few operand panels), and the tiles of
    // a product are numbered in groups of four tile rows, column by column inside a group: the tiles that run
    // at the same time share their A panels (four per group) and their B panels (one per four tiles).
    const int bid = xcd_block_id();
    int pi = 0;
    while (pi + 1 < tab.count && bid >= tab.p[pi + 1].blk_start) ++pi;
    const GemmSProb &pr = tab.p[pi];
    // uniform over the workgroup, before any barrier or load
    if (pr.gate && !(__int_as_float(pr.gate[0]) * __int_as_float(pr.gate[1]) > pr.gate_cond)) return;
    int local = bid - pr.blk_start;
    int I, J;
    const bool lower = pr.mode != kStore;         // read-modify-write below the line n = m + doff
    const bool rows_skip = pr.mode == kSubLowerSkip;
    const bool add = pr.mode == kAddRect;
    {
        auto row_len = [&](int i) { return i >= pr.tI ? 0 : split_row_len(pr.mode, pr.tJ, pr.doff, i); };
        int g = 0;
        for (;;) {
            const int c = row_len(4 * g) + row_len(4 * g + 1) + row_len(4 * g + 2) + row_len(4 * g + 3);
            if (local < c) break;
            local -= c;
            ++g;
        }
        // inside the group: column J holds the rows whose length exceeds J (row lengths grow with i)
        const int l0 = row_len(4 * g), l1 = row_len(4 * g + 1), l2 = row_len(4 * g + 2), l3 = row_len(4 * g + 3);
        J = 0;
        for (;;) {
            const int c = (J < l0) + (J < l1) + (J < l2) + (J < l3);
            if (local < c) break;
            local -= c;
            ++J;
        }
        // the local-th row (in increasing order) among those with length > J
        int i = 0;
        for (int seen = 0;; ++i) {
            const int len = i == 0 ? l0 : (i == 1 ? l1 : (i == 2 ? l2 : l3));
            if (J < len) {
                if (seen == local) break;
                ++seen;
            }
        }
        I = 4 * g + i;
    }
    const int m0 = I * S_BM, n0 = J * S_BN;
    if (lower) {
        // tiles wholly inside the pivot rows or columns are left untouched
        const int m1 = min(m0 + S_BM, pr.M), n1 = min(n0 + S_BN, pr.N);
        if ((rows_skip && m0 >= pr.p0 && m1 <= pr.p1) || (n0 >= pr.p0 && n1 <= pr.p1)) return;
    }

    const int lda = pr.lda, ldb = pr.ldb;
    const int nstages = (pr.K + S_KT - 1) / S_KT;
    int4v rsrcA, rsrcB;
    {
        const unsigned long ba = (unsigned long)pr.A, bb = (unsigned long)pr.B;
        const long na = (long)pr.K * lda * 4, nb = (long)pr.K * ldb * 4;
        rsrcA.x = (int)(unsigned)ba; rsrcA.y = (int)(unsigned)(ba >> 32);
        rsrcA.z = na > 0x7fffffffl ? 0x7fffffff : (int)na; rsrcA.w = 0x00020000;
        rsrcB.x = (int)(unsigned)bb; rsrcB.y = (int)(unsigned)(bb >> 32);
        rsrcB.z = nb > 0x7fffffffl ? 0x7fffffff : (int)nb; rsrcB.w = 0x00020000;
    }
    // this wave's copies of a stage: rows 4 w .. 4 w + 3 of the A panel (one instruction per row: 64 lanes x
    // 4 columns) and of the B panel (one instruction per two rows: 32 lanes x 4 columns each)
    const unsigned lds_base = (unsigned)(unsigned long)(__attribute__((address_space(3))) float *)lds;
    const int ca = m0 + 4 * lane, cb = n0 + 4 * (lane & 31);
    const unsigned voa = ca < pr.M ? (unsigned)(ca * 4) : W_OOB;
    const unsigned vob = cb < pr.N ? (unsigned)(((lane >> 5) * ldb + cb) * 4) : W_OOB;
    const unsigned rowa = (unsigned)lda * 4u, rowb = (unsigned)ldb * 4u;
    const int dbg = tab.debug;
    auto issue = [&](int g) {
        const bool live_stage = g < nstages;
        const unsigned buf = lds_base + (unsigned)((g % S_NSTAGE) * S_STAGE * 4);
        const unsigned k0 = (unsigned)(g * S_KT + 4 * w);
#pragma unroll
        for (int r = 0; r < 4; ++r)
            dma16(buf + (unsigned)((4 * w + r) * S_BM * 4), live_stage ? voa : W_OOB, rsrcA,
                  live_stage ? (k0 + r) * rowa : 0u);
#pragma unroll
        for (int r = 0; r < 2; ++r)
            dma16(buf + (unsigned)((S_PANEL_A + (4 * w + 2 * r) * S_BN) * 4), live_stage ? vob : W_OOB, rsrcB,
                  live_stage ? (k0 + 2 * r) * rowb : 0u);
    };

    floatx16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;

    const int lr = lane & 31, lg = lane >> 5;
    // a wave whose 128 x 64 part lies wholly above the line n = m + doff has nothing to compute
    const bool idle = lower && (n0 + wn * 64 > m0 + wm * 128 + 127 + pr.doff);
    const int fa = 8 * lg * S_BM + wm * 128 + lr;                    // + e * S_BM (k) + t * 32 (tile)
    const int fb = S_PANEL_A + 8 * lg * S_BN + wn * 64 + lr;

    issue(0);
    issue(1);
    asm volatile("s_waitcnt vmcnt(6)\n\ts_barrier" ::: "memory");
    for (int g = 0; g < nstages; ++g) {
        issue(g + 2);        // into the buffer every wave left at the last barrier (stages past the end: zeros)
        if (!idle) {
            const float *buf = lds + (g % S_NSTAGE) * S_STAGE;
            suint4 b1[2], b2[2], b3[2];
            float xa[8], xn[8];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                float x[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) x[e] = buf[fb + e * S_BN + t * 32];
                if (t == 0) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) xa[e] = buf[fa + e * S_BM];
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) xn[e] = buf[fa + e * S_BM + 32];
                }
                split_pieces(x, b1[t], b2[t], b3[t]);
            }
            suint4 c1, c2, c3;          // pieces of the A tile being multiplied
            split_pieces(xa, c1, c2, c3);
            __builtin_amdgcn_sched_barrier(0);
            // Tile ti: its twelve products, with the conversions of tile ti + 1 (and the panel reads of tile
            // ti + 2) issued between them, four VALU operations in the shadow of every MFMA.
#pragma unroll
            for (int ti = 0; ti < 4; ++ti) {
                suint4 n1, n2, n3;
                if (ti + 1 < 4) split_pieces(xn, n1, n2, n3);
                if (ti + 2 < 4) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) xn[e] = buf[fa + e * S_BM + (ti + 2) * 32];
                }
                const sbf16x8 A1 = __builtin_bit_cast(sbf16x8, c1), A2 = __builtin_bit_cast(sbf16x8, c2),
                              A3 = __builtin_bit_cast(sbf16x8, c3);
                {
                    // Smallest terms first.  The two column tiles alternate: an MFMA that accumulates into the result of the one
                    // just before it waits for that result (a single chain reaches 67 % of the rate of two, measured), and the
                    // order of the six terms of each accumulator is what fixes the bits, not the interleaving.
                    const sbf16x8 P1 = __builtin_bit_cast(sbf16x8, b1[0]), P2 = __builtin_bit_cast(sbf16x8, b2[0]),
                                  P3 = __builtin_bit_cast(sbf16x8, b3[0]);
                    const sbf16x8 Q1 = __builtin_bit_cast(sbf16x8, b1[1]), Q2 = __builtin_bit_cast(sbf16x8, b2[1]),
                                  Q3 = __builtin_bit_cast(sbf16x8, b3[1]);
                    floatx16 c = acc[ti * 2], d = acc[ti * 2 + 1];
                    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A2, P2, c, 0, 0, 0);
                    d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A2, Q2, d, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A3, P1, c, 0, 0, 0);
                    d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A3, Q1, d, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A1, P3, c, 0, 0, 0);
                    d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A1, Q3, d, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A2, P1, c, 0, 0, 0);
                    d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A2, Q1, d, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A1, P2, c, 0, 0, 0);
                    d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A1, Q2, d, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A1, P1, c, 0, 0, 0);
                    d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A1, Q1, d, 0, 0, 0);
                    acc[ti * 2] = c;
                    acc[ti * 2 + 1] = d;
                }
                if (ti + 1 < 4) {
#pragma unroll
                    for (int k = 0; k < 12; ++k) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
                        __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);   // four VALU
                        if (ti + 2 < 4 && k < 8) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read
                    }
                    c1 = n1; c2 = n2; c3 = n3;
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // at most the copies of the stage issued last are still on their way, then meet the other waves
        asm volatile("s_waitcnt vmcnt(6)\n\ts_barrier" ::: "memory");
    }
    // the zero-filling copies of the stages past the end may still be landing
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    if (idle || (dbg & 8)) return;

    // ---- epilogue: acc[ti*2 + tj][v] = C[m0 + wm*128 + ti*32 + 8*(v>>2) + 4*lg + (v&3)][n0 + wn*64 + tj*32 + lr]
    // A lane of the MFMA result holds single elements of many rows: written or updated from there, every memory
    // instruction moves 4 bytes per lane.  Instead each wavefront passes its part through LDS (the ring is free
    // now: 18 KB per wavefront), 32 rows x 64 columns at a time, and reads it back with 16 lanes along a row, four
    // columns each: the accesses to C are 16 bytes per lane and 256 contiguous bytes per row.  (C need not be
    // 16-byte aligned: the vector type below asks for 4.)  A chunk that the bounds of the product, the line
    // n = m + doff or the pivot rows and columns cut through takes the element-wise path further down.
    const int mw = m0 + wm * 128, nw = n0 + wn * 64;
    const long ldc = pr.ldc;
    const int p0 = pr.p0, p1 = pr.p1, doff = pr.doff;
    typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));
    constexpr int EP = 68;                                   // LDS row pitch of a chunk (floats)
    float *wl = lds + w * (S_LDS_FLOATS / 4);
    const int rr = lane >> 4, c4 = (lane & 15) * 4;
    const unsigned lane_off = (unsigned)(4 * lg) * (unsigned)pr.ldc + (unsigned)lr;
    auto row_ptr = [&](int t, int r) { return pr.C + ((long)(mw + (t >> 1) * 32 + r) * ldc + nw + (t & 1) * 32); };
    auto live = [&](int m, int n) {
        if (!lower) return m < pr.M && n < pr.N;
        return m < pr.M && n < pr.N && n <= m + doff && !(rows_skip && m >= p0 && m < p1) && !(n >= p0 && n < p1);
    };
#pragma unroll
    for (int ti = 0; ti < 4; ++ti) {
        const int mr0 = mw + ti * 32;
        bool whole = mr0 + 32 <= pr.M && nw + 64 <= pr.N;                    // uniform over the wavefront
        if (lower)
            whole = whole && nw + 63 <= mr0 + doff && !(rows_skip && mr0 < p1 && mr0 + 32 > p0) &&
                    !(nw < p1 && nw + 64 > p0);
        if (whole) {
#pragma unroll
            for (int tj = 0; tj < 2; ++tj)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    wl[(8 * (v >> 2) + 4 * lg + (v & 3)) * EP + tj * 32 + lr] = acc[ti * 2 + tj][v];
            // (LDS operations of one wavefront complete in order: no barrier between these writes and the reads)
            float *crow = pr.C + ((long)(mr0 + rr) * ldc + nw + c4);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                f4u val[4], old[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int row = 4 * (4 * h + q);      // + rr, in crow and below
                    val[q] = *reinterpret_cast<const f4u *>(wl + (row + rr) * EP + c4);
                    if (lower) old[q] = *reinterpret_cast<const f4u *>(crow + (long)row * ldc);
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int row = 4 * (4 * h + q);
                    f4u out = val[q];
                    if (lower) out = add ? old[q] + val[q] : old[q] - val[q];
                    *reinterpret_cast<f4u *>(crow + (long)row * ldc) = out;
                }
            }
            continue;
        }
        // element-wise: the 16 loads of a tile are issued together
#pragma unroll
        for (int tj = 0; tj < 2; ++tj) {
            const int t = ti * 2 + tj;
            const int n = nw + tj * 32 + lr;
            float old[16];
            if (lower) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int r = 8 * (v >> 2) + (v & 3);
                    old[v] = live(mr0 + r + 4 * lg, n) ? row_ptr(t, r)[lane_off] : 0.f;
                }
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = 8 * (v >> 2) + (v & 3);
                if (!live(mr0 + r + 4 * lg, n)) continue;
                row_ptr(t, r)[lane_off] = !lower ? acc[t][v] : (add ? old[v] + acc[t][v] : old[v] - acc[t][v]);
            }
        }
    }
}

}  // namespace kfac

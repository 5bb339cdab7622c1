// X^T X partial products for fp32 X (row-major patch matrices and linear-layer inputs, NCHW inputs of 1x1
// convolutions and output gradients) on the bf16 MFMA units at fp32 accuracy: the split-bf16 scheme of
// gemm_split.hpp (every fp32 value as three bf16 pieces, six piece products per fp32 product) applied to the
// Kronecker factors of Eq. 4 of the DP-KFAC paper.
//
// Same tiling and pipeline as gemm_split_kernel: a workgroup of four wavefronts owns a 256 x 128 tile of the
// lower triangle (256 columns of X as rows of the factor, 128 as columns) for one K slice, panels of 16 rows
// come in by buffer_load_dwordx4 ... lds in a ring of three stages, the conversions run in the shadow of the
// MFMAs.  Partial tiles go to the workspace in the 256 x 256 block layout of the bf16 kernel (two workgroup
// tiles per block), so the same reduction finishes them (fixed order, running average, mirror image).
//
// Row-major X: a stage is [16 k][columns], one copy instruction per row of the A panel, one per two rows of
// the B panel.  NCHW X (element (k = n hw + p, c) at (n ctot + c) hw + p: k runs along memory): a stage never
// crosses an image; a copy instruction moves 4 consecutive positions of 64 consecutive channels, which lands
// as [4-position group][column][4 positions] in LDS, so a lane's eight k of a column are two 16-byte reads
// without bank conflicts.  Positions past the end of an image in its last stage hold the next channel's data:
// they are cleared in the A operand registers (and in the column sums); what they meet in the B operand is finite.
//
// The bias border (column sums of X) is summed on the side, in plain fp32, by the four wavefronts of the first
// tile of every diagonal block from the A panel they already hold: 64 columns per wavefront, a lane per column.
#pragma once

#include "split_common.hpp"
#include "syrk_types.hpp"

namespace kfac {

// workgroup tiles (256 x 128) of the lower triangle of a d x d factor
__host__ __device__ inline int syrk_split_tiles(int d)
{
    const int tI = (d + S_BM - 1) / S_BM, tJ = (d + S_BN - 1) / S_BN;
    int n = 0;
    for (int i = 0; i < tI; ++i) n += (2 * i + 2 < tJ) ? 2 * i + 2 : tJ;
    return n;
}

template <int LAYOUT>
__global__ __launch_bounds__(256, 2) void syrk_split_kernel(const SyrkTable tab)
{
    __shared__ __attribute__((aligned(16))) float lds[S_LDS_FLOATS];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = w >> 1, wn = w & 1;

    // every XCD takes a contiguous range of workgroups: the tiles of a K slice, which share its panels, are
    // neighbours and meet in one L2
    const int bid = xcd_block_id();
    int pi = 0, hi = tab.count - 1;
    while (pi < hi) {
        const int mid = (pi + hi + 1) >> 1;
        if (bid >= tab.starts[mid]) pi = mid;
        else hi = mid - 1;
    }
    const SyrkProb &pr = tab.p[pi];
    const int d = pr.d;
    const int tJ = (d + S_BN - 1) / S_BN;
    const int bps = syrk_split_tiles(d);
    const int local = bid - pr.blk_start;
    const int split = local / bps;
    int rest = local - split * bps;
    int I = 0;
    for (;;) {
        const int c = min(tJ, 2 * I + 2);
        if (rest < c) break;
        rest -= c;
        ++I;
    }
    const int J = rest;
    const int m0 = I * S_BM, n0 = J * S_BN;
    const bool sums = pr.has_bias && J == 2 * I;      // first tile of a diagonal block: column sums of the A panel

    // ---- K range of this slice ----
    const long t0 = (long)split * pr.tiles_per_split;
    int nstages, tpi = 1, hw = 0, img0 = 0, kt0 = 0;
    unsigned img_bytes = 0;
    int4v rsrc;
    rsrc.w = 0x00020000;
    const int ld = (int)pr.ld;
    if (LAYOUT == kRows) {
        const long ktiles = (pr.K + S_KT - 1) / S_KT;
        const long t1 = (t0 + pr.tiles_per_split < ktiles) ? t0 + pr.tiles_per_split : ktiles;
        nstages = (int)(t1 - t0);
        const long row0 = t0 * S_KT;
        const unsigned long ba = (unsigned long)(reinterpret_cast<const float *>(pr.x) + row0 * pr.ld);
        const long bytes_left = (pr.K - row0) * pr.ld * 4;
        rsrc.x = (int)(unsigned)ba;
        rsrc.y = (int)(unsigned)(ba >> 32);
        rsrc.z = bytes_left > 0x7fffffffl ? 0x7fffffff : (int)bytes_left;
    } else {
        hw = pr.hw;
        const int nimg = (int)(pr.K / hw);
        tpi = (hw + S_KT - 1) / S_KT;
        const long ktiles = (long)nimg * tpi;
        const long t1 = (t0 + pr.tiles_per_split < ktiles) ? t0 + pr.tiles_per_split : ktiles;
        nstages = (int)(t1 - t0);
        img0 = (int)(t0 / tpi);
        kt0 = (int)(t0 - (long)img0 * tpi);
        img_bytes = (unsigned)pr.ctot * (unsigned)hw * 4u;
        const unsigned long ba = (unsigned long)pr.x;
        rsrc.x = (int)(unsigned)ba;
        rsrc.y = (int)(unsigned)(ba >> 32);
        rsrc.z = (int)((long)nimg * img_bytes);      // the host checked that the tensor is below 2 GiB
    }

    // ---- this wave's copies of a stage (six instructions) ----
    const unsigned lds_base = (unsigned)(unsigned long)(__attribute__((address_space(3))) float *)lds;
    unsigned vo[6];
    if (LAYOUT == kRows) {
        // rows 4 w .. 4 w + 3 of the A panel (64 lanes x 4 columns), then of the B panel (two rows per instruction)
        const int ca = m0 + 4 * lane, cb = n0 + 4 * (lane & 31);
        const unsigned a = ca < ld ? (unsigned)(ca * 4) : W_OOB;      // whole 16-byte pieces of the row pitch
        const unsigned b = cb < ld ? (unsigned)(((lane >> 5) * ld + cb) * 4) : W_OOB;
        vo[0] = vo[1] = vo[2] = vo[3] = a;
        vo[4] = vo[5] = b;
    } else {
        // positions 4 w .. 4 w + 3 of the stage: four groups of 64 channels of A, two of B
#pragma unroll
        for (int cg = 0; cg < 4; ++cg) {
            const int c = m0 + 64 * cg + lane;
            vo[cg] = c < d ? (unsigned)c * (unsigned)hw * 4u : W_OOB;
        }
#pragma unroll
        for (int cg = 0; cg < 2; ++cg) {
            const int c = n0 + 64 * cg + lane;
            vo[4 + cg] = c < d ? (unsigned)c * (unsigned)hw * 4u : W_OOB;
        }
    }
    // stage walk of the copies (NCHW: image and stage inside the image)
    int ii = img0, ik = kt0;
    auto issue = [&](int g) {
        const bool live_stage = g < nstages;
        const unsigned buf = lds_base + (unsigned)((g % S_NSTAGE) * S_STAGE * 4);
        if (LAYOUT == kRows) {
            const unsigned k0 = (unsigned)(g * S_KT + 4 * w);
            const unsigned row = (unsigned)ld * 4u;
#pragma unroll
            for (int r = 0; r < 4; ++r)
                dma16(buf + (unsigned)((4 * w + r) * S_BM * 4), live_stage ? vo[r] : W_OOB, rsrc,
                      live_stage ? (k0 + r) * row : 0u);
#pragma unroll
            for (int r = 0; r < 2; ++r)
                dma16(buf + (unsigned)((S_PANEL_A + (4 * w + 2 * r) * S_BN) * 4), live_stage ? vo[4 + r] : W_OOB, rsrc,
                      live_stage ? (k0 + 2 * r) * row : 0u);
        } else {
            const unsigned so = (unsigned)ii * img_bytes + (unsigned)((ik * S_KT + 4 * w) * 4);
#pragma unroll
            for (int cg = 0; cg < 4; ++cg)
                dma16(buf + (unsigned)((w * S_BM + 64 * cg) * 16), live_stage ? vo[cg] : W_OOB, rsrc, live_stage ? so : 0u);
#pragma unroll
            for (int cg = 0; cg < 2; ++cg)
                dma16(buf + (unsigned)(S_PANEL_A * 4 + (w * S_BN + 64 * cg) * 16), live_stage ? vo[4 + cg] : W_OOB, rsrc,
                      live_stage ? so : 0u);
            if (++ik == tpi) { ik = 0; ++ii; }
        }
    };

    floatx16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    float csum = 0.f;

    const int lr = lane & 31, lg = lane >> 5;
    // a wave whose 128 x 64 part lies wholly above the diagonal has nothing to multiply
    const bool idle = n0 + wn * 64 > m0 + wm * 128 + 127;
    const int ca0 = wm * 128 + lr, cb0 = wn * 64 + lr;      // the lane's column in the first tile of each operand

    // eight k of column `col` (+ 32 t) of a panel: k = 8 lg .. 8 lg + 7
    auto read8 = [&](const float *panel, int pitch, int col, float (&x)[8]) {
        if (LAYOUT == kRows) {
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] = panel[(8 * lg + e) * pitch + col];
        } else {
            const floatx4 lo = *reinterpret_cast<const floatx4 *>(panel + ((2 * lg) * pitch + col) * 4);
            const floatx4 hi2 = *reinterpret_cast<const floatx4 *>(panel + ((2 * lg + 1) * pitch + col) * 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) { x[e] = lo[e]; x[4 + e] = hi2[e]; }
        }
    };

    int ck = kt0;                      // NCHW: stage inside the image of the stage being multiplied
    issue(0);
    issue(1);
    asm volatile("s_waitcnt vmcnt(6)\n\ts_barrier" ::: "memory");
    for (int g = 0; g < nstages; ++g) {
        issue(g + 2);        // into the buffer every wave left at the last barrier (stages past the end: zeros)
        const float *buf = lds + (g % S_NSTAGE) * S_STAGE;
        // NCHW: valid positions of this stage (16 except in the last stage of an image)
        const int valid = (LAYOUT == kNCHW) ? min(S_KT, hw - ck * S_KT) : S_KT;
        if (LAYOUT == kNCHW && ++ck == tpi) ck = 0;
        if (sums) {
            // column 64 w + lane of the A panel, all 16 k
            const int col = 64 * w + lane;
            if (LAYOUT == kRows) {
#pragma unroll
                for (int k = 0; k < S_KT; ++k) csum += buf[k * S_BM + col];
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const floatx4 v4 = *reinterpret_cast<const floatx4 *>(buf + (q * S_BM + col) * 4);
#pragma unroll
                    for (int e = 0; e < 4; ++e) csum += (4 * q + e < valid) ? v4[e] : 0.f;
                }
            }
        }
        if (!idle) {
            suint4 b1[2], b2[2], b3[2];
            float xa[8], xn[8];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                float x[8];
                read8(buf + S_PANEL_A, S_BN, cb0 + t * 32, x);
                if (t == 0) read8(buf, S_BM, ca0, xa);
                else read8(buf, S_BM, ca0 + 32, xn);
                split_pieces(x, b1[t], b2[t], b3[t]);
            }
            if (LAYOUT == kNCHW && valid < S_KT) {
#pragma unroll
                for (int e = 0; e < 8; ++e) xa[e] = (8 * lg + e < valid) ? xa[e] : 0.f;
            }
            suint4 c1, c2, c3;          // pieces of the A tile being multiplied
            split_pieces(xa, c1, c2, c3);
            __builtin_amdgcn_sched_barrier(0);
            // Tile ti: its twelve products, with the conversions of tile ti + 1 (and the panel reads of tile
            // ti + 2) issued between them, four VALU operations in the shadow of every MFMA.
#pragma unroll
            for (int ti = 0; ti < 4; ++ti) {
                suint4 n1, n2, n3;
                if (ti + 1 < 4) {
                    if (LAYOUT == kNCHW && valid < S_KT) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) xn[e] = (8 * lg + e < valid) ? xn[e] : 0.f;
                    }
                    split_pieces(xn, n1, n2, n3);
                }
                if (ti + 2 < 4) read8(buf, S_BM, ca0 + (ti + 2) * 32, xn);
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

    // ---- partial tile -> block (bi, bj) = (I, J / 2) of the slice, columns 128 (J & 1) .. of the block ----
    const int nblk = pr.nb * (pr.nb + 1) / 2;
    if (sums) {
        float *cs = pr.partial + (long)pr.splits * nblk * (S_BM * S_BM);
        cs[((long)split * pr.nb + I) * S_BM + 64 * w + lane] = csum;
    }
    if (idle) return;
    const int blk = I * (I + 1) / 2 + (J >> 1);
    // Each wavefront passes its 128 x 64 part through LDS (the ring is free now), 32 rows at a time, and reads it
    // back with 16 lanes along a row: the stores are 16 bytes per lane and 256 contiguous bytes per row instead of
    // 4 bytes per lane.  (LDS operations of one wavefront complete in order: no barrier between writes and reads.)
    float *dst = pr.partial + ((long)split * nblk + blk) * (S_BM * S_BM) + (J & 1) * S_BN + wn * 64;
    constexpr int EP = 68;                                   // LDS row pitch of a chunk (floats)
    float *wl = lds + w * (S_LDS_FLOATS / 4);
    const int rr = lane >> 4, c4 = (lane & 15) * 4;
#pragma unroll
    for (int ti = 0; ti < 4; ++ti) {
#pragma unroll
        for (int tj = 0; tj < 2; ++tj)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                wl[(8 * (v >> 2) + 4 * lg + (v & 3)) * EP + tj * 32 + lr] = acc[ti * 2 + tj][v];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int row = 4 * q + rr;
            const floatx4 val = *reinterpret_cast<const floatx4 *>(wl + row * EP + c4);
            *reinterpret_cast<floatx4 *>(dst + (long)(wm * 128 + ti * 32 + row) * S_BM + c4) = val;
        }
    }
}

}  // namespace kfac

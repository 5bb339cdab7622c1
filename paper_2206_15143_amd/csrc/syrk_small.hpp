// Factor of a narrow NCHW operand (conv output gradients with d <= 64 channels): G = X^T X where
// X^T is stored [image][channel][position], i.e. K is contiguous.  The work is bound by reading X
// once, so there is no LDS staging: lane (lr, lk) of a wave ends up with 16 bytes = four consecutive
// positions of channel 16*t + lr, and the four components feed four MFMAs.  That is legal because
// a symmetric product only needs both operands to agree on which K element sits where (here the
// same register is both operands).  The load itself is issued in a memory-friendly lane order (four
// adjacent lanes read the 64 contiguous bytes of one channel) and a cross-lane permutation
// (ds_bpermute, no memory traffic) brings the pieces to the lanes the MFMA layout wants.  Each wave walks its own range of 16-position groups with the
// loads of the next groups in flight, the four waves of a block add up through LDS and the block
// writes one partial tile for the split reduction.
#pragma once

#include "tn_engine.hpp"

namespace kfac {

template <int NTL>   // 16-wide channel tiles (d <= 16 * NTL)
__global__ __launch_bounds__(256) void syrk_small_nchw_kernel(const SyrkTable tab)
{
    constexpr int BM = NTL <= 2 ? 32 : 64;      // partial tile pitch expected by the reduction kernel
    constexpr int NACC = NTL * (NTL + 1) / 2;
    constexpr int DEPTH = NTL <= 2 ? 8 : 4;      // groups of loads in flight per wave
    __shared__ float red[3][NACC * 256];

    const int tid = threadIdx.x;
    const int lane = tid & 63, w = tid >> 6;
    const int lr = lane & 15, lk = lane >> 4;

    int pi = 0;
    while (pi + 1 < tab.count && (int)blockIdx.x >= tab.p[pi + 1].blk_start) ++pi;
    const SyrkProb &pr = tab.p[pi];
    const int split = blockIdx.x - pr.blk_start;
    const float *x = reinterpret_cast<const float *>(pr.x);
    const int hw = pr.hw, d = pr.d;
    const long nimg = pr.K / hw;
    const int gpi = (hw + 15) / 16;              // 16-position groups per image
    const long groups = nimg * gpi;
    // this block's groups, dealt to its four waves in contiguous quarters
    const long g0 = (long)split * pr.tiles_per_split;
    const long g1 = (g0 + pr.tiles_per_split < groups) ? g0 + pr.tiles_per_split : groups;
    const long per = (g1 - g0 + 3) / 4;
    long gb = g0 + w * per;
    long ge = (gb + per < g1) ? gb + per : g1;
    if (gb > ge) gb = ge;

    floatx4 acc[NACC];
#pragma unroll
    for (int i = 0; i < NACC; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};

    // (image, group-in-image) of the next group to fetch
    long n = gb / gpi;
    int gi = (int)(gb - n * gpi);
    // load order: lane l reads piece l & 3 (positions 4*(l&3)..+3) of channel l >> 2; the MFMA lane
    // (lr, lk) = lane lk*16 + lr needs piece lk of channel lr, i.e. the data of load lane lr*4 + lk
    const int lc = lane >> 2, lq = lane & 3;
    const int src_byte = (lr * 4 + lk) * 4;
    auto fetch = [&](floatx4 (&v)[NTL]) {
        const int p = gi * 16 + 4 * lq;
#pragma unroll
        for (int t = 0; t < NTL; ++t) {
            const int c = t * 16 + lc;
            v[t] = floatx4{0.f, 0.f, 0.f, 0.f};
            if (c < d && p < hw) v[t] = *reinterpret_cast<const floatx4 *>(x + (n * pr.ctot + c) * (long)hw + p);
        }
        if (++gi == gpi) { gi = 0; ++n; }
    };
    auto to_mfma_lanes = [&](floatx4 (&v)[NTL]) {
#pragma unroll
        for (int t = 0; t < NTL; ++t)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                v[t][e] = __int_as_float(__builtin_amdgcn_ds_bpermute(src_byte, __float_as_int(v[t][e])));
    };
    auto mma = [&](const floatx4 (&v)[NTL]) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int ti = 0; ti < NTL; ++ti)
#pragma unroll
                for (int tj = 0; tj <= ti; ++tj)
                    acc[ti * (ti + 1) / 2 + tj] =
                        __builtin_amdgcn_mfma_f32_16x16x4f32(v[ti][e], v[tj][e], acc[ti * (ti + 1) / 2 + tj], 0, 0, 0);
    };

    floatx4 buf[DEPTH][NTL];
    const long cnt = ge - gb;
    // software pipeline: DEPTH groups of loads are always in flight
#pragma unroll
    for (int s = 0; s < DEPTH; ++s) {
        if (s < cnt) fetch(buf[s]);
    }
    long done = 0;
    for (; done + DEPTH <= cnt; done += DEPTH) {
#pragma unroll
        for (int s = 0; s < DEPTH; ++s) {
            floatx4 cur[NTL];
#pragma unroll
            for (int t = 0; t < NTL; ++t) cur[t] = buf[s][t];
            if (done + DEPTH + s < cnt) fetch(buf[s]);
            to_mfma_lanes(cur);
            mma(cur);
        }
    }
#pragma unroll
    for (int s = 0; s < DEPTH; ++s) {
        if (done + s < cnt) {
            to_mfma_lanes(buf[s]);
            mma(buf[s]);
        }
    }

    // add the four waves (fixed order) and write the block's partial tile, row-major BM x BM
    if (w > 0) {
#pragma unroll
        for (int i = 0; i < NACC; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v) red[w - 1][(i * 4 + v) * 64 + lane] = acc[i][v];
    }
    __syncthreads();
    if (w == 0) {
        float *dst = pr.partial + (long)split * (BM * BM);
#pragma unroll
        for (int ti = 0; ti < NTL; ++ti)
#pragma unroll
            for (int tj = 0; tj <= ti; ++tj) {
                const int i = ti * (ti + 1) / 2 + tj;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    float s = acc[i][v];
                    s += red[0][(i * 4 + v) * 64 + lane];
                    s += red[1][(i * 4 + v) * 64 + lane];
                    s += red[2][(i * 4 + v) * 64 + lane];
                    dst[(ti * 16 + 4 * lk + v) * BM + tj * 16 + lr] = s;
                }
            }
    }
}

}  // namespace kfac

// Factor of a narrow NCHW operand (conv output gradients with d <= 64 channels): G = X^T X where
// X^T is stored [image][channel][position], i.e. K is contiguous.  The work is bound by reading X
// once, so there is no LDS staging: lane (lr, lk) of a wave ends up with 16 bytes = four consecutive
// positions of channel 16*t + lr, and the four components feed four MFMAs.  That is legal because
// a symmetric product only needs both operands to agree on which K element sits where (here the
// same register is both operands).  K is walked in groups of 32 positions.  The loads are issued in a
// memory-friendly lane order: eight adjacent lanes read the 128 contiguous bytes (one cache line) that a
// channel has in the group, so one load covers eight channels and two loads a 16-channel tile; the second
// load swaps its two 64-byte halves between the lanes.  With that swap the lanes that hold the first
// half of the group are the low four of every eight in one load and the high four in the other: one
// select per register merges "this half of the group, all 16 channels" into a single register, and a
// cross-lane permutation (ds_bpermute, no memory traffic) brings the pieces to the lanes the MFMA layout
// wants.  Each wave walks its own range of groups with the loads of the next groups in flight, the four
// waves of a block add up through LDS and the block writes one partial tile for the split reduction.
#pragma once

#include "tn_engine.hpp"

namespace kfac {

constexpr int S_GROUP = 32;   // positions per group (the host plans the splits in these units)

template <int NTL>   // 16-wide channel tiles (d <= 16 * NTL)
__global__ __launch_bounds__(256) void syrk_small_nchw_kernel(const SyrkTable tab)
{
    constexpr int BM = NTL <= 2 ? 32 : 64;      // partial tile pitch expected by the reduction kernel
    constexpr int NACC = NTL * (NTL + 1) / 2;
    constexpr int DEPTH = NTL <= 2 ? 4 : 2;      // groups of loads in flight per wave
    __shared__ float red[3][NACC * 256];

    const int tid = threadIdx.x;
    const int lane = tid & 63, w = tid >> 6;
    const int lr = lane & 15, lk = lane >> 4;

    int pi = 0, hi = tab.count - 1;
    while (pi < hi) {
        const int mid = (pi + hi + 1) >> 1;
        if ((int)blockIdx.x >= tab.starts[mid]) pi = mid;
        else hi = mid - 1;
    }
    const SyrkProb &pr = tab.p[pi];
    const int split = blockIdx.x - pr.blk_start;
    const float *x = reinterpret_cast<const float *>(pr.x);
    const int hw = pr.hw, d = pr.d;
    const long nimg = pr.K / hw;
    const int gpi = (hw + S_GROUP - 1) / S_GROUP;   // groups per image
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
    // load order: lane l reads a 16-byte piece of channel (l >> 3) [first load] or 8 + (l >> 3) [second load] of
    // the tile: piece l & 7 in the first load, (l & 7) ^ 4 in the second.  The MFMA lane (lr, lk) needs, for the
    // half j of the group, piece lk + 4 j of channel lr: that is lane 8 lr + lk + 4 j of the first load when
    // lr < 8, and lane 8 (lr - 8) + lk + 4 (1 - j) of the second load otherwise.  For either half those source
    // lanes are the low four of eight in one load and the high four in the other.
    const int lc = lane >> 3, lq = lane & 7;
    const bool low = lq < 4;
    const int src0 = ((lr < 8 ? 8 * lr + lk : 8 * (lr - 8) + lk + 4)) * 4;       // half 0, byte address for bpermute
    const int src1 = ((lr < 8 ? 8 * lr + lk + 4 : 8 * (lr - 8) + lk)) * 4;       // half 1
    // Every load is issued unconditionally, from an address clamped into the image: what a lane must not
    // contribute (a channel past d, a position past the end of the map in a ragged last group) is zeroed
    // when the group is consumed.  Loads under a condition would cost the prefetch: the compiler can only
    // count in-flight loads that are certain to have been issued, and waits for all of them otherwise.
    bool cv0[NTL], cv1[NTL];                 // this lane's channel of the first / second load exists
    unsigned co0[NTL], co1[NTL];             // element offset of that channel's row in the image (clamped)
#pragma unroll
    for (int t = 0; t < NTL; ++t) {
        const int c0 = t * 16 + lc, c1 = c0 + 8;
        cv0[t] = c0 < d;
        cv1[t] = c1 < d;
        co0[t] = (unsigned)((c0 < d ? c0 : d - 1) * hw);
        co1[t] = (unsigned)((c1 < d ? c1 : d - 1) * hw);
    }
    // returns the number of positions the group has (32, fewer in a ragged last group of an image)
    auto fetch = [&](floatx4 (&v)[NTL][2]) -> int {
        const float *img = x + n * pr.ctot * (long)hw;
        const int p0 = gi * S_GROUP + 4 * lq, p1 = gi * S_GROUP + 4 * (lq ^ 4);
        const unsigned q0 = (unsigned)(p0 < hw ? p0 : hw - 4), q1 = (unsigned)(p1 < hw ? p1 : hw - 4);
#pragma unroll
        for (int t = 0; t < NTL; ++t) {
            v[t][0] = *reinterpret_cast<const floatx4 *>(img + (co0[t] + q0));
            v[t][1] = *reinterpret_cast<const floatx4 *>(img + (co1[t] + q1));
        }
        const int left = hw - gi * S_GROUP;
        if (++gi == gpi) { gi = 0; ++n; }
        return left;
    };
    // v: the two loads per tile; o: the two halves of the group per tile, in MFMA lane order
    auto to_mfma_lanes = [&](const floatx4 (&v)[NTL][2], int left, floatx4 (&o)[NTL][2]) {
        const bool okp0 = 4 * lq < left, okp1 = 4 * (lq ^ 4) < left;
#pragma unroll
        for (int t = 0; t < NTL; ++t) {
            const bool ok0 = cv0[t] && okp0, ok1 = cv1[t] && okp1;
            const bool m0 = low ? ok0 : ok1, m1 = low ? ok1 : ok0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float h0 = low ? v[t][0][e] : v[t][1][e];
                float h1 = low ? v[t][1][e] : v[t][0][e];
                h0 = m0 ? h0 : 0.f;
                h1 = m1 ? h1 : 0.f;
                o[t][0][e] = __int_as_float(__builtin_amdgcn_ds_bpermute(src0, __float_as_int(h0)));
                o[t][1][e] = __int_as_float(__builtin_amdgcn_ds_bpermute(src1, __float_as_int(h1)));
            }
        }
    };
    auto mma = [&](const floatx4 (&v)[NTL][2]) {
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int ti = 0; ti < NTL; ++ti)
#pragma unroll
                    for (int tj = 0; tj <= ti; ++tj)
                        acc[ti * (ti + 1) / 2 + tj] = __builtin_amdgcn_mfma_f32_16x16x4f32(
                            v[ti][j][e], v[tj][j][e], acc[ti * (ti + 1) / 2 + tj], 0, 0, 0);
    };

    floatx4 buf[DEPTH][NTL][2];
    int left[DEPTH];
    const long cnt = ge - gb;
    long done = 0;
    // software pipeline: DEPTH groups of loads are always in flight.  The long ranges run a prologue and a
    // steady loop without any condition around a fetch (see above); what remains takes the general loop.
    if (cnt >= 2 * DEPTH) {
#pragma unroll
        for (int s = 0; s < DEPTH; ++s) {
            left[s] = fetch(buf[s]);
            __builtin_amdgcn_sched_barrier(0);      // issued in the order the loop consumes them
        }
        for (; done + 2 * DEPTH <= cnt; done += DEPTH) {
#pragma unroll
            for (int s = 0; s < DEPTH; ++s) {
                // the registers of the set are free for the next loads once the permutation has read them
                floatx4 cur[NTL][2];
                to_mfma_lanes(buf[s], left[s], cur);
                left[s] = fetch(buf[s]);
                mma(cur);
                // keep the groups in program order: hoisting the permutations of the later sets to the top of
                // the iteration would make it wait for every load in flight
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    } else {
#pragma unroll
        for (int s = 0; s < DEPTH; ++s) {
            left[s] = 0;
            if (s < cnt) left[s] = fetch(buf[s]);
        }
    }
    for (; done + DEPTH <= cnt; done += DEPTH) {
#pragma unroll
        for (int s = 0; s < DEPTH; ++s) {
            floatx4 cur[NTL][2];
            to_mfma_lanes(buf[s], left[s], cur);
            if (done + DEPTH + s < cnt) left[s] = fetch(buf[s]);
            mma(cur);
        }
    }
#pragma unroll
    for (int s = 0; s < DEPTH; ++s) {
        if (done + s < cnt) {
            floatx4 cur[NTL][2];
            to_mfma_lanes(buf[s], left[s], cur);
            mma(cur);
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

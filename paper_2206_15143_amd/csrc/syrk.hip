// Kronecker-factor construction (Eq. 4 of the DP-KFAC paper) with the running
// average of Eqs. 10-11 fused into the reduction epilogue:
//
//     F <- decay * F + (1 - decay) * scale * X^T X          (lower triangle, mirrored)
//
// and, for layers with a bias, the border of the homogeneous column
// (F[d][c] = column sums of X, F[d][d] = number of rows) computed on the side
// from the values the loader already holds, so the ones column is never
// materialised and the MFMA tiles stay multiples of 16.
//
// Every factor goes through a partial-product kernel (lower-triangular tiles x
// split-K slices, partial tiles to the workspace) and the reduction kernel:
//   syrk_partial_kernel    : block-tile fp32 MFMA kernel, any layout / dtype (this file)
//   syrk_wave_kernel       : wave-unit kernel, row-major fp32 (syrk_wave.hpp)
//   syrk_wave_nchw_kernel  : wave-unit kernel, wide NCHW fp32 (syrk_wave.hpp)
//   syrk_conv3_kernel      : 3x3 convolution inputs, patch matrix never built (syrk_conv3.hpp)
//   syrk_small_nchw_kernel : narrow NCHW fp32, no LDS staging (syrk_small.hpp)
//   syrk_bf16_kernel       : bf16 inputs on the bf16 MFMA units (syrk_bf16.hpp)
//   syrk_split_kernel      : wide fp32 inputs as three bf16 pieces on the bf16 MFMA units (syrk_split.hpp)
//   syrk_reduce_kernel     : sums the slices in a fixed order (deterministic), applies scale and
//                            the running average, writes both triangles.
// The planner below picks the kernel and the split of K per factor and groups
// equal choices into launches of up to 40 factors.
#include <type_traits>
#include "tn_engine.hpp"

#include <algorithm>
#include <cmath>

#include "syrk_wave.hpp"
#include "syrk_conv3.hpp"
#include "syrk_corr3.hpp"
#include "syrk_small.hpp"
#include "syrk_bf16.hpp"
#include "syrk_split.hpp"

namespace kfac {

template <class T, int LAYOUT, int DT>
__global__ __launch_bounds__(T::NT) void syrk_partial_kernel(const SyrkTable tab)
{
    __shared__ float lds[2][2][T::PANEL];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / T::NW, wn = wave % T::NW;

    int pi = 0;
    while (pi + 1 < tab.count && (int)blockIdx.x >= tab.p[pi + 1].blk_start) ++pi;
    const SyrkProb &pr = tab.p[pi];
    const int local = blockIdx.x - pr.blk_start;
    const int nblk = pr.nb * (pr.nb + 1) / 2;
    const int split = local / nblk;
    const int blk = local - split * nblk;
    int bi, bj;
    tri_decode(blk, bi, bj);
    const bool diag = (bi == bj);
    const bool do_colsum = pr.has_bias && bj == 0;

    Operand op;
    op.x = pr.x; op.K = pr.K; op.ld = pr.ld; op.d = pr.d; op.hw = pr.hw; op.ctot = pr.ctot; op.vec = pr.vec;

    const long ktiles = (pr.K + T::KT - 1) / T::KT;
    const long t0 = (long)split * pr.tiles_per_split;
    const long t1 = (t0 + pr.tiles_per_split < ktiles) ? t0 + pr.tiles_per_split : ktiles;

    floatx4 acc[T::WT][T::WT];
#pragma unroll
    for (int i = 0; i < T::WT; ++i)
#pragma unroll
        for (int j = 0; j < T::WT; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};

    floatx4 cs[T::PASSES];
#pragma unroll
    for (int p = 0; p < T::PASSES; ++p) cs[p] = floatx4{0.f, 0.f, 0.f, 0.f};

    const int u0 = bi * T::BM, v0 = bj * T::BM;
    const bool active = !diag || wn <= wm;
    const bool tri = diag && wn == wm;

    if constexpr (LAYOUT == kRows && T::BM <= 64) {
        // Small tiles, row-major operand: a few workgroups walk a long K with little work per stage, so the loop
        // is bound by the latency of its loads.  The panels are fetched D stages ahead into a ring of register
        // sets; every load is unconditional (clamped address, zeroed before use) and the shape of the loop
        // (vector or scalar loads, one panel or two) is fixed at compile time, so that the compiler can count
        // the loads in flight and wait for the oldest set only.
        constexpr int D = 3;
        auto k_loop = [&](auto vec_c, auto diag_c) {
            constexpr bool VEC = decltype(vec_c)::value, DG = decltype(diag_c)::value;
            floatx4 su[D][T::PASSES], sv[D][T::PASSES];
#pragma unroll
            for (int r = 0; r < D; ++r) {
                fetch_rows_clamped<T, DT, VEC>(su[r], op, (t0 + r) * T::KT, u0, tid);
                if (!DG) fetch_rows_clamped<T, DT, VEC>(sv[r], op, (t0 + r) * T::KT, v0, tid);
                __builtin_amdgcn_sched_barrier(0);      // issued in the order the loop consumes them
            }
            auto stage_in = [&](floatx4 (&pu)[T::PASSES], floatx4 (&pv)[T::PASSES], long t, int buf) {
                mask_rows<T>(pu, op, t * T::KT, u0, tid);
                if (do_colsum) {
#pragma unroll
                    for (int p = 0; p < T::PASSES; ++p) cs[p] += pu[p];
                }
                commit_panel<T, kRows>(pu, lds[buf][0], tid);
                if (!DG) {
                    mask_rows<T>(pv, op, t * T::KT, v0, tid);
                    commit_panel<T, kRows>(pv, lds[buf][1], tid);
                }
            };
            stage_in(su[0], sv[0], t0, 0);
            __syncthreads();
            for (long tb = t0; tb < t1; tb += D) {
#pragma unroll
                for (int r = 0; r < D; ++r) {
                    const long t = tb + r;
                    if (t >= t1) break;
                    const int cur = (int)((t - t0) & 1);
                    // stages past the split (or past K) are read from clamped rows and never used
                    fetch_rows_clamped<T, DT, VEC>(su[r], op, (t + D) * T::KT, u0, tid);
                    if (!DG) fetch_rows_clamped<T, DT, VEC>(sv[r], op, (t + D) * T::KT, v0, tid);
                    if (active) {
                        const float *Us = lds[cur][0];
                        const float *Vs = DG ? lds[cur][0] : lds[cur][1];
                        if (tri)
                            mma_stage<T, LAYOUT, LAYOUT, true>(Us, Vs, wm, wn, lane, acc);
                        else
                            mma_stage<T, LAYOUT, LAYOUT, false>(Us, Vs, wm, wn, lane, acc);
                    }
                    if (t + 1 < t1) stage_in(su[(r + 1) % D], sv[(r + 1) % D], t + 1, cur ^ 1);
                    __syncthreads();
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        };
        if (t0 < t1) {
            if (op.vec) {
                if (diag) k_loop(std::true_type{}, std::true_type{});
                else k_loop(std::true_type{}, std::false_type{});
            } else {
                if (diag) k_loop(std::false_type{}, std::true_type{});
                else k_loop(std::false_type{}, std::false_type{});
            }
        }
    } else {
        floatx4 su[T::PASSES], sv[T::PASSES];
        if (t0 < t1) {
            fetch_panel<T, LAYOUT, DT>(su, op, t0 * T::KT, u0, tid);
            if (!diag) fetch_panel<T, LAYOUT, DT>(sv, op, t0 * T::KT, v0, tid);
            if (do_colsum) {
    #pragma unroll
                for (int p = 0; p < T::PASSES; ++p) cs[p] += su[p];
            }
            commit_panel<T, LAYOUT>(su, lds[0][0], tid);
            if (!diag) commit_panel<T, LAYOUT>(sv, lds[0][1], tid);
        }
        __syncthreads();

        for (long t = t0; t < t1; ++t) {
            const int cur = (int)((t - t0) & 1);
            const bool more = (t + 1 < t1);
            if (more) {
                fetch_panel<T, LAYOUT, DT>(su, op, (t + 1) * T::KT, u0, tid);
                if (!diag) fetch_panel<T, LAYOUT, DT>(sv, op, (t + 1) * T::KT, v0, tid);
            }
            if (active) {
                const float *Us = lds[cur][0];
                const float *Vs = diag ? lds[cur][0] : lds[cur][1];
                if (tri)
                    mma_stage<T, LAYOUT, LAYOUT, true>(Us, Vs, wm, wn, lane, acc);
                else
                    mma_stage<T, LAYOUT, LAYOUT, false>(Us, Vs, wm, wn, lane, acc);
            }
            if (more) {
                if (do_colsum) {
    #pragma unroll
                    for (int p = 0; p < T::PASSES; ++p) cs[p] += su[p];
                }
                commit_panel<T, LAYOUT>(su, lds[cur ^ 1][0], tid);
                if (!diag) commit_panel<T, LAYOUT>(sv, lds[cur ^ 1][1], tid);
            }
            __syncthreads();
        }

    }

    // ---- partial tile out ----
    if (active) {
        float *dst = pr.partial + ((long)split * nblk + blk) * (T::BM * T::BM);
        const int lr = lane & 15, lk = lane >> 4;
#pragma unroll
        for (int ti = 0; ti < T::WT; ++ti)
#pragma unroll
            for (int tj = 0; tj < T::WT; ++tj) {
                if (tri && tj > ti) continue;
                const int row = (wm * T::WT + ti) * 16 + 4 * lk;
                const int col = (wn * T::WT + tj) * 16 + lr;
#pragma unroll
                for (int v = 0; v < 4; ++v) dst[(row + v) * T::BM + col] = acc[ti][tj][v];
            }
    }

    // ---- column sums of the U panel (bias border) ----
    if (do_colsum) {
        float *red = &lds[0][0][0];   // all waves are past the last barrier of the K loop
        constexpr int SLOTS = (LAYOUT == kRows) ? T::NT / (T::BM / 4) : T::KT / 4;
#pragma unroll
        for (int p = 0; p < T::PASSES; ++p) {
            const int idx = tid + p * T::NT;
            if (LAYOUT == kRows) {
                // every pass of a thread hits the same column group
                if (p > 0) cs[0] += cs[p];
            } else if (idx < T::V4) {
                const int c = idx / (T::KT / 4), kq = idx % (T::KT / 4);
                red[kq * T::BM + c] = cs[p].x + cs[p].y + cs[p].z + cs[p].w;
            }
        }
        if (LAYOUT == kRows) {
            const int slot = tid / (T::BM / 4);
            const int c = (tid % (T::BM / 4)) * 4;
            red[slot * T::BM + c + 0] = cs[0].x;
            red[slot * T::BM + c + 1] = cs[0].y;
            red[slot * T::BM + c + 2] = cs[0].z;
            red[slot * T::BM + c + 3] = cs[0].w;
        }
        __syncthreads();
        if (tid < T::BM) {
            float s = 0.f;
#pragma unroll
            for (int k = 0; k < SLOTS; ++k) s += red[k * T::BM + tid];
            float *csum = pr.partial + (long)pr.splits * nblk * (T::BM * T::BM);
            csum[((long)split * pr.nb + bi) * T::BM + tid] = s;
        }
    }
}

// Split reduction + running average.  Each block owns kRedGroup 16 x 16 sub-tiles
// of one BM x BM tile of the lower triangle (plus, with a bias, one block per
// block row for the border).  Fixed summation order over the splits.
constexpr int kRedChunk = 256;
constexpr int kRedGroup = 4;   // sub-tiles per block

// NATIVE: the partial tiles are stored as the MFMA accumulators lie in registers (per 16x16 tile
// [lane][4], tiles row-major inside the 144-wide macro tile), which lets the wave kernels store
// 16 bytes per lane; element e of a macro tile then maps to row / column as decoded below.
template <class T, bool NATIVE>
__device__ __forceinline__ void syrk_reduce_body(const SyrkProb &pr, int local, float (*mir)[16][17])
{
    const int nblk = pr.nb * (pr.nb + 1) / 2;
    const int dF = pr.d + pr.has_bias;
    const float wnew = (1.0f - pr.decay) * pr.scale;
    constexpr int TILE = T::BM * T::BM;
    constexpr int CPT = (TILE + kRedChunk - 1) / kRedChunk;   // chunks per tile

    constexpr int GPT = (CPT + kRedGroup - 1) / kRedGroup;    // blocks per tile
    if constexpr (T::BM == 256 && !NATIVE) {
        // 256-wide tiles (the bf16 MFMA kernels: the factors with the most slices).  The kRedGroup sub-tiles of a
        // block lie side by side, 16 rows x 64 columns of the tile: thread t takes four consecutive columns of
        // row t / 16, so a slice is read with 16 bytes per lane and 256 contiguous bytes per row, eight slices
        // in flight.  (The partial tiles are allocated whole: a vector that straddles the diagonal or the edge
        // of the factor reads defined or stale words, and only live elements are used.)
        if (local < nblk * GPT) {
            static_assert(kRedGroup == 4 && kRedChunk == 256, "the strip of a block is 16 x 64");
            float(*tr)[65] = reinterpret_cast<float(*)[65]>(&mir[0][0][0]);    // 16 x 65 <= 4 x 16 x 17
            const int tile = local / GPT;
            const int grp = local - tile * GPT;
            int bi, bj;
            tri_decode(tile, bi, bj);
            const float *src = pr.partial + (long)tile * TILE;
            const long sstride = (long)nblk * TILE;
            const int t = threadIdx.x;
            const int r = t >> 4, c4 = (t & 15) * 4;
            const int sr = grp >> 2, c0 = (grp & 3) * 64;
            const int u = bi * 256 + sr * 16 + r, v0 = bj * 256 + c0 + c4;
            const int e = (sr * 16 + r) * 256 + c0 + c4;
            const bool any = u < pr.d && v0 <= u;         // some element of the four is in the lower triangle
            floatx4 sum = {0.f, 0.f, 0.f, 0.f};
            if (any) {
                if (pr.splits == 1) {
                    sum = *reinterpret_cast<const floatx4 *>(src + e);
                } else {
                    floatx4 a[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) a[j] = floatx4{0.f, 0.f, 0.f, 0.f};
                    int k = 0;
                    for (; k + 8 <= pr.splits; k += 8) {
#pragma unroll
                        for (int j = 0; j < 8; ++j) a[j] += *reinterpret_cast<const floatx4 *>(src + (k + j) * sstride + e);
                    }
                    for (; k < pr.splits; ++k) a[0] += *reinterpret_cast<const floatx4 *>(src + k * sstride + e);
#pragma unroll
                    for (int h = 4; h > 0; h >>= 1)
#pragma unroll
                        for (int j = 0; j < h; ++j) a[j] += a[j + h];
                    sum = a[0];
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int v = v0 + i;
                float out = 0.f;
                if (any && v <= u) {
                    out = pr.decay * pr.F[(long)u * dF + v] + wnew * sum[i];
                    pr.F[(long)u * dF + v] = out;
                }
                tr[r][c4 + i] = out;
            }
            __syncthreads();
            // the mirror image, along rows of F: thread t writes row (column of the strip) t / 16 + 16 j
            const int r2 = t & 15;
            const int u2 = bi * 256 + sr * 16 + r2;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int cc = (t >> 4) + 16 * j;
                const int v2 = bj * 256 + c0 + cc;
                if (u2 < pr.d && v2 < u2) pr.F[(long)v2 * dF + u2] = tr[r2][cc];
            }
            return;
        }
    }
    if (local < nblk * GPT) {
        // kRedGroup 16 x 16 sub-tiles per block: thread t holds one element of each; all loads are issued
        // before the first store.  The mirror image goes through LDS so that both stores run along rows of F.
        const int tile = local / GPT;
        const int grp = local - tile * GPT;
        int bi, bj;
        tri_decode(tile, bi, bj);
        const float *src = pr.partial + (long)tile * TILE;
        const long sstride = (long)nblk * TILE;
        constexpr int S = T::BM / 16;            // sub-tiles per tile side
        const int t = threadIdx.x;
        int r, c;
        if (NATIVE) {
            const int ln = t >> 2, vv = t & 3;
            r = 4 * (ln >> 4) + vv;
            c = ln & 15;
        } else {
            r = t >> 4;
            c = t & 15;
        }
        float sum[kRedGroup], old[kRedGroup];
        bool live[kRedGroup];
#pragma unroll
        for (int q = 0; q < kRedGroup; ++q) {
            const int chunk = grp * kRedGroup + q;
            const int sr = chunk / S, sc = chunk - sr * S;
            const int e = NATIVE ? chunk * 256 + t : (sr * 16 + r) * T::BM + sc * 16 + c;
            const int u = bi * T::BM + sr * 16 + r, v = bj * T::BM + sc * 16 + c;
            live[q] = chunk < CPT && u < pr.d && v <= u;
            sum[q] = 0.f;
            old[q] = 0.f;
            if (live[q]) {
                old[q] = pr.F[(long)u * dF + v];
                if (pr.splits == 1) {
                    sum[q] = src[e];
                } else {
                    // sixteen interleaved running sums (fixed order, so still deterministic) keep loads in flight
                    float a[16];
#pragma unroll
                    for (int j = 0; j < 16; ++j) a[j] = 0.f;
                    int k = 0;
                    for (; k + 16 <= pr.splits; k += 16) {
#pragma unroll
                        for (int j = 0; j < 16; ++j) a[j] += src[(k + j) * sstride + e];
                    }
                    for (; k + 4 <= pr.splits; k += 4) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) a[j] += src[(k + j) * sstride + e];
                    }
                    for (; k < pr.splits; ++k) a[0] += src[k * sstride + e];
#pragma unroll
                    for (int h = 8; h > 0; h >>= 1)
#pragma unroll
                        for (int j = 0; j < h; ++j) a[j] += a[j + h];
                    sum[q] = a[0];
                }
            }
        }
#pragma unroll
        for (int q = 0; q < kRedGroup; ++q) {
            const int chunk = grp * kRedGroup + q;
            const int sr = chunk / S, sc = chunk - sr * S;
            const int u = bi * T::BM + sr * 16 + r, v = bj * T::BM + sc * 16 + c;
            float out = 0.f;
            if (live[q]) {
                out = pr.decay * old[q] + wnew * sum[q];
                pr.F[(long)u * dF + v] = out;
            }
            mir[q][r][c] = out;
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < kRedGroup; ++q) {
            const int chunk = grp * kRedGroup + q;
            const int sr = chunk / S, sc = chunk - sr * S;
            const int c2 = t >> 4, r2 = t & 15;
            const int u2 = bi * T::BM + sr * 16 + r2, v2 = bj * T::BM + sc * 16 + c2;
            if (chunk < CPT && u2 < pr.d && v2 < u2) pr.F[(long)v2 * dF + u2] = mir[q][r2][c2];
        }
    } else {
        // bias row: LP adjacent lanes share an element and take every LP-th split, four loads in flight each;
        // their sums meet by shuffles (fixed order: deterministic).  A single serial chain over a hundred
        // splits cost more than the tiles of the factor.
        const int bi = local - nblk * GPT;
        const float *csum = pr.partial + (long)pr.splits * nblk * TILE;
        constexpr int LP = T::BM <= 32 ? 8 : T::BM <= 64 ? 4 : T::BM <= 128 ? 2 : 1;
        const int r = threadIdx.x / LP, j = threadIdx.x % LP;
        const int u = bi * T::BM + r;
        const bool live = r < T::BM && u < pr.d;
        float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
        if (live) {
            const long step = (long)pr.nb * T::BM;
            const float *col = csum + (long)bi * T::BM + r;
            int k = j;
            for (; k + 3 * LP < pr.splits; k += 4 * LP) {
                a0 += col[k * step];
                a1 += col[(k + LP) * step];
                a2 += col[(k + 2 * LP) * step];
                a3 += col[(k + 3 * LP) * step];
            }
            for (; k < pr.splits; k += LP) a0 += col[k * step];
        }
        float s = (a0 + a1) + (a2 + a3);
#pragma unroll
        for (int h = 1; h < LP; h <<= 1) s += __shfl_xor(s, h);
        if (live && j == 0) {
            const float out = pr.decay * pr.F[(long)pr.d * dF + u] + wnew * s;
            pr.F[(long)pr.d * dF + u] = out;
            pr.F[(long)u * dF + pr.d] = out;
        }
        if (bi == 0 && threadIdx.x == 0) {
            const long dd = (long)pr.d * dF + pr.d;
            pr.F[dd] = pr.decay * pr.F[dd] + wnew * (float)pr.K;
        }
    }
}

// One reduce launch for the factors of a whole call, whatever kernel produced their partial tiles: the reduce
// of a group of layers is a few small workgroups, a launch of its own per group costs more than it runs.
constexpr int kMaxRedProblems = 128;   // a 14 KB kernel argument

struct RedTable {
    int count;
    int starts[kMaxRedProblems];       // first block of every problem, searched by bisection
    int kind[kMaxRedProblems];         // partial tile layout, see the switch below
    SyrkProb p[kMaxRedProblems];
};

__global__ __launch_bounds__(256) void syrk_reduce_kernel(const RedTable tab)
{
    __shared__ float mir[kRedGroup][16][17];
    int pi = 0, hi = tab.count - 1;
    while (pi < hi) {
        const int mid = (pi + hi + 1) >> 1;
        if ((int)blockIdx.x >= tab.starts[mid]) pi = mid;
        else hi = mid - 1;
    }
    const SyrkProb &pr = tab.p[pi];
    const int local = blockIdx.x - tab.starts[pi];
    switch (tab.kind[pi]) {
        case 0: syrk_reduce_body<Tile<4, 2>, false>(pr, local, mir); break;
        case 1: syrk_reduce_body<Tile<3, 3>, false>(pr, local, mir); break;
        case 2: syrk_reduce_body<Tile<2, 2>, false>(pr, local, mir); break;
        case 3: syrk_reduce_body<Tile<1, 2>, false>(pr, local, mir); break;
        case 4: syrk_reduce_body<Tile<3, 3>, true>(pr, local, mir); break;    // 144-wide tiles in accumulator order
        default: syrk_reduce_body<Tile<8, 2>, false>(pr, local, mir); break;
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
namespace {

struct Cfg { int wt, nw, bm; };
// the last entry is the wave-unit kernel (syrk_wave.hpp): 144-wide macro tiles, same partial layout as Tile<3,3>
const Cfg kCfgs[] = {{4, 2, 128}, {3, 3, 144}, {2, 2, 64}, {1, 2, 32}, {0, 0, 144}, {0, 0, 144}, {0, 0, 32}, {0, 0, 64},
                     {0, 0, 256}, {0, 0, 144}, {0, 0, 16}, {0, 0, 16}, {0, 0, 16}, {0, 0, 256}};
constexpr int kWaveCfg = 4;
constexpr int kCorr3Cfg = 10;  // 3x3 convolution factors from autocorrelations (syrk_corr3.hpp): 10 / 11 / 12 = 16 / 32 / 64 channels
constexpr int kConv3Cfg = 5;   // fused 3x3 convolution kernel (syrk_conv3.hpp), same partial layout
constexpr int kSmall32Cfg = 6; // narrow NCHW operands (syrk_small.hpp), partial tile 32 x 32 (d <= 32)
constexpr int kSmall64Cfg = 7; // same, 64 x 64 (d <= 64)
constexpr int kWaveNchwCfg = 9; // wave-unit kernel for NCHW fp32 operands (same partial layout as kWaveCfg)
constexpr int kBf16Cfg = 8;    // row-major bf16 operands on the bf16 MFMA units (syrk_bf16.hpp), 256 x 256 tiles
inline bool is_corr3_cfg(int cfg) { return cfg >= kCorr3Cfg && cfg < kCorr3Cfg + 3; }
constexpr int kSplitCfg = 13;  // wide fp32 operands on the bf16 MFMA units (syrk_split.hpp), same partial layout as kBf16Cfg

bool small_eligible(const FactorJob &j)
{
    return tuning().use_small_kernel && j.dtype == 0 && j.layout == kNCHW && j.d_core <= 64 && !j.has_bias &&
           j.hw % 4 == 0 && j.hw < (1l << 22);      // 32-bit element offsets inside an image
}

bool bf16_eligible(const FactorJob &j)
{
    // rows of whole 16-byte pieces; columns between d_core and the next multiple of 8 must exist and be
    // zero (true for patch matrices, whose pitch is d_core rounded up to 16 bytes with zero padding)
    if (!(tuning().use_bf16_mfma && j.dtype == 1 && j.d_core >= 96)) return false;
    if (j.layout == kRows)
        return j.ld % 8 == 0 && (j.d_core + 7) / 8 * 8 <= j.ld && j.ld < (1l << 22);
    // NCHW: channel rows must start on 4-byte boundaries and the tensor must fit 32-bit buffer offsets
    return j.layout == kNCHW && j.hw % 2 == 0 && (j.K / j.hw) * (long)j.ctot * j.hw * 2 < 0x7fffffffl;
}

// Wide fp32 factors on the bf16 MFMA units.  The 256 x 128 tiles of that kernel cover the lower triangle of a
// narrow factor badly (d = 576: 46 %), and the kernel runs about twice as fast per tile as the fp32 kernels it
// competes with: the wave-unit kernel for row-major operands, the slower block-tile kernel for NCHW ones.
bool split_syrk_eligible(const FactorJob &j)
{
    if (!(tuning().use_split_syrk && j.dtype == 0 && j.d_core >= tuning().split_syrk_min_d)) return false;
    const double fill = 0.5 * j.d_core * (double)j.d_core / ((double)syrk_split_tiles(j.d_core) * S_BM * S_BN);
    if (j.layout == kRows) {
        if (!(j.ld % 4 == 0 && j.ld < (1l << 22))) return false;
        return fill * 100 >= tuning().split_syrk_fill_rows;
    }
    if (j.layout != kNCHW || j.hw <= 0) return false;
    if ((j.K / j.hw) * (long)j.ctot * j.hw * 4 >= 0x7fffffffl) return false;
    // K stages of 16 positions that never cross an image: small odd maps pad K (7 x 7: by 30 %)
    const long slots = (j.hw + S_KT - 1) / S_KT * S_KT;
    return fill * (double)j.hw / (double)slots * 100 >= tuning().split_syrk_fill_nchw;
}

bool wave_waste_ok(int d)
{
    // the wave kernels always multiply whole 45-tile units: use them only where that wastes little
    // (measured: with a quarter of padding, as 2^n channel counts have, they only tie with the block-tile kernel)
    const long T = (d + 15) / 16, m = (d + W_MT - 1) / W_MT;
    const long exact = T * (T + 1) / 2, padded = 45 * m + 81 * m * (m - 1) / 2;
    return padded * 100 <= exact * 115;
}

bool wave_nchw_eligible(const FactorJob &j)
{
    if (!(tuning().use_wave_kernel && j.dtype == 0 && j.layout == kNCHW && j.hw > 0)) return false;
    // K stages of 16 positions that never cross an image: small odd maps (7 x 7) would pad K by a quarter
    const long slots = (j.hw + W_KT - 1) / W_KT * W_KT;
    if (slots * 10 > (long)j.hw * 11) return false;
    return (j.K / j.hw) * (long)j.ctot * j.hw * 4 < 0x7fffffffl && wave_waste_ok(j.d_core);
}

bool wave_eligible(const FactorJob &j)
{
    // shape-only test (the C ABI requires 16-byte aligned inputs), so that the workspace plan made
    // without pointers matches the launch
    if (!(tuning().use_wave_kernel && j.dtype == 0 && j.layout == kRows && j.ld % 4 == 0 && j.ld < (1l << 22)))
        return false;
    return wave_waste_ok(j.d_core);
}

// padded MFMA work (in 16x16 tiles) of the lower triangle for a config
long tri_tiles(int d, const Cfg &c)
{
    const long nb = (d + c.bm - 1) / c.bm;
    const long nw = nb * c.nw;
    return nw * (nw - 1) / 2 * c.wt * c.wt + nw * (c.wt * (c.wt + 1) / 2);
}

int choose_cfg(int d)
{
    const long force = tuning().syrk_force_bm;
    int best = 0;
    double best_cost = 1e300;
    for (int i = 0; i < 4; ++i) {
        if (force && kCfgs[i].bm != force) continue;
        // small tiles re-read the panels more often and run at a fraction of the MFMA rate of the large
        // ones (measured on long-K problems: 32-wide tiles are about 3x slower per padded tile)
        const double penalty = kCfgs[i].bm >= 128 ? 1.0 : (kCfgs[i].bm >= 64 ? 1.3 : 2.2);
        const double cost = (double)tri_tiles(d, kCfgs[i]) * penalty;
        if (cost < best_cost - 1e-9) { best_cost = cost; best = i; }
    }
    return best;
}

// Strip height of the autocorrelation kernel: the largest divisor of H whose two slabs fit 72 KB of LDS and
// whose slab is at most 12 float4 items per thread (0 = not eligible).  plane = floats per channel, padded
// so that consecutive channels start 4 banks apart.
int corr3_rows(int C, int H, int W, int *plane_out)
{
    int best = 0;
    for (int SR = 1; SR <= H; ++SR) {
        if (H % SR) continue;
        if ((SR * W) % 16) continue;                           // whole groups of 16 pixels
        int plane = (SR + 2) * (W + 8);
        plane += (4 - plane % 32 + 32) % 32;
        const long bytes = 2l * C * plane * 4;
        const long copies = ((long)C * plane / 4 + 63) / 64;       // 1 KB global -> LDS copies per slab, nine per staging wavefront at most
        if (bytes > std::min<long>(tuning().corr3_lds_kb, 80) * 1024 || copies > 36) continue;   // 80 KB: what the launch asks the runtime for
        best = SR;
        if (plane_out) *plane_out = plane;
    }
    return best;
}

bool corr3_eligible(const FactorJob &j)
{
    if (!(tuning().use_corr3 && j.layout == kConv3 && j.dtype == 0)) return false;
    if (!(j.ctot == 16 || j.ctot == 32 || j.ctot == 64)) return false;
    if (j.w % 4 != 0 || j.w > 64 || j.h > 64 || j.h < 2) return false;
    const long B = j.K / j.hw;
    if (B < 1 || B > 4 * 64) return false;                     // corners: a chunk of images is one LDS line
    if ((long)B * j.ctot * j.hw * 4 >= 0x7fffffffl) return false;
    return corr3_rows(j.ctot, j.h, j.w, nullptr) > 0;
}

struct Planned {
    int cfg;
    int nb, nblk, splits, tps;
    int bps;   // blocks per split
    int unit_rows = 16, rows_per_stage = 0;   // K rows per tile / conv stage; output rows per conv stage
    int stretch = 1;                          // relative speed of this problem's blocks per K row
    size_t partial_floats;
};

// jobs of one launch group share (cfg, layout, dtype)
void plan_group(const FactorJob *jobs, const std::vector<int> &idx, std::vector<Planned> &pl)
{
    const Tuning &tu = tuning();
    if (is_corr3_cfg(pl[idx[0]].cfg)) {
        // autocorrelation kernel: (image, strip) units dealt evenly to about target_blocks workgroups
        const long halves = pl[idx[0]].cfg == kCorr3Cfg + 2 ? 2 : 1;
        const long per = std::max<long>(1, tu.target_blocks / ((long)idx.size() * halves));
        for (int j : idx) {
            Planned &p = pl[j];
            const FactorJob &job = jobs[j];
            const int C = job.ctot;
            int plane = 0;
            p.rows_per_stage = corr3_rows(C, job.h, job.w, &plane);
            p.unit_rows = plane;                                   // carried to the launch
            const long units = (job.K / job.hw) * (job.h / p.rows_per_stage);
            p.tps = (int)std::max<long>(1, (units + per - 1) / per);       // units per block
            p.splits = (int)((units + p.tps - 1) / p.tps);
            p.nb = 1; p.nblk = 1; p.bps = 1;
            const size_t parts = (size_t)p.splits * (C == 16 ? 4 : 1);
            const size_t nF = (size_t)C3_LAGS * C * C, nB = (size_t)C3_BQ * C * C + (size_t)C3_BV * C;
            p.partial_floats = parts * (nF + C) + (nF + C) + (size_t)C3_CHUNKS * nB + nB + 64 +
                               nF + (size_t)C3_BQ * C * C +                        // transposed copies
                               (size_t)(job.K / job.hw) * 2 * C * job.h;          // + border columns
        }
        return;
    }
    double work = 0;
    for (int j : idx) {
        Planned &p = pl[j];
        const Cfg &c = kCfgs[p.cfg];
        p.nb = (jobs[j].d_core + c.bm - 1) / c.bm;
        p.nblk = p.nb * (p.nb + 1) / 2;
        p.bps = (p.cfg == kWaveCfg || p.cfg == kConv3Cfg || p.cfg == kWaveNchwCfg) ? wave_blocks_per_split(p.nb)
                : p.cfg == kSplitCfg ? syrk_split_tiles(jobs[j].d_core) : p.nblk;
        if (p.cfg == kConv3Cfg) {
            // K is walked in conv stages of R output rows; count them in units of 16 patch rows
            p.rows_per_stage = conv3_choose_rows(jobs[j].h, jobs[j].w);
            p.unit_rows = p.rows_per_stage * jobs[j].w;
        } else {
            p.unit_rows = (p.cfg == kBf16Cfg) ? H_KT : (p.cfg == kSmall32Cfg || p.cfg == kSmall64Cfg) ? S_GROUP : 16;
        }
        // A block that holds a single unit (one macro tile in all) spreads it over its four waves and
        // needs a quarter of the time per K row: give it four times the rows.
        p.stretch = ((p.cfg == kWaveCfg || p.cfg == kConv3Cfg || p.cfg == kWaveNchwCfg) && p.nb == 1) ? 4 : 1;
        const long ktiles = (jobs[j].K + 15) / 16;
        work += (double)p.bps * (double)ktiles / p.stretch;
    }
    // The narrow-NCHW kernel is bound by loads in flight, not by MFMAs: several of its light workgroups
    // share a CU, so it gets four times the blocks.
    const int cfg0 = pl[idx[0]].cfg;
    const long target = (cfg0 == kSmall32Cfg || cfg0 == kSmall64Cfg) ? tu.small_blocks_x * tu.target_blocks : tu.target_blocks;
    long tpb = (long)std::ceil(work / (double)target);
    tpb = std::max<long>(tpb, tu.min_tiles_per_split);
    // Blocks of a launch carry equal work and run about one per CU, so a launch a few blocks over the
    // target costs a whole extra round: grow the slice until the total fits.
    for (int iter = 0; iter < 64; ++iter) {
        long total = 0;
        for (int j : idx) {
            Planned &p = pl[j];
            const Cfg &c = kCfgs[p.cfg];
            long ktiles = std::max<long>(1, (jobs[j].K + p.unit_rows - 1) / p.unit_rows);
            if (p.cfg == kSmall32Cfg || p.cfg == kSmall64Cfg)   // walked in groups of positions that never cross an image
                ktiles = (jobs[j].K / jobs[j].hw) * ((jobs[j].hw + S_GROUP - 1) / S_GROUP);
            if ((p.cfg == kWaveNchwCfg || p.cfg == kSplitCfg) && jobs[j].layout == kNCHW)   // 16-position stages that never cross an image
                ktiles = (jobs[j].K / jobs[j].hw) * ((jobs[j].hw + W_KT - 1) / W_KT);
            if (p.cfg == kBf16Cfg && jobs[j].layout == kNCHW)   // 32-position stages that never cross an image
                ktiles = (jobs[j].K / jobs[j].hw) * ((jobs[j].hw + H_KT - 1) / H_KT);
            long tpb_j = std::max<long>(1, tpb * p.stretch * 16 / p.unit_rows);
            if (p.cfg == kWaveCfg || (p.cfg == kSplitCfg && jobs[j].layout == kRows))   // a split's byte range must stay below 2^31 (32-bit buffer offsets)
                tpb_j = std::max<long>(1, std::min<long>(tpb_j, 0x7fffffffl / (64 * jobs[j].ld) - 1));
            if (p.cfg == kBf16Cfg && jobs[j].layout == kRows)
                tpb_j = std::max<long>(1, std::min<long>(tpb_j, 0x7fffffffl / (2 * H_KT * jobs[j].ld) - 1));
            // The bf16 MFMA adds its sixteen products to the accumulator with the low bits of the aligned addends cut
            // off: on non-negative inputs (post-ReLU activations) every stage biases the sum down by about a
            // quarter of an ulp, measured -1.6e-8 per stage relative to the result (-3e-6 over 200 stages, where
            // the fp32 MFMA kernels stay at 2.5e-7).  Slices are therefore kept short; the reduction adds them in
            // fp32 with round-to-nearest.
            if (p.cfg == kSplitCfg) tpb_j = std::max<long>(1, std::min<long>(tpb_j, tu.split_syrk_max_stages));
            p.splits = (int)((ktiles + tpb_j - 1) / tpb_j);
            // every element of the block-tile kernels' partials is summed serially over the splits by one
            // thread of the reduction: keep that chain short
            if (p.cfg < kWaveCfg) p.splits = std::min<int>(p.splits, (int)tu.tile_max_splits);
            p.tps = (int)((ktiles + p.splits - 1) / p.splits);
            p.splits = (int)((ktiles + p.tps - 1) / p.tps);
            p.partial_floats = (size_t)p.splits * ((size_t)p.nblk * c.bm * c.bm + (size_t)p.nb * c.bm);
            total += (long)p.bps * p.splits;
        }
        if (total <= target || tpb > (1l << 40)) break;
        bool can_shrink = false;
        for (int j : idx) can_shrink |= pl[j].splits > 1;
        if (!can_shrink) break;
        tpb += std::max<long>(1, tpb / 32);
    }
}

int group_key(const FactorJob &j, int cfg) { return cfg * 8 + j.layout * 2 + j.dtype; }   // layout 0..2, dtype 0..1

void plan_all(const FactorJob *jobs, int n, std::vector<Planned> &pl, std::vector<std::vector<int>> &groups)
{
    pl.assign(n, Planned());
    std::vector<int> keys(n);
    for (int i = 0; i < n; ++i) {
        if (corr3_eligible(jobs[i])) pl[i].cfg = kCorr3Cfg + (jobs[i].ctot == 16 ? 0 : (jobs[i].ctot == 32 ? 1 : 2));
        else if (jobs[i].layout == kConv3) pl[i].cfg = kConv3Cfg;
        else if (small_eligible(jobs[i])) pl[i].cfg = jobs[i].d_core <= 32 ? kSmall32Cfg : kSmall64Cfg;
        else if (bf16_eligible(jobs[i])) pl[i].cfg = kBf16Cfg;
        else if (split_syrk_eligible(jobs[i])) pl[i].cfg = kSplitCfg;
        else if (wave_nchw_eligible(jobs[i])) pl[i].cfg = kWaveNchwCfg;
        else pl[i].cfg = wave_eligible(jobs[i]) ? kWaveCfg : choose_cfg(jobs[i].d_core);
        keys[i] = group_key(jobs[i], pl[i].cfg);
    }
    groups.clear();
    for (int key = 0; key < 8 * (kSplitCfg + 1); ++key) {
        std::vector<int> cur;
        for (int i = 0; i < n; ++i) {
            if (keys[i] != key) continue;
            cur.push_back(i);
            if ((int)cur.size() == kMaxProblems) { groups.push_back(cur); cur.clear(); }
        }
        if (!cur.empty()) groups.push_back(cur);
    }
    for (auto &g : groups) plan_group(jobs, g, pl);
}

bool vec_ok(const FactorJob &j)
{
    const size_t eb = j.dtype == 0 ? 4 : 2;
    if (((uintptr_t)j.x) % (4 * eb) != 0) return false;
    if (j.layout == kRows) return j.ld % 4 == 0;
    return j.hw % 4 == 0;
}

template <class T, int LAYOUT, int DT>
hipError_t launch_cfg(const SyrkTable &tab, int blocks, double flops, hipStream_t s)
{
    KFAC_LAUNCH(KFAC_K_SYRK, s, (syrk_partial_kernel<T, LAYOUT, DT>), dim3(blocks), dim3(T::NT), 0, tab);
    timing_work(flops);
    return hipGetLastError();
}

template <class T>
hipError_t launch_ld(const SyrkTable &tab, int layout, int dt, int blocks, double flops, hipStream_t s)
{
    if (layout == kRows) {
        if (dt == 0) return launch_cfg<T, kRows, 0>(tab, blocks, flops, s);
        return launch_cfg<T, kRows, 1>(tab, blocks, flops, s);
    }
    if (dt == 0) return launch_cfg<T, kNCHW, 0>(tab, blocks, flops, s);
    return launch_cfg<T, kNCHW, 1>(tab, blocks, flops, s);
}

// reduce work of the groups launched so far, flushed as one launch
struct PendingReduce {
    RedTable tab;
    int blocks = 0;
    double bytes = 0.0;
};

hipError_t red_flush(PendingReduce &pend, hipStream_t s)
{
    if (pend.tab.count == 0) return hipSuccess;
    KFAC_LAUNCH(KFAC_K_SYRK_REDUCE, s, syrk_reduce_kernel, dim3(pend.blocks), dim3(256), 0, pend.tab);
    timing_work(pend.bytes);
    pend.tab.count = 0;
    pend.blocks = 0;
    pend.bytes = 0.0;
    return hipGetLastError();
}

int red_kind(int cfg)
{
    switch (cfg) {
        case 0: return 0;
        case 1: return 1;
        case 2: return 2;
        case 3: return 3;
        case kSmall32Cfg: return 3;
        case kSmall64Cfg: return 2;
        case kBf16Cfg: return 5;
        case kSplitCfg: return 5;
        default: return 4;             // wave-unit and fused convolution kernels
    }
}

}  // namespace

namespace {

template <int NT>
hipError_t corr3_launch_nt(CorrTable &tab, const std::vector<size_t> &lds, double flops, double exflops, hipStream_t s)
{
    // main kernel
    int blocks = 0;
    size_t lds_bytes = 0;
    for (int k = 0; k < tab.count; ++k) {
        tab.p[k].blk_start = blocks;
        tab.starts[k] = blocks;
        blocks += tab.p[k].splits * (NT == 4 ? 2 : 1);   // 64 channels: two workgroups per range of units
        lds_bytes = std::max(lds_bytes, lds[k]);
    }
    {   // per device and cheap: set on every launch rather than remembered in a process-wide flag
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&corr3_main_kernel<NT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024);
        if (e != hipSuccess) return e;
    }
    KFAC_LAUNCH(KFAC_K_SYRK_CORR3, s, (corr3_main_kernel<NT>), dim3(blocks), dim3(512), lds_bytes, tab);
    timing_work(flops, exflops);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // border terms: small maps of at least 32 channels from whole images (the problems of a launch share a
    // shape class, not a shape: both kernels may run, each on its own table)
    CorrTable line_tab, plane_tab;
    line_tab.count = plane_tab.count = 0;
    int line_blocks = 0, plane_blocks = 0;
    for (int k = 0; k < tab.count; ++k) {
        const bool plane = NT >= 2 && tab.p[k].H * tab.p[k].W <= 64;
        CorrTable &t = plane ? plane_tab : line_tab;
        int &nb = plane ? plane_blocks : line_blocks;
        t.p[t.count] = tab.p[k];
        t.p[t.count].blk_start = nb;
        t.starts[t.count] = nb;
        ++t.count;
        nb += plane ? C3_CHUNKS * (NT * NT / 4) : 5 * C3_CHUNKS;      // line kernel: 5 sides x image chunks
    }
    if (line_tab.count > 0) {
        KFAC_LAUNCH(KFAC_K_CORR3_ASM, s, (corr3_border_kernel<NT>), dim3(line_blocks), dim3(256), 0, line_tab);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (NT >= 2 && plane_tab.count > 0) {
        KFAC_LAUNCH(KFAC_K_CORR3_ASM, s, (corr3_border_plane_kernel<(NT >= 2 ? NT : 2)>), dim3(plane_blocks), dim3(256), 0,
                    plane_tab);
        e = hipGetLastError();
    }
    return e;
}

hipError_t corr3_launch(const FactorJob *jobs, const std::vector<int> &g, const std::vector<Planned> &pl,
                        const std::vector<size_t> &offs, void *work, double flops, double exflops, hipStream_t s)
{
    CorrTable tab;
    tab.count = (int)g.size();
    std::vector<size_t> lds(g.size());
    for (int k = 0; k < tab.count; ++k) {
        const int j = g[k];
        const FactorJob &job = jobs[j];
        const Planned &P = pl[j];
        CorrProb &p = tab.p[k];
        const int C = job.ctot;
        const size_t nF = (size_t)C3_LAGS * C * C, nB = (size_t)C3_BQ * C * C + (size_t)C3_BV * C;
        p.x = static_cast<const float *>(job.x);
        p.C = C; p.H = job.h; p.W = job.w; p.B = (int)(job.K / job.hw);
        p.SR = P.rows_per_stage; p.strips = job.h / P.rows_per_stage;
        p.units = p.B * p.strips;
        p.splits = P.splits; p.upb = P.tps;
        p.parts = P.splits * (C == 16 ? 4 : 1);
        p.plane = P.unit_rows;
        p.has_bias = job.has_bias; p.scale = job.scale; p.decay = job.decay;
        p.F = job.F;
        float *base = reinterpret_cast<float *>(static_cast<char *>(work) + offs[j]);
        p.Fp = base;
        p.Fs = p.Fp + (size_t)p.parts * (nF + C);
        p.Bp = p.Fs + (nF + C);
        p.Bs = p.Bp + (size_t)C3_CHUNKS * nB;
        p.FsT = p.Bs + nB;
        p.BsT = p.FsT + nF;
        p.cols = p.BsT + (size_t)C3_BQ * C * C;
        p.blk_start = 0;
        lds[k] = (size_t)2 * C * p.plane * sizeof(float);
    }
    const int cfg = pl[g[0]].cfg;
    hipError_t e = cfg == kCorr3Cfg ? corr3_launch_nt<1>(tab, lds, flops, exflops, s)
                 : cfg == kCorr3Cfg + 1 ? corr3_launch_nt<2>(tab, lds, flops, exflops, s)
                                        : corr3_launch_nt<4>(tab, lds, flops, exflops, s);
    if (e != hipSuccess) return e;
    // sums over parts and chunks
    int blocks = 0;
    for (int k = 0; k < tab.count; ++k) {
        const CorrProb &p = tab.p[k];
        tab.p[k].blk_start = blocks;
        tab.starts[k] = blocks;
        const long total = (long)(C3_LAGS + C3_BQ) * p.C * p.C / 4 + (long)(1 + C3_BV) * p.C;   // four matrix elements per thread
        blocks += (int)((total + 255) / 256);
    }
    KFAC_LAUNCH(KFAC_K_CORR3_ASM, s, corr3_sum_kernel, dim3(blocks), dim3(256), 0, tab);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    // assembly, scale, running average
    blocks = 0;
    for (int k = 0; k < tab.count; ++k) {
        const CorrProb &p = tab.p[k];
        tab.p[k].blk_start = blocks;
        tab.starts[k] = blocks;
        blocks += (3 * p.C + p.has_bias + C3_ARW - 1) / C3_ARW;       // one wavefront per channel and kernel row (+ the bias row)
    }
    KFAC_LAUNCH(KFAC_K_CORR3_ASM, s, corr3_assemble_kernel, dim3(blocks), dim3(256), 0, tab);
    return hipGetLastError();
}

}  // namespace

int conv3_rows(int h, int w) { return conv3_choose_rows(h, w); }

size_t syrk_workspace_bytes(const FactorJob *jobs, int n)
{
    std::vector<Planned> pl;
    std::vector<std::vector<int>> groups;
    plan_all(jobs, n, pl, groups);
    size_t total = 0;
    for (int i = 0; i < n; ++i) total += align_up(pl[i].partial_floats * sizeof(float), 256);
    return total;
}

hipError_t syrk_launch(const FactorJob *jobs, int n, void *work, size_t work_bytes, hipStream_t s)
{
    std::vector<Planned> pl;
    std::vector<std::vector<int>> groups;
    plan_all(jobs, n, pl, groups);
    size_t off = 0;
    std::vector<size_t> offs(n);
    for (int i = 0; i < n; ++i) {
        offs[i] = off;
        off += align_up(pl[i].partial_floats * sizeof(float), 256);
    }
    if (off > work_bytes) return hipErrorInvalidValue;

    PendingReduce pend;
    pend.tab.count = 0;
    for (auto &g : groups) {
        SyrkTable tab;
        tab.count = (int)g.size();
        tab.debug = (int)tuning().wave_debug;
        int blocks = 0;
        double flops = 0.0, corr_flops = 0.0;   // corr_flops: 13 lag tiles per channel-tile pair and pixel, 26 C^2 per pixel
        std::vector<int> red_n(g.size());
        std::vector<double> red_b(g.size());
        for (int k = 0; k < tab.count; ++k) {
            const int j = g[k];
            const FactorJob &job = jobs[j];
            flops += (double)job.K * (job.d_core + job.has_bias) * (job.d_core + job.has_bias + 1);
            corr_flops += 26.0 * job.ctot * job.ctot * (double)job.K;
            {   // reduce + running average: the split slices and the old factor read (one triangle), the factor written (both)
                const double dF = job.d_core + job.has_bias, tri = dF * (dF + 1) / 2;
                red_b[k] = 4.0 * ((pl[j].splits + 1) * tri + dF * dF);
            }
            SyrkProb &p = tab.p[k];
            p.x = job.x;
            p.partial = reinterpret_cast<float *>(static_cast<char *>(work) + offs[j]);
            p.F = job.F;
            p.K = job.K;
            p.ld = (pl[j].cfg == kConv3Cfg) ? conv3_pack(job.h, job.w, pl[j].rows_per_stage) : job.ld;
            p.d = job.d_core;
            p.hw = job.hw > 0 ? job.hw : 1;
            p.ctot = job.ctot;
            p.nb = pl[j].nb;
            p.splits = pl[j].splits;
            p.tiles_per_split = pl[j].tps;
            p.blk_start = blocks;
            tab.starts[k] = blocks;
            p.red_start = 0;
            p.vec = vec_ok(job) ? 1 : 0;
            p.has_bias = job.has_bias;
            p.scale = job.scale;
            p.decay = job.decay;
            blocks += pl[j].bps * pl[j].splits;
            {
                const int bm = kCfgs[pl[j].cfg].bm;
                const int cpt = (bm * bm + kRedChunk - 1) / kRedChunk;
                const int gpt = (cpt + kRedGroup - 1) / kRedGroup;
                red_n[k] = pl[j].nblk * gpt + (job.has_bias ? pl[j].nb : 0);
            }
        }
        const int cfg = pl[g[0]].cfg;
        const int layout = jobs[g[0]].layout, dt = jobs[g[0]].dtype;
        hipError_t e = hipSuccess;
        if (is_corr3_cfg(cfg)) {
            e = corr3_launch(jobs, g, pl, offs, work, flops, corr_flops, s);
            if (e != hipSuccess) return e;
            continue;
        }
        switch (cfg) {
            case kConv3Cfg: {
                size_t lds_bytes = 0;
                for (int k = 0; k < tab.count; ++k) {
                    const FactorJob &job = jobs[g[k]];
                    const Conv3Geo geo = conv3_geo(job.h, job.w, pl[g[k]].rows_per_stage);
                    lds_bytes = std::max(lds_bytes, (size_t)(C3_PRE + C3_NSTAGE * W_SLOTS * geo.slab + 256) * 4);
                }
                // per device and cheap: set on every launch rather than remembered in a process-wide flag
                e = hipFuncSetAttribute(reinterpret_cast<const void *>(&syrk_conv3_kernel<4>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
                if (e != hipSuccess) break;
                KFAC_LAUNCH(KFAC_K_SYRK_CONV3, s, (syrk_conv3_kernel<4>), dim3(blocks), dim3(256), lds_bytes, tab);
                timing_work(flops);
                e = hipGetLastError();
                break;
            }
            case kSmall32Cfg:
            case kSmall64Cfg: {
                int ntl = 1;
                for (int k = 0; k < tab.count; ++k) ntl = std::max(ntl, (jobs[g[k]].d_core + 15) / 16);
                if (ntl == 1) KFAC_LAUNCH(KFAC_K_SYRK_SMALL, s, (syrk_small_nchw_kernel<1>), dim3(blocks), dim3(256), 0, tab);
                else if (ntl == 2) KFAC_LAUNCH(KFAC_K_SYRK_SMALL, s, (syrk_small_nchw_kernel<2>), dim3(blocks), dim3(256), 0, tab);
                else if (ntl == 3) KFAC_LAUNCH(KFAC_K_SYRK_SMALL, s, (syrk_small_nchw_kernel<3>), dim3(blocks), dim3(256), 0, tab);
                else KFAC_LAUNCH(KFAC_K_SYRK_SMALL, s, (syrk_small_nchw_kernel<4>), dim3(blocks), dim3(256), 0, tab);
                timing_work(flops);
                e = hipGetLastError();
                break;
            }
            case kBf16Cfg: {
                if (layout == kRows)
                    KFAC_LAUNCH(KFAC_K_SYRK_BF16, s, syrk_bf16_kernel<kRows>, dim3(blocks), dim3(512), 0, tab);
                else
                    KFAC_LAUNCH(KFAC_K_SYRK_BF16, s, syrk_bf16_kernel<kNCHW>, dim3(blocks), dim3(512), 0, tab);
                timing_work(flops);
                e = hipGetLastError();
                break;
            }
            case kSplitCfg: {
                if (layout == kRows)
                    KFAC_LAUNCH(KFAC_K_SYRK_SPLIT, s, syrk_split_kernel<kRows>, dim3(blocks), dim3(256), 0, tab);
                else
                    KFAC_LAUNCH(KFAC_K_SYRK_SPLIT, s, syrk_split_kernel<kNCHW>, dim3(blocks), dim3(256), 0, tab);
                timing_work(flops, 6.0 * flops);
                e = hipGetLastError();
                break;
            }
            case kWaveNchwCfg: {
                KFAC_LAUNCH(KFAC_K_SYRK_WAVE, s, syrk_wave_nchw_kernel, dim3(blocks), dim3(256), 0, tab);
                timing_work(flops);
                e = hipGetLastError();
                break;
            }
            case kWaveCfg: {
                KFAC_LAUNCH(KFAC_K_SYRK_WAVE, s, syrk_wave_kernel, dim3(blocks), dim3(256), 0, tab);
                timing_work(flops);
                e = hipGetLastError();
                break;
            }
            case 0: e = launch_ld<Tile<4, 2>>(tab, layout, dt, blocks, flops, s); break;
            case 1: e = launch_ld<Tile<3, 3>>(tab, layout, dt, blocks, flops, s); break;
            case 2: e = launch_ld<Tile<2, 2>>(tab, layout, dt, blocks, flops, s); break;
            default: e = launch_ld<Tile<1, 2>>(tab, layout, dt, blocks, flops, s); break;
        }
        if (e != hipSuccess) return e;
        // the reduce of this group joins the launch at the end of the call
        const int kind = red_kind(cfg);
        for (int k = 0; k < tab.count; ++k) {
            if (pend.tab.count == kMaxRedProblems) {
                e = red_flush(pend, s);
                if (e != hipSuccess) return e;
            }
            const int i = pend.tab.count++;
            pend.tab.p[i] = tab.p[k];
            pend.tab.starts[i] = pend.blocks;
            pend.tab.kind[i] = kind;
            pend.blocks += red_n[k];
            pend.bytes += red_b[k];
        }
    }
    return red_flush(pend, s);
}

}  // namespace kfac

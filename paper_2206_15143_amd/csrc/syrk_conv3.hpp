// A factor of a 3x3 / stride 1 / pad 1 convolution straight from the NCHW
// input: the patch matrix (footnote of section 3 of the DP-KFAC paper: a
// convolution as a linear map over im2col patches) is never written to memory.
//
// Same wave-unit scheme as syrk_wave.hpp (a macro tile of 144 patch columns is
// exactly 16 input channels x 9 taps), but what is staged in LDS is the raw
// input: for a stage of R output rows of one image, the R + 2 input rows of
// the 16 channels of each panel, each row padded to W + 4 floats.  The MFMA
// operand for patch row (oh, ow) and column (c, i, j) is then just
//     slab[(c*(R+2) + (oh - oh0) + i) * (W+4) + ow + j - 1]
// i.e. a per-lane constant (from the column) plus a per-k-step scalar (from
// the position).  The four pad floats of every row are written as zeros by the
// same load instruction that brings the row in (their lanes point out of
// range), and rows above / below the image are whole out-of-range rows, so the
// zero padding of the convolution costs no instruction in the MFMA loop.
// Traffic drops from (write + read of 9x the input) to one read of the input
// (plus the halo rows), which turns the 16-channel layers from HBM-bound into
// MFMA-bound.
#pragma once

#include "syrk_wave.hpp"

namespace kfac {

constexpr int C3_NSTAGE = 3;   // ring of stage buffers (two stages of loads in flight)
constexpr int C3_PRE = 4;      // zero floats in front of the first slab (left halo of its first row)

struct Conv3Geo {
    int H, W, R;      // image size, output rows per stage
    int Wp, SR;       // padded row pitch (floats), slab rows per channel
    int LPR, RPI;     // lanes per row (16 bytes each, incl. the pad lane), rows per load instruction
    int rows;         // LDS rows per panel slab (16 channels)
    int NI;           // load instructions per slab
    int slab;         // floats per slab
    int nks;          // k-steps (4 patch rows each) per stage
    int spi;          // stages per image
};

__host__ __device__ inline Conv3Geo conv3_geo(int H, int W, int R)
{
    Conv3Geo g;
    g.H = H; g.W = W; g.R = R;
    g.Wp = W + 4;
    g.SR = R + 2;
    g.LPR = g.Wp / 4;
    g.RPI = 64 / g.LPR;
    g.rows = 16 * g.SR;
    g.NI = (g.rows + g.RPI - 1) / g.RPI;
    g.slab = g.rows * g.Wp;
    g.nks = R * W / 4;
    g.spi = H / R;
    return g;
}

__host__ __device__ inline long conv3_pack(int H, int W, int R) { return ((long)H << 40) | ((long)W << 20) | (long)R; }

// Output rows per stage: the largest divisor of H whose ring of slabs fits LDS (0 = shape not supported).
// A stage must hold at least 8 k-steps: with fewer (maps of 4 x 4 and below) the barrier and the slab loads of
// every stage outweigh its products, and the explicit patch matrix is the faster route (measured on
// 512-channel 4 x 4 layers).
inline int conv3_choose_rows(int H, int W)
{
    if (W % 4 != 0 || W < 4 || W > 252) return 0;
    int best = 0;
    for (int R = 1; R <= H; ++R) {
        if (H % R != 0 || (R * W) % 16 != 0) continue;
        const Conv3Geo g = conv3_geo(H, W, R);
        const long bytes = ((long)C3_NSTAGE * W_SLOTS * g.slab + C3_PRE + 256) * 4;
        if (bytes > 150 * 1024 || (g.NI + 3) / 4 > 4 || g.nks < 8) continue;
        // the bias border is summed by one thread per slab row and at most four 16-byte pieces per thread
        if (g.rows > 256 || g.rows * (W / 4) > 4 * 256) continue;
        best = R;
    }
    return best;
}

struct Conv3Ctx {
    int4v rsrc;
    Conv3Geo g;
    unsigned lds_base;        // LDS byte address of the first slab (after the leading zero floats)
    int nslots, nst, nstages; // nst = conv stages in this split; nstages = ring steps (3 conv stages each in single blocks)
    long sg0;                 // first conv stage of the split
    int C;
    int w, lane, tid;
    int rslot, cslot, ctile0;
    bool single, owns_colsum;
    bool no_mfma, no_load, no_issue;   // measurement switches
};

template <int NIW>
struct Conv3Lanes {
    unsigned vo[W_SLOTS][NIW];   // byte offset of this lane's 16 bytes (relative to one row before the tensor)
    unsigned flag[NIW];          // bit0 lane takes part, bit1 data lane (not the pad lane), bit2 first slab row of a
                                 // channel (input row oh0-1), bit3 last slab row (input row oh0+R)
};

// Loads of ring step g: 3 * NIW instructions per wave, always.
template <int NIW>
__device__ __forceinline__ void conv3_issue(const Conv3Ctx &c, const Conv3Lanes<NIW> &ln, int g)
{
    const Conv3Geo &G = c.g;
    if (c.no_issue) return;
    const unsigned stage_bytes = (unsigned)(W_SLOTS * G.slab * 4);
    const unsigned buf = c.lds_base + (unsigned)(g % C3_NSTAGE) * stage_bytes;
    const unsigned dummy = c.lds_base + (unsigned)C3_NSTAGE * stage_bytes;
#pragma unroll
    for (int s = 0; s < W_SLOTS; ++s) {
        const int st = c.single ? 3 * g + s : g;       // conv stage (relative to the split) this slot holds
        const bool live = (s < c.nslots) && (g < c.nstages) && (st < c.nst) && !c.no_load;
        const unsigned sg = (unsigned)(c.sg0 + st);
        const unsigned n = sg / (unsigned)G.spi;
        const int oh0 = (int)(sg - n * (unsigned)G.spi) * G.R;
        const unsigned so = live ? (unsigned)(((int)n * c.C * G.H + oh0) * G.W * 4) : 0u;
        const bool top = oh0 == 0, bottom = oh0 + G.R == G.H;
#pragma unroll
        for (int qi = 0; qi < NIW; ++qi) {
            const int q = c.w + 4 * qi;
            if (live && q < G.NI) {
                const unsigned f = ln.flag[qi];
                if (f & 1u) {   // lanes past the slab rows of this instruction stay out of it
                    const bool ok = (f & 2u) && !((f & 4u) && top) && !((f & 8u) && bottom);
                    dma16(buf + (unsigned)((s * G.slab + q * G.RPI * G.Wp) * 4), ok ? ln.vo[s][qi] : W_OOB, c.rsrc, so);
                }
            } else {
                dma16(dummy, W_OOB, c.rsrc, 0u);
            }
        }
    }
}

template <int NIW>
__device__ __forceinline__ void conv3_sync()
{
    // at most one ring step of this wave's loads (3 * NIW instructions) stays outstanding
    if (NIW == 1) asm volatile("s_waitcnt vmcnt(3)\n\ts_barrier" ::: "memory");
    else if (NIW == 2) asm volatile("s_waitcnt vmcnt(6)\n\ts_barrier" ::: "memory");
    else if (NIW == 3) asm volatile("s_waitcnt vmcnt(9)\n\ts_barrier" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(12)\n\ts_barrier" ::: "memory");
}

// Operands of one k-step, gathered from the slab: cb / cc = per-lane slab offsets of the 16 patch
// columns of each row / column tile, pos = offset of the k-step's first position.
struct Conv3Ops {
    float a[W_NT];
    float b[5];
};

template <int KIND>
__device__ __forceinline__ void conv3_load(Conv3Ops &o, const float *slabR, const float *slabC, const int (&cb)[W_NT],
                                           const int (&cc)[5], int pos)
{
#pragma unroll
    for (int t = 0; t < W_NT; ++t) o.a[t] = slabR[cb[t] + pos];
    if (KIND == kHalf5 || KIND == kHalf4) {
#pragma unroll
        for (int t = 0; t < (KIND == kHalf5 ? 5 : 4); ++t) o.b[t] = slabC[cc[t] + pos];
    }
}

template <int KIND>
__device__ __forceinline__ void conv3_mma(const Conv3Ops &o, floatx4 (&acc)[45])
{
    if (KIND == kSingle || KIND == kDiag) {
#pragma unroll
        for (int ti = 0; ti < W_NT; ++ti)
#pragma unroll
            for (int tj = 0; tj <= ti; ++tj)
                acc[ti * (ti + 1) / 2 + tj] =
                    __builtin_amdgcn_mfma_f32_16x16x4f32(o.a[ti], o.a[tj], acc[ti * (ti + 1) / 2 + tj], 0, 0, 0);
    } else {
#pragma unroll
        for (int ti = 0; ti < W_NT; ++ti)
#pragma unroll
            for (int tj = 0; tj < (KIND == kHalf5 ? 5 : 4); ++tj)
                acc[ti * 5 + tj] = __builtin_amdgcn_mfma_f32_16x16x4f32(o.a[ti], o.b[tj], acc[ti * 5 + tj], 0, 0, 0);
    }
}

// slab offset of patch column `col` (0..143 of a macro tile) for the first position of a stage
__device__ __forceinline__ int conv3_col_offset(const Conv3Geo &G, int col)
{
    const int cl = col / 9, tap = col - cl * 9;
    const int i = tap / 3, j = tap - i * 3;
    return (cl * G.SR + i) * G.Wp + j - 1;
}

// Bias border.  Instead of summing every patch column, the workgroup sums the slab rows (channel, input
// row): a patch column (c, i, j) sees a row shifted by j - 1, so its sum over ow is the full row sum
// (j = 1), minus the last element (j = 0) or minus the first (j = 2).  The 16-byte pieces of a slab
// are dealt to all 256 threads (piece p of thread t is item t + 256 p, always the same across stages,
// so the sums stay in registers); threads below the row count also keep the first and last element
// of "their" row.  Index 0 / 1: macro tiles of panel slots 0 / 1.
constexpr int C3_NIT = 4;   // pieces per thread and slab (a slab has at most 1024 pieces)
struct Conv3ColAcc {
    float it[2][C3_NIT];
    float first[2], last[2];
};

template <int KIND, int NIW>
__device__ __forceinline__ void conv3_loop(const Conv3Ctx &c, const Conv3Lanes<NIW> &ln, const float *lds,
                                           floatx4 (&acc)[45], Conv3ColAcc &ca)
{
    const Conv3Geo &G = c.g;
    const int lr = c.lane & 15, lk = c.lane >> 4;
    int cb[W_NT], cc[5];
#pragma unroll
    for (int t = 0; t < W_NT; ++t) cb[t] = conv3_col_offset(G, t * 16 + lr) + lk;
#pragma unroll
    for (int t = 0; t < 5; ++t) {
        const int tile = c.ctile0 + t;
        cc[t] = (tile < W_NT) ? conv3_col_offset(G, tile * 16 + lr) + lk : 0;
    }

    // slab offsets of this thread's pieces for the row sums (-1: none), the same at every stage
    int ioff[C3_NIT];
    {
        const int w4 = G.W / 4, nitems = G.rows * w4;
#pragma unroll
        for (int q = 0; q < C3_NIT; ++q) {
            const int item = c.tid + 256 * q;
            const int row = item / w4, x4 = item - row * w4;
            ioff[q] = (c.owns_colsum && item < nitems) ? row * G.Wp + 4 * x4 : -1;
        }
    }
    const int eoff = (c.owns_colsum && c.tid < G.rows) ? c.tid * G.Wp : -1;

    conv3_issue<NIW>(c, ln, 0);
    conv3_issue<NIW>(c, ln, 1);
    conv3_sync<NIW>();
    for (int g = 0; g < c.nstages; ++g) {
        conv3_issue<NIW>(c, ln, g + 2);
        const float *buf = lds + (g % C3_NSTAGE) * (W_SLOTS * G.slab);
        if (c.no_mfma) {
            // measurement only
        } else {
            // k-steps of this wave: single blocks give wave w the steps w, w+4, ... of each of the three
            // staged conv stages; otherwise the wave walks all steps of its own panels.  The operands of
            // step i+1 are fetched from LDS (two register sets, A and B) while the MFMAs of step i run.
            const int inc = (KIND == kSingle) ? 16 : 4;
            const int steps = (KIND == kSingle) ? (G.nks - c.w + 3) / 4 : G.nks;
            const int nsl = (KIND == kSingle) ? W_SLOTS : 1;
#pragma unroll 1
            for (int s = 0; s < nsl; ++s) {
                if (KIND == kSingle && 3 * g + s >= c.nst) break;   // past the end of the split: stale rows
                const float *slabR = buf + ((KIND == kSingle) ? s : c.rslot) * G.slab;
                const float *slabC = buf + c.cslot * G.slab;
                // single blocks: the row-sum fetches of this slab go out ahead of the MFMA loop and are
                // added up after it (their LDS latency hides behind the MFMAs)
                floatx4 cv[C3_NIT];
                float cf = 0.f, cl = 0.f;
                if (KIND == kSingle && c.owns_colsum) {
#pragma unroll
                    for (int q = 0; q < C3_NIT; ++q) {
                        cv[q] = floatx4{0.f, 0.f, 0.f, 0.f};
                        if (ioff[q] >= 0) cv[q] = *reinterpret_cast<const floatx4 *>(slabR + ioff[q]);
                    }
                    if (eoff >= 0) {
                        cf = slabR[eoff];
                        cl = slabR[eoff + G.W - 1];
                    }
                }
                // position of the k-step inside the stage: column ow, row offset ro (floats); advanced
                // without branches so that fetches and MFMAs stay in one basic block
                const int inc_rows = (inc / G.W) * G.Wp, inc_cols = inc % G.W;
                int ow = ((KIND == kSingle) ? 4 * c.w : 0) % G.W;
                int ro = (((KIND == kSingle) ? 4 * c.w : 0) / G.W) * G.Wp;
                auto advance = [&]() {
                    ow += inc_cols;
                    ro += inc_rows;
                    const bool wrap = ow >= G.W;
                    ow -= wrap ? G.W : 0;
                    ro += wrap ? G.Wp : 0;
                };
                // Two register sets of operands used alternately (no copies): while the 45 MFMAs of one
                // step run, the 13-14 LDS fetches of the next step are already issued into the other
                // set.  The fetch after the last step reads a little past the stage's rows, still inside
                // the LDS allocation (next slab or the landing zone), and the values are dropped.
                // Scheduling fences keep "fetches, then MFMAs" as written.
                Conv3Ops p, q;
                conv3_load<KIND>(p, slabR, slabC, cb, cc, ro + ow);
                int i = 0;
#pragma unroll 1
                for (; i + 2 <= steps; i += 2) {
                    advance();
                    conv3_load<KIND>(q, slabR, slabC, cb, cc, ro + ow);
                    __builtin_amdgcn_sched_barrier(0);
                    conv3_mma<KIND>(p, acc);
                    __builtin_amdgcn_sched_barrier(0);
                    advance();
                    conv3_load<KIND>(p, slabR, slabC, cb, cc, ro + ow);
                    __builtin_amdgcn_sched_barrier(0);
                    conv3_mma<KIND>(q, acc);
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (i < steps) conv3_mma<KIND>(p, acc);   // odd number of steps
                if (KIND == kSingle && c.owns_colsum) {
#pragma unroll
                    for (int q = 0; q < C3_NIT; ++q) ca.it[0][q] += (cv[q].x + cv[q].y) + (cv[q].z + cv[q].w);
                    ca.first[0] += cf;
                    ca.last[0] += cl;
                }
            }
        }
        if (KIND != kSingle && c.owns_colsum) {
            const int nsl = (KIND == kSingle) ? 3 : 2;
            for (int s = 0; s < nsl; ++s) {
                if (KIND == kSingle && 3 * g + s >= c.nst) break;
                const int cls = (KIND == kSingle || s == 0) ? 0 : 1;
                const float *sl = buf + s * G.slab;
#pragma unroll
                for (int q = 0; q < C3_NIT; ++q) {
                    if (ioff[q] >= 0) {
                        const floatx4 v = *reinterpret_cast<const floatx4 *>(sl + ioff[q]);
                        ca.it[cls][q] += (v.x + v.y) + (v.z + v.w);
                    }
                }
                if (eoff >= 0) {
                    ca.first[cls] += sl[eoff];
                    ca.last[cls] += sl[eoff + G.W - 1];
                }
            }
        }
        conv3_sync<NIW>();
    }
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
}

template <int NIW>
__global__ __launch_bounds__(256) void syrk_conv3_kernel(const SyrkTable tab)
{
    extern __shared__ __align__(16) float lds_dyn[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);

    int pi = 0;
    while (pi + 1 < tab.count && (int)blockIdx.x >= tab.p[pi + 1].blk_start) ++pi;
    const SyrkProb &pr = tab.p[pi];
    const int m = pr.nb;
    const int nbps = wave_blocks_per_split(m);
    const int local = blockIdx.x - pr.blk_start;
    const int split = local / nbps;
    const int b = local - split * nbps;

    const BlockRole r = decode_role(m, b, w, pr.has_bias != 0);
    Conv3Ctx c;
    c.g = conv3_geo((int)(pr.ld >> 40), (int)((pr.ld >> 20) & 0xfffff), (int)(pr.ld & 0xfffff));
    const Conv3Geo &G = c.g;
    c.single = r.single; c.owns_colsum = r.owns_colsum; c.nslots = r.nslots;
    c.rslot = r.rslot; c.cslot = r.cslot; c.ctile0 = r.ctile0;
    c.C = pr.ctot;
    c.w = w; c.lane = lane; c.tid = tid;
    c.no_mfma = (tab.debug & 1) != 0;
    c.no_load = (tab.debug & 2) != 0;
    c.no_issue = (tab.debug & 4) != 0;

    // conv stages of this split
    const long nimg = pr.K / pr.hw;
    const long total = nimg * G.spi;
    c.sg0 = (long)split * pr.tiles_per_split;
    const long sg1 = (c.sg0 + pr.tiles_per_split < total) ? c.sg0 + pr.tiles_per_split : total;
    c.nst = (int)(sg1 - c.sg0);
    c.nstages = (c.nst + (c.single ? 3 : 1) - 1) / (c.single ? 3 : 1);

    {   // raw buffer resource starting one image row BEFORE the tensor (the slab row above the first output
        // row has a non-negative offset that way; it is only ever read when it exists)
        const unsigned long ba = (unsigned long)pr.x - (unsigned long)(G.W * 4);
        c.rsrc.x = (int)(unsigned)ba;
        c.rsrc.y = (int)(unsigned)(ba >> 32);
        c.rsrc.z = (int)(nimg * pr.ctot * pr.hw * 4 + G.W * 4);
        c.rsrc.w = 0x00020000;
    }

    // zero the whole ring once: pad cells are only ever written with zeros afterwards
    const int lds_floats = C3_PRE + C3_NSTAGE * W_SLOTS * G.slab + 256;
    for (int i = tid; i < lds_floats; i += 256) lds_dyn[i] = 0.f;
    float *lds = lds_dyn + C3_PRE;
    c.lds_base = (unsigned)(unsigned long)(__attribute__((address_space(3))) float *)lds;
    __syncthreads();

    Conv3Lanes<NIW> ln;
#pragma unroll
    for (int qi = 0; qi < NIW; ++qi) {
        const int q = w + 4 * qi;
        const int rl = lane / G.LPR, x4 = lane - rl * G.LPR;
        const int row = q * G.RPI + rl;
        const bool part = (rl < G.RPI) && (row < G.rows) && (q < G.NI);
        const int cl = row / G.SR, ir = row - cl * G.SR;
        unsigned f = 0;
        if (part) f |= 1u;
        if (x4 < G.W / 4) f |= 2u;
        if (ir == 0) f |= 4u;
        if (ir == G.SR - 1) f |= 8u;
        ln.flag[qi] = f;
        const unsigned lane_off = (unsigned)((cl * G.H + ir) * G.W * 4 + x4 * 16);
        ln.vo[0][qi] = lane_off + (unsigned)(r.mac0 * 16 * G.H * G.W * 4);
        ln.vo[1][qi] = lane_off + (unsigned)(r.mac1 * 16 * G.H * G.W * 4);
        ln.vo[2][qi] = lane_off + (unsigned)(r.mac2 * 16 * G.H * G.W * 4);
    }

    floatx4 acc[45];
#pragma unroll
    for (int i = 0; i < 45; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
    Conv3ColAcc ca;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
#pragma unroll
        for (int q = 0; q < C3_NIT; ++q) ca.it[k][q] = 0.f;
        ca.first[k] = 0.f;
        ca.last[k] = 0.f;
    }

    if (r.kind == kSingle)     conv3_loop<kSingle, NIW>(c, ln, lds, acc, ca);
    else if (r.kind == kDiag)  conv3_loop<kDiag, NIW>(c, ln, lds, acc, ca);
    else if (r.kind == kHalf5) conv3_loop<kHalf5, NIW>(c, ln, lds, acc, ca);
    else                       conv3_loop<kHalf4, NIW>(c, ln, lds, acc, ca);

    // piece sums -> slab-row sums (fixed order) -> sums of the 144 patch columns of each owned macro tile
    // (the ring is idle now)
    float cs0 = 0.f, cs1 = 0.f;
    if (r.owns_colsum) {
        const int w4 = G.W / 4, nitems = G.rows * w4;
        float *pieces = lds;                         // [2][nitems]
        float *t = lds + 2 * nitems;                 // [2][rows][3]
#pragma unroll
        for (int q = 0; q < C3_NIT; ++q) {
            const int item = tid + 256 * q;
            if (item < nitems) {
                pieces[item] = ca.it[0][q];
                pieces[nitems + item] = ca.it[1][q];
            }
        }
        __syncthreads();
        if (tid < G.rows) {
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                float sum = 0.f;
                for (int x = 0; x < w4; ++x) sum += pieces[k * nitems + tid * w4 + x];
                t[(k * G.rows + tid) * 3 + 0] = sum - ca.last[k];
                t[(k * G.rows + tid) * 3 + 1] = sum;
                t[(k * G.rows + tid) * 3 + 2] = sum - ca.first[k];
            }
        }
        __syncthreads();
        if (tid < W_MT) {
            const int cl = tid / 9, tap = tid - cl * 9;
            const int i = tap / 3, j = tap - i * 3;
            for (int ohl = 0; ohl < G.R; ++ohl) {
                const int row = cl * G.SR + ohl + i;
                cs0 += t[(0 * G.rows + row) * 3 + j];
                cs1 += t[(1 * G.rows + row) * 3 + j];
            }
        }
        __syncthreads();
    }

    wave_epilogue(pr, r, split, w, lane, tid, W_NT, lds, acc, cs0, cs1);
}

}  // namespace kfac

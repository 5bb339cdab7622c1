// A factor of a 3x3 / stride 1 / pad 1 convolution from spatial autocorrelations of its input.
//
// With zero padding, entry ((c,i,j), (c',i',j')) of  A = sum over patches of  a a^T  (Eq. 4 of the DP-KFAC
// paper, the convolution seen as a linear map over patches) is
//     sum_n sum_{a in Ra(i)} sum_{b in Rb(j)}  x[n,c,a,b] * x[n,c',a+di,b+dj],      (di, dj) = (i'-i, j'-j),
// where x is 0 outside the image and Ra(0) = [0,H-2], Ra(1) = [0,H-1], Ra(2) = [1,H-1] (likewise Rb).  The sum
// over ALL (a,b) depends on (di,dj) only: the autocorrelation F(di,dj)[c][c'] of the input at one of 25 lags,
// of which 13 are independent (F(-d)[c][c'] = F(d)[c'][c]).  What the window removes is a single image row
// (for i = 0 or 2) and/or a single column (j = 0 or 2), and such a term is non-zero only when the partner
// lands in the same row (i' = i) resp. column (j' = j):
//     A = F(d) - [i'=i in {0,2}] Row(a*, dj) - [j'=j in {0,2}] Col(b*, di) + [both] Corner(a*, b*),
// with a* = H-1 for i = 0 and 0 for i = 2 (b* likewise), Row / Col the 1-D autocorrelations of that border
// row / column and Corner the outer product of the corner pixel.  The bias border (column sums of the patch
// matrix) follows the same inclusion-exclusion on plain sums.  The result is the same matrix as the direct
// sum (up to rounding order) for 13 instead of 45 MFMA tiles per 16 x 16 channel pair and k-step.
//
// Three steps: corr3_main_kernel (the 13 lag matrices, split over images, on the MFMA units),
// corr3_border_kernel (rows, columns, corners; MFMA as well, K = border pixels), corr3_sum_kernel +
// corr3_assemble_kernel (sum of the splits, assembly of A with scale and running average, both triangles).
#pragma once

#include "common.hpp"
#include "tn_engine.hpp"
#include "wave_common.hpp"

namespace kfac {

constexpr int C3_LAGS = 13;
constexpr int C3_BQ = 16;          // border matrices per layer: 6 row, 6 column, 4 corner
constexpr int C3_BV = 8;           // border vectors per layer: 2 row sums, 2 column sums, 4 corner sums
constexpr int C3_CHUNKS = 5;       // image chunks of the border kernels (5 x 4 pair groups x 36 layers = 720 workgroups at 64 channels: under 3 per CU)

struct CorrProb {
    const float *x;    // NCHW input [B, C, H, W]
    float *Fp;         // [parts][13][C][C] lag matrices per part, then [parts][C] channel sums per part
    float *Fs;         // [13][C][C] + [C]: summed over the parts
    float *Bp;         // [chunks][16][C][C], then [chunks][8][C]
    float *Bs;         // [16][C][C] + [8][C]: summed over the chunks
    float *FsT, *BsT;  // the matrices of Fs and Bs transposed ([l][c'][c]): the assembly reads both orders along rows
    float *cols;       // [B][2][C][H]: first and last image column, written by the main kernel for the border kernel
    float *F;          // factor [dF, dF], dF = 9 C + has_bias
    int C, H, W, B;
    int SR, strips;    // rows per strip, strips per image
    int units;         // B * strips
    int splits, upb;   // blocks of the main kernel, units per block
    int parts;         // splits * (wavefronts that split the k-steps)
    int plane;         // floats per channel plane of a slab
    int blk_start;     // first block of this problem in the kernel at hand
    int has_bias;
    float scale, decay;
};

struct CorrTable {
    int count;
    int starts[kMaxProblems];     // blk_start of every problem, compact: searched by bisection
    CorrProb p[kMaxProblems];
};

__device__ __forceinline__ int corr_locate(const CorrTable &tab, int blk)
{
    int lo = 0, hi = tab.count - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (blk >= tab.starts[mid]) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}

// ---------------------------------------------------------------------------------------------------------
// Lag matrices.  A workgroup (four product and four staging wavefronts) walks (image, strip) units: the strip of
// all C channels with two halo rows below is staged in LDS (double buffered, the next unit's global loads in
// flight under the products) with four zero columns left and right; the A operand of a k-step is channel tile
// ct at four pixels, the B operand channel tile ct' at the pixels shifted by the lag.
//   NT = 1 (C = 16): one tile pair; the four product wavefronts take every fourth group (four parts per block).
//   NT = 2 (C = 32): four tile pairs, one per product wavefront.
//   NT = 4 (C = 64): product wavefront w = A tile w and two of the four B tiles; two workgroups share a range of
//   units (all 52 lag tiles per wavefront would leave one wavefront per SIMD).
template <int NT>
__global__ __launch_bounds__(512) void corr3_main_kernel(const CorrTable tab)
{
    extern __shared__ __align__(16) float corr_lds[];
    constexpr int C = 16 * NT;
    constexpr int KS = NT == 1 ? 4 : 1;        // wavefronts that split the pixel groups
    constexpr int PW = NT == 4 ? 2 : 1;        // B tiles per wavefront
    constexpr int HALVES = NT == 4 ? 2 : 1;    // workgroups that share a range of units (each takes half the B tiles)
    constexpr int SCI = 2;                     // border-column cells per staging thread with a precomputed address

    const CorrProb &pr = tab.p[corr_locate(tab, blockIdx.x)];
    const int blk_raw = blockIdx.x - pr.blk_start;
    const int blk = blk_raw / HALVES, half = blk_raw - blk * HALVES;
    const int u0 = blk * pr.upb, u1 = min(pr.units, u0 + pr.upb);
    const int lane = threadIdx.x & 63, w8 = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int H = pr.H, W = pr.W, Wp = W + 8, SR = pr.SR, plane = pr.plane, w4 = W >> 2;
    float *buf0 = corr_lds, *buf1 = corr_lds + C * plane;

    // Wavefronts 4 .. 7 stage the slabs, wavefronts 0 .. 3 only read operands and issue products.  Workgroups
    // that share a CU advance at the same pace (the MFMA unit alternates between their wavefronts), so staging
    // done by the product wavefronts themselves would fall into the same moments in all of them and leave the
    // MFMA unit idle; as wavefronts of their own the loads, LDS stores and address arithmetic run beside it.
    // One barrier per unit: past barrier `it` the slab of unit `it` is complete and every product wavefront is
    // done with unit it - 1, whose buffer the staging wavefronts then fill with unit it + 1.
    if (w8 >= 4) {
        const int tid = threadIdx.x - 256;
        // The slab is filled by global -> LDS copies of 1 KB (64 lanes x 16 bytes, consecutive in LDS): instruction
        // i of a slab covers its 16-byte cells 64 i .. 64 i + 63; a lane whose cell is a pixel piece reads it from
        // the input, a lane whose cell is padding (the four columns either side of a row, the tail of a plane)
        // reads out of range, which stores zeros, and so does a halo row below the image.  Per unit that is at
        // most MAXD copies per wavefront with precomputed lane offsets and one scalar base: every instruction of
        // these wavefronts takes an issue slot from the product wavefronts of its SIMD.
        constexpr int MAXD = 9;                    // copies per wavefront and slab at most (checked by the planner)
        const int rows = SR + 2;
        const int cells = C * plane / 4, ninstr = (cells + 63) / 64;
        const int lw = w8 - 4;
        unsigned vo[MAXD];
        int vr[MAXD];                              // slab row of the cell (rows below the image are masked per unit)
        bool vlive[MAXD];
#pragma unroll
        for (int j = 0; j < MAXD; ++j) {
            const int q = (lw + 4 * j) * 64 + lane;
            vo[j] = W_OOB;
            vr[j] = 0;
            vlive[j] = lw + 4 * j < ninstr && q < cells;
            if (vlive[j]) {
                const int f = 4 * q, c = f / plane, rem = f - c * plane;
                const int r = rem / Wp, x = rem - r * Wp;
                vr[j] = r;
                if (r < rows && x >= 4 && x < 4 + W) vo[j] = (unsigned)(((c * H + r) * W + x - 4) * 4);
            }
        }
        int4v rsrc;
        {
            const unsigned long ba = (unsigned long)pr.x;
            rsrc.x = (int)(unsigned)ba;
            rsrc.y = (int)(unsigned)(ba >> 32);
            rsrc.z = (int)((long)pr.B * C * H * W * 4);          // below 2^31 (checked by the planner)
            rsrc.w = 0x00020000;
        }
        const unsigned lds0 = (unsigned)(unsigned long)(__attribute__((address_space(3))) float *)corr_lds;
        const unsigned slab_bytes = (unsigned)(C * plane * 4);
        auto issue = [&](unsigned dst, int u) {
            const int n = u / pr.strips, a0 = (u - n * pr.strips) * SR;
            const unsigned so = (unsigned)((n * C * H + a0) * W) * 4u;
            const bool tail = a0 + rows > H;       // uniform: this slab reaches below the image
#pragma unroll
            for (int j = 0; j < MAXD; ++j) {
                if (lw + 4 * j < ninstr) {         // uniform
                    const unsigned v = (tail && a0 + vr[j] >= H) ? W_OOB : vo[j];
                    const unsigned to = (unsigned)__builtin_amdgcn_readfirstlane((int)(dst + (unsigned)(lw + 4 * j) * 1024u));
                    if (vlive[j]) dma16(to, v, rsrc, (unsigned)__builtin_amdgcn_readfirstlane((int)so));
                }
            }
        };
        // the first and the last pixel of every image row also go to a compact buffer (the border kernel would
        // otherwise pull a whole cache line per pixel of those two columns): read back from the slab,
        // consecutive threads = consecutive rows of a channel
        int sc_l[SCI], sc_g[SCI];
#pragma unroll
        for (int j = 0; j < SCI; ++j) {
            const int t = tid + 256 * j;
            sc_l[j] = -1;
            sc_g[j] = 0;
            if (NT != 4 && t < 2 * C * SR) {
                const int side = t / (C * SR), rem = t - side * (C * SR);
                const int c = rem / SR, r = rem - c * SR;
                sc_l[j] = c * plane + r * Wp + 4 + (side ? W - 1 : 0);
                sc_g[j] = (side * C + c) * H + r;
            }
        }
        auto save_cols = [&](const float *b, int u) {
            if (NT == 4) return;             // 64 channels: short columns, the border kernel reads them from the input
            const int n = u / pr.strips, a0 = (u - n * pr.strips) * SR;
            float *cbase = pr.cols + (long)n * 2 * C * H + a0;
#pragma unroll
            for (int j = 0; j < SCI; ++j)
                if (sc_l[j] >= 0) cbase[sc_g[j]] = b[sc_l[j]];
            for (int t = tid + 256 * SCI; t < 2 * C * SR; t += 256) {
                const int side = t / (C * SR), rem = t - side * (C * SR);
                const int c = rem / SR, r = rem - c * SR;
                cbase[(side * C + c) * H + r] = b[c * plane + r * Wp + 4 + (side ? W - 1 : 0)];
            }
        };
        if (u0 < u1) issue(lds0, u0);
        for (int u = u0, it = 0; u < u1; ++u, ++it) {
            float *b = (it & 1) ? buf1 : buf0;
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");    // the copies of this unit have landed
            __syncthreads();
            // the other buffer is free now: every product wavefront is past unit it - 1
            if (u + 1 < u1) issue(lds0 + ((it & 1) ? 0u : slab_bytes), u + 1);
            save_cols(b, u);                    // the slab stays as it is until the barrier after next
        }
        return;
    }

    const int w = w8;
    const int lr = lane & 15, kk = lane >> 4;
    int ct, ctp0;
    if (NT == 1) { ct = 0; ctp0 = 0; }
    else if (NT == 2) { ct = w >> 1; ctp0 = w & 1; }
    else { ct = w; ctp0 = 2 * half; }

    floatx4 acc[PW][C3_LAGS];
#pragma unroll
    for (int p = 0; p < PW; ++p)
#pragma unroll
        for (int l = 0; l < C3_LAGS; ++l) acc[p][l] = floatx4{0.f, 0.f, 0.f, 0.f};
    float tsum = 0.f;

    // A group is 16 consecutive pixels of the strip (row-major); lane kk holds pixels 4 kk .. 4 kk + 3 of it and
    // k-step e of the group takes pixel 4 kk + e from every lane.  For the shifted operand a lane reads, per
    // row lag, the window around its four pixels: every lag (di, dj) of k-step e is element e + dj of the window
    // of row di, a register chosen at compile time.
    // A stage is one group and one B tile: 52 products on 9 operand reads.  Two register sets alternate, the
    // reads of the next stage are issued before the products of the current one (all wavefronts of a SIMD
    // advance at the same pace, so none of them would cover the read latency of another).
    const int ngroups = SR * W / 16;
    const int gfirst = (KS == 4) ? w : 0;
    const int nstages = ((ngroups - gfirst + KS - 1) / KS) * PW;
    const int q0 = 16 * gfirst + 4 * kk;                       // first pixel of this lane in its first group
    const int row0 = q0 / W, col0 = q0 - row0 * W;
    const int drow = (16 * KS) / W, dcol = 16 * KS - drow * W;  // from a group to the next of this wavefront
    for (int u = u0, it = 0; u < u1; ++u, ++it) {
        float *b = (it & 1) ? buf1 : buf0;
        __syncthreads();
        const float *pa = b + (16 * ct + lr) * plane + 4;
        const float *pb[PW];
#pragma unroll
        for (int p = 0; p < PW; ++p) pb[p] = b + (16 * (ctp0 + p) + lr) * plane + 4;
        // operand registers of a set: the four pixels of the A tile, and per row lag the window elements that
        // some lag uses (pixels -2 .. 5 around the lane's first pixel; 0 .. 5 for row lag 0), read as 8 + 16 + 8 bytes
        typedef float floatx2 __attribute__((ext_vector_type(2)));
        floatx4 a4[2], wmid[2][3];
        floatx2 wlo[2][3], whi[2][3];
        auto load = [&](int set, int base, int p) {
            a4[set] = *reinterpret_cast<const floatx4 *>(pa + base);
#pragma unroll
            for (int di = 0; di < 3; ++di) {
                const float *q = pb[p] + base + di * Wp;
                if (di > 0) wlo[set][di] = *reinterpret_cast<const floatx2 *>(q - 2);
                wmid[set][di] = *reinterpret_cast<const floatx4 *>(q);
                whi[set][di] = *reinterpret_cast<const floatx2 *>(q + 4);
            }
        };
        auto products = [&](int set, int p) {
            if (p == 0) tsum += (a4[set].x + a4[set].y) + (a4[set].z + a4[set].w);
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int l = 0; l < C3_LAGS; ++l) {
                    const int di = l < 3 ? 0 : (l < 8 ? 1 : 2);
                    const int dj = l < 3 ? l : (l < 8 ? l - 5 : l - 10);
                    const int idx = e + dj;                           // -2 .. 5 relative to the lane's first pixel
                    const float bv = idx < 0 ? wlo[set][di][idx + 2] : (idx < 4 ? wmid[set][di][idx] : whi[set][di][idx - 4]);
                    acc[p][l] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[set][e], bv, acc[p][l], 0, 0, 0);
                }
        };
        // Positions run one stage ahead of the reads, which run one stage ahead of the products: no address
        // arithmetic and no branch between the reads of a stage and the products before them.
        int row = row0, col = col0;
        auto advance = [&](bool take, int base) {               // next group of this wavefront, if there is one
            int c = col + dcol, r = row + drow;
            const bool wrap = c >= W;
            c -= wrap ? W : 0;
            r += wrap ? 1 : 0;
            col = take ? c : col;
            row = take ? r : row;
            return take ? r * Wp + c : base;
        };
        const int b0 = row0 * Wp + col0;
        if (nstages > 0) load(0, b0, 0);        // a wavefront without a group has no valid address to read
        int b1 = PW == 1 ? advance(1 < nstages, b0) : b0;
        for (int s = 0; s < nstages; s += 2) {
            // stage s sits in set 0; with two B tiles per wavefront stage s + 1 is the same group, second tile.
            // The reads are unconditional (past the last stage they repeat a valid address and are dropped):
            // reads under a branch of their own would be moved down to the products that use them.
            const bool more1 = s + 1 < nstages;
            load(1, b1, PW - 1);
            const int b2 = advance(s + 2 < nstages, b1);
            products(0, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 9, 0);      // the reads first,
            __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);      // the address arithmetic under the products
            __builtin_amdgcn_sched_group_barrier(0x002, 16, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 48, 0);
            if (more1) {
                load(0, b2, 0);
                b1 = PW == 1 ? advance(s + 3 < nstages, b2) : b2;
                products(1, PW - 1);
                __builtin_amdgcn_sched_group_barrier(0x100, 9, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 16, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 48, 0);
            }
        }
    }

    // channel sums: the four k-lanes of a channel
    tsum += __shfl_xor(tsum, 16);
    tsum += __shfl_xor(tsum, 32);
    const int part = blk * KS + (KS == 4 ? w : 0);
    float *Fo = pr.Fp + (long)part * (C3_LAGS * C * C);
#pragma unroll
    for (int p = 0; p < PW; ++p)
#pragma unroll
        for (int l = 0; l < C3_LAGS; ++l)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                Fo[(l * C + 16 * ct + 4 * kk + v) * C + 16 * (ctp0 + p) + lr] = acc[p][l][v];
    if (ctp0 == 0 && kk == 0)
        pr.Fp[(long)pr.parts * (C3_LAGS * C * C) + (long)part * C + 16 * ct + lr] = tsum;
}

// ---------------------------------------------------------------------------------------------------------
// Border terms.  One workgroup per (layer, side, image chunk); side 0 / 1 = image row 0 / H-1, 2 / 3 = column
// 0 / W-1, 4 = the four corners.  For a row or column: per image the line [C][L] (+2 zero cells) is staged in
// LDS, a k-step is four consecutive pixels of the line, lags 0, 1, 2.  Corners: the "line" of a corner is its
// value in the images of the chunk (k runs over images), lag 0 only.
// Wavefront w takes the channel-tile pairs w, w + 4, ...
template <int NT>
__global__ __launch_bounds__(256) void corr3_border_kernel(const CorrTable tab)
{
    constexpr int C = 16 * NT;
    constexpr int NP = NT * NT;                       // tile pairs
    constexpr int PPW = (NP + 3) / 4;                 // pairs per wavefront
    constexpr int LMAX = 64 + 4;
    __shared__ float line[C * LMAX];

    const CorrProb &pr = tab.p[corr_locate(tab, blockIdx.x)];
    const int local = blockIdx.x - pr.blk_start;
    const int side = local / C3_CHUNKS, ch = local - side * C3_CHUNKS;
    const int per = (pr.B + C3_CHUNKS - 1) / C3_CHUNKS;
    const int n0 = ch * per, n1 = min(pr.B, n0 + per);
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int lr = lane & 15, kk = lane >> 4;
    const int H = pr.H, W = pr.W;
    float *Bm = pr.Bp + (long)ch * (C3_BQ * C * C);
    float *Bv = pr.Bp + (long)C3_CHUNKS * (C3_BQ * C * C) + (long)ch * (C3_BV * C);

    if (side < 4) {
        const bool is_row = side < 2;
        const int L = is_row ? W : H;                 // line length (a multiple of 4 for rows; any for columns)
        const int fixed = (side & 1) ? (is_row ? H - 1 : W - 1) : 0;
        for (int i = tid; i < C * LMAX; i += 256) line[i] = 0.f;
        floatx4 acc[PPW][3];
#pragma unroll
        for (int p = 0; p < PPW; ++p)
#pragma unroll
            for (int l = 0; l < 3; ++l) acc[p][l] = floatx4{0.f, 0.f, 0.f, 0.f};
        float vs[PPW];
#pragma unroll
        for (int p = 0; p < PPW; ++p) vs[p] = 0.f;
        const int nks = (L + 3) / 4;
        // the elements of the line this thread moves (same for every image): global offset inside an image, LDS index
        constexpr int EPT = (C * 64 + 255) / 256;
        int goff[EPT], loff[EPT];
        constexpr int DEPTH = 4;                              // images whose loads are in flight
        float nxt[DEPTH][EPT];
#pragma unroll
        for (int k = 0; k < EPT; ++k) {
            const int i = tid + 256 * k;
            goff[k] = -1;
            loff[k] = 0;
            if (i < C * L) {
                const int c = i / L, p = i - c * L;
                goff[k] = is_row ? (c * H + fixed) * W + p
                                 : (NT == 4 ? (c * H + p) * W + fixed : ((side & 1) * C + c) * H + p);   // columns: compact buffer below 64 channels
                loff[k] = c * LMAX + p;
            }
        }
#pragma unroll
        for (int j = 0; j < DEPTH; ++j) {
            if (n0 + j < n1) {
                const float *img = (is_row || NT == 4) ? pr.x + (long)(n0 + j) * C * H * W : pr.cols + (long)(n0 + j) * 2 * C * H;
#pragma unroll
                for (int k = 0; k < EPT; ++k) nxt[j][k] = goff[k] >= 0 ? img[goff[k]] : 0.f;
            }
        }
        for (int nb = n0; nb < n1; nb += DEPTH) {
#pragma unroll
            for (int j = 0; j < DEPTH; ++j) {
                const int n = nb + j;
                if (n >= n1) break;
                __syncthreads();                              // the products on the previous line are done
#pragma unroll
                for (int k = 0; k < EPT; ++k)
                    if (goff[k] >= 0) line[loff[k]] = nxt[j][k];
                __syncthreads();
                if (n + DEPTH < n1) {                         // refill this register set: in flight for DEPTH lines
                    const float *img = (is_row || NT == 4) ? pr.x + (long)(n + DEPTH) * C * H * W
                                                            : pr.cols + (long)(n + DEPTH) * 2 * C * H;
#pragma unroll
                    for (int k = 0; k < EPT; ++k) nxt[j][k] = goff[k] >= 0 ? img[goff[k]] : 0.f;
                }
#pragma unroll
                for (int p = 0; p < PPW; ++p) {
                    const int pair = w + 4 * p;
                    if (pair >= NP) continue;
                    const int ct = pair / NT, ctp = pair - ct * NT;
                    const float *pa = line + (16 * ct + lr) * LMAX + kk;
                    const float *pb = line + (16 * ctp + lr) * LMAX + kk;
                    for (int ks = 0; ks < nks; ++ks) {
                        const float a = pa[4 * ks];
                        if (ctp == 0) vs[p] += a;
#pragma unroll
                        for (int l = 0; l < 3; ++l)
                            acc[p][l] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, pb[4 * ks + l], acc[p][l], 0, 0, 0);
                    }
                }
            }
        }
#pragma unroll
        for (int p = 0; p < PPW; ++p) {
            const int pair = w + 4 * p;
            if (pair >= NP) continue;
            const int ct = pair / NT, ctp = pair - ct * NT;
#pragma unroll
            for (int l = 0; l < 3; ++l)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    Bm[((3 * side + l) * C + 16 * ct + 4 * kk + v) * C + 16 * ctp + lr] = acc[p][l][v];
            float s = vs[p];
            s += __shfl_xor(s, 16);
            s += __shfl_xor(s, 32);
            if (ctp == 0 && kk == 0) Bv[side * C + 16 * ct + lr] = s;
        }
    } else {
        // corners: line[q][c][k] = value of corner q of channel c in image n0 + k
        const int nimg = n1 - n0;                     // at most LMAX - 4 (checked by the planner)
        floatx4 acc[PPW][4];
#pragma unroll
        for (int p = 0; p < PPW; ++p)
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[p][q] = floatx4{0.f, 0.f, 0.f, 0.f};
        float vs[PPW][4];
#pragma unroll
        for (int p = 0; p < PPW; ++p)
#pragma unroll
            for (int q = 0; q < 4; ++q) vs[p][q] = 0.f;
        const int nks = (nimg + 3) / 4;
        for (int q = 0; q < 4; ++q) {
            const int a = (q & 2) ? H - 1 : 0, b = (q & 1) ? W - 1 : 0;
            // one cache line per value: all loads of a thread in flight before the first is stored
            constexpr int EPC = (C * LMAX + 255) / 256;
            float val[EPC];
#pragma unroll
            for (int e = 0; e < EPC; ++e) {
                const int i = tid + 256 * e;
                const int c = i / LMAX, k = i - c * LMAX;
                const bool ok = i < C * LMAX && k < nimg;
                const float v = pr.x[ok ? (((long)(n0 + k) * C + c) * H + a) * W + b : 0];
                val[e] = ok ? v : 0.f;
            }
            __syncthreads();
#pragma unroll
            for (int e = 0; e < EPC; ++e) {
                const int i = tid + 256 * e;
                if (i < C * LMAX) line[i] = val[e];
            }
            __syncthreads();
#pragma unroll
            for (int p = 0; p < PPW; ++p) {
                const int pair = w + 4 * p;
                if (pair >= NP) continue;
                const int ct = pair / NT, ctp = pair - ct * NT;
                const float *pa = line + (16 * ct + lr) * LMAX + kk;
                const float *pb = line + (16 * ctp + lr) * LMAX + kk;
                for (int ks = 0; ks < nks; ++ks) {
                    const float av = pa[4 * ks];
                    if (ctp == 0) vs[p][q] += av;
                    acc[p][q] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, pb[4 * ks], acc[p][q], 0, 0, 0);
                }
            }
        }
#pragma unroll
        for (int p = 0; p < PPW; ++p) {
            const int pair = w + 4 * p;
            if (pair >= NP) continue;
            const int ct = pair / NT, ctp = pair - ct * NT;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    Bm[((12 + q) * C + 16 * ct + 4 * kk + v) * C + 16 * ctp + lr] = acc[p][q][v];
                float s = vs[p][q];
                s += __shfl_xor(s, 16);
                s += __shfl_xor(s, 32);
                if (ctp == 0 && kk == 0) Bv[(4 + q) * C + 16 * ct + lr] = s;
            }
        }
    }
}

// Border terms of small maps (H * W <= 64, 32 or 64 channels), where rows, columns and corners together are a
// large part of every plane and gathering them side by side pulls the input several times over: a workgroup
// stages whole images (contiguous, read once per group of channel-tile pairs) and takes all sixteen border
// matrices from LDS.  One workgroup per (layer, image chunk, group of four tile pairs), one pair per wavefront;
// the loads of two images are in flight.
// Cells past the end of a line are masked in the operand, not padded.
template <int NT>
__global__ __launch_bounds__(256) void corr3_border_plane_kernel(const CorrTable tab)
{
    constexpr int C = 16 * NT;
    constexpr int NG = NT * NT / 4;                   // groups of four tile pairs
    constexpr int PL = 64 + 4;                        // cells per channel plane in LDS
    constexpr int DEPTH = 2;                          // images whose loads are in flight (more would cost a wavefront per SIMD)
    __shared__ __align__(16) float img[C * PL];

    const CorrProb &pr = tab.p[corr_locate(tab, blockIdx.x)];
    const int local = blockIdx.x - pr.blk_start;
    const int ch = local / NG, pg = local - ch * NG;
    const int per = (pr.B + C3_CHUNKS - 1) / C3_CHUNKS;
    const int n0 = ch * per, n1 = min(pr.B, n0 + per);
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lr = lane & 15, kk = lane >> 4;
    const int H = pr.H, W = pr.W, HW = H * W;
    const int pair = 4 * pg + w, ct = pair / NT, ctp = pair - ct * NT;
    float *Bm = pr.Bp + (long)ch * (C3_BQ * C * C);
    float *Bv = pr.Bp + (long)C3_CHUNKS * (C3_BQ * C * C) + (long)ch * (C3_BV * C);

    // what this thread moves per image: float4 f of the image -> plane c, cell p
    int gofs[NT], lofs[NT];
#pragma unroll
    for (int k = 0; k < NT; ++k) {
        const int e = 4 * (tid + 256 * k);
        gofs[k] = -1;
        lofs[k] = 0;
        if (e < C * HW) {
            const int c = e / HW;
            gofs[k] = e;
            lofs[k] = c * PL + (e - c * HW);
        }
    }
    floatx4 regs[DEPTH][NT];
    auto fetch = [&](int j, int n) {
        const float *src = pr.x + (long)n * C * HW;
#pragma unroll
        for (int k = 0; k < NT; ++k) regs[j][k] = *reinterpret_cast<const floatx4 *>(src + (gofs[k] >= 0 ? gofs[k] : 0));
    };
    // matrices: 3 * side + lag for the sides row 0, row H-1, column 0, column W-1, then the four corners;
    // vectors: the four sides, then the four corners
    floatx4 acc[C3_BQ];
    float vs[C3_BV];
#pragma unroll
    for (int m = 0; m < C3_BQ; ++m) acc[m] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int m = 0; m < C3_BV; ++m) vs[m] = 0.f;
    const float *pa = img + (16 * ct + lr) * PL;
    const float *pb = img + (16 * ctp + lr) * PL;

    // one k-step of the two sides of a direction: position p = 4 ks + kk of the line, cells org + p * step
    auto lines = [&](int L, int step, int org1, int m0, int v0) {
        const int nks = (L + 3) / 4;
#pragma unroll 2
        for (int ks = 0; ks < nks; ++ks) {
            const int p = 4 * ks + kk;
            const int c0 = min(p, L - 1) * step, c1 = min(p + 1, L - 1) * step, c2 = min(p + 2, L - 1) * step;
            // all eight operand cells first, then the six products; cells past the end of the line are masked
            const float a0 = pa[c0], b00 = pb[c0], b01 = pb[c1], b02 = pb[c2];
            const float a1 = pa[org1 + c0], b10 = pb[org1 + c0], b11 = pb[org1 + c1], b12 = pb[org1 + c2];
            const bool in0 = p < L, in1 = p + 1 < L, in2 = p + 2 < L;
            const float a0m = in0 ? a0 : 0.f, a1m = in0 ? a1 : 0.f;
            vs[v0] += a0m;
            vs[v0 + 1] += a1m;
            acc[m0 + 0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0m, in0 ? b00 : 0.f, acc[m0 + 0], 0, 0, 0);
            acc[m0 + 1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0m, in1 ? b01 : 0.f, acc[m0 + 1], 0, 0, 0);
            acc[m0 + 2] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0m, in2 ? b02 : 0.f, acc[m0 + 2], 0, 0, 0);
            acc[m0 + 3] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1m, in0 ? b10 : 0.f, acc[m0 + 3], 0, 0, 0);
            acc[m0 + 4] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1m, in1 ? b11 : 0.f, acc[m0 + 4], 0, 0, 0);
            acc[m0 + 5] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1m, in2 ? b12 : 0.f, acc[m0 + 5], 0, 0, 0);
        }
    };

#pragma unroll
    for (int j = 0; j < DEPTH; ++j)
        if (n0 + j < n1) fetch(j, n0 + j);
    for (int nb = n0; nb < n1; nb += DEPTH) {
#pragma unroll
        for (int j = 0; j < DEPTH; ++j) {
            const int n = nb + j;
            if (n >= n1) break;
            __syncthreads();                          // the products on the previous image are done
#pragma unroll
            for (int k = 0; k < NT; ++k)
                if (gofs[k] >= 0) *reinterpret_cast<floatx4 *>(img + lofs[k]) = regs[j][k];
            __syncthreads();
            if (n + DEPTH < n1) fetch(j, n + DEPTH);  // refill this register set: in flight for DEPTH images
            float av[4], bv[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int cell = ((q & 2) ? (H - 1) * W : 0) + ((q & 1) ? W - 1 : 0);
                av[q] = pa[cell];
                bv[q] = pb[cell];
            }
            lines(W, 1, (H - 1) * W, 0, 0);           // rows 0 and H-1: k runs along the row
            lines(H, W, W - 1, 6, 2);                 // columns 0 and W-1: k runs down the column
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                // a corner is a single cell: only k = 0 of the step carries it
                const float a = kk == 0 ? av[q] : 0.f;
                vs[4 + q] += a;
                acc[12 + q] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, bv[q], acc[12 + q], 0, 0, 0);
            }
        }
    }

#pragma unroll
    for (int m = 0; m < C3_BQ; ++m)
#pragma unroll
        for (int v = 0; v < 4; ++v) Bm[((long)m * C + 16 * ct + 4 * kk + v) * C + 16 * ctp + lr] = acc[m][v];
#pragma unroll
    for (int m = 0; m < C3_BV; ++m) {
        float sm = vs[m];
        sm += __shfl_xor(sm, 16);
        sm += __shfl_xor(sm, 32);
        if (ctp == 0 && kk == 0) Bv[m * C + 16 * ct + lr] = sm;
    }
}

// Sums over the parts (lag matrices, channel sums) and over the image chunks (border terms), fixed order.
__global__ __launch_bounds__(256) void corr3_sum_kernel(const CorrTable tab)
{
    const CorrProb &pr = tab.p[corr_locate(tab, blockIdx.x)];
    const int C = pr.C, cc = C * C;
    const long nF = (long)C3_LAGS * cc, nB = (long)C3_BQ * cc;
    const long qF = nF / 4, qB = nB / 4;            // matrices: four consecutive elements (one row) per thread
    const long q = (long)(blockIdx.x - pr.blk_start) * 256 + threadIdx.x;
    auto store_both = [&](float *dst, float *dstT, long e, const floatx4 &v) {
        *reinterpret_cast<floatx4 *>(dst + e) = v;
        const int l = (int)(e / cc), rem = (int)(e - (long)l * cc), c = rem / C, c2 = rem - c * C;
        float *t = dstT + (long)l * cc + (long)c2 * C + c;
#pragma unroll
        for (int i = 0; i < 4; ++i) t[(long)i * C] = v[i];
    };
    if (q < qF) {
        // four interleaved running sums (fixed order) keep loads in flight
        const long e = 4 * q;
        floatx4 a[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) a[j] = floatx4{0.f, 0.f, 0.f, 0.f};
        int p = 0;
        for (; p + 4 <= pr.parts; p += 4)
#pragma unroll
            for (int j = 0; j < 4; ++j) a[j] += *reinterpret_cast<const floatx4 *>(pr.Fp + (long)(p + j) * nF + e);
        for (; p < pr.parts; ++p) a[0] += *reinterpret_cast<const floatx4 *>(pr.Fp + (long)p * nF + e);
        store_both(pr.Fs, pr.FsT, e, (a[0] + a[1]) + (a[2] + a[3]));
    } else if (q < qF + qB) {
        const long i = 4 * (q - qF);
        floatx4 sum = {0.f, 0.f, 0.f, 0.f};
        for (int k = 0; k < C3_CHUNKS; ++k) sum += *reinterpret_cast<const floatx4 *>(pr.Bp + (long)k * nB + i);
        store_both(pr.Bs, pr.BsT, i, sum);
    } else if (q < qF + qB + C) {
        const long c = q - qF - qB;
        float sum = 0.f;
        for (int p = 0; p < pr.parts; ++p) sum += pr.Fp[(long)pr.parts * nF + (long)p * C + c];
        pr.Fs[nF + c] = sum;
    } else if (q < qF + qB + C + C3_BV * C) {
        const long i = q - qF - qB - C;
        float sum = 0.f;
        for (int k = 0; k < C3_CHUNKS; ++k) sum += pr.Bp[(long)C3_CHUNKS * nB + (long)k * (C3_BV * C) + i];
        pr.Bs[nB + i] = sum;
    }
}

// Assembly of A from the lag matrices and the border terms, with scale and running average.  A wavefront
// takes three rows of A (input channel c, kernel row i), lane c2 their entries for the channel pair (c, c2):
// every lag matrix and border matrix is read once at [c][c2] and once at [c2][c] (F(-d)[c][c'] = F(d)[c'][c]; the
// summation kernel leaves a transposed copy, so both reads run along rows),
// and which of them enters element ((i,j), (i',j')) is known at compile time.  The nine values of a lane per
// row go to an LDS strip and are read back along the row of A, so the old factor is read and the new one
// stored in whole rows; both triangles are computed, nothing is stored transposed.  The wavefront after the
// last channel writes the bias row.
constexpr int C3_ARW = 4;          // row triples (wavefronts) per workgroup

template <int I>
__device__ __forceinline__ void corr3_assemble_rows(const CorrProb &pr, int c, int lane, float *st)
{
    const int C = pr.C, d = 9 * C, dF = d + pr.has_bias;
    const float *Fs = pr.Fs, *Ts = pr.Fs + (long)C3_LAGS * C * C;
    const float *Bs = pr.Bs, *Bv = pr.Bs + (long)C3_BQ * C * C;
    const float wnew = (1.0f - pr.decay) * pr.scale, decay = pr.decay;
    const int c2 = lane < C ? lane : 0;                              // idle lanes repeat a valid address
    // the old rows (clamped addresses: no branch, all loads in flight at once) and the bias column entries:
    // column sum of patch column (c, I, j) = all pixels minus the removed row / column plus the corner
    float old[3][9], oldb[3];
#pragma unroll
    for (int j = 0; j < 3; ++j) {
        const float *row = pr.F + (long)(9 * c + 3 * I + j) * dF;
#pragma unroll
        for (int k = 0; k < 9; ++k) old[j][k] = row[min(lane + 64 * k, dF - 1)];
        float t = Ts[c];
        if (I != 1) t -= Bv[(I == 0 ? 1 : 0) * C + c];
        if (j != 1) t -= Bv[(j == 0 ? 3 : 2) * C + c];
        if (I != 1 && j != 1) t += Bv[(4 + (I == 0 ? 2 : 0) + (j == 0 ? 1 : 0)) * C + c];
        oldb[j] = decay * row[dF - 1] + wnew * t;
    }
    float Fp[C3_LAGS], Fn[C3_LAGS], Rp[4][3], Rn[4][3], Cq[4];
#pragma unroll
    for (int l = 0; l < C3_LAGS; ++l) {
        Fp[l] = Fs[((long)l * C + c) * C + c2];
        Fn[l] = pr.FsT[((long)l * C + c) * C + c2];
    }
#pragma unroll
    for (int sd = 0; sd < 4; ++sd)
#pragma unroll
        for (int lag = 0; lag < 3; ++lag) {
            Rp[sd][lag] = Bs[((long)(3 * sd + lag) * C + c) * C + c2];
            Rn[sd][lag] = pr.BsT[((long)(3 * sd + lag) * C + c) * C + c2];
        }
#pragma unroll
    for (int q = 0; q < 4; ++q) Cq[q] = Bs[((long)(12 + q) * C + c) * C + c2];
#pragma unroll
    for (int j = 0; j < 3; ++j) {
#pragma unroll
        for (int ij2 = 0; ij2 < 9; ++ij2) {
            const int i2 = ij2 / 3, j2 = ij2 - 3 * i2;
            const int di = i2 - I, dj = j2 - j;
            const bool pos = di > 0 || (di == 0 && dj >= 0);
            const int adi = pos ? di : -di, adj = pos ? dj : -dj;
            const int l = adi == 0 ? adj : (adi == 1 ? 5 + adj : 10 + adj);
            float val = pos ? Fp[l] : Fn[l];
            if (i2 == I && I != 1) {          // removed row a* = H-1 (i = 0) or 0 (i = 2); lag j2 - j along the row
                const int sd = I == 0 ? 1 : 0;
                val -= dj >= 0 ? Rp[sd][dj >= 0 ? dj : 0] : Rn[sd][dj < 0 ? -dj : 0];
            }
            if (j2 == j && j != 1) {
                const int sd = j == 0 ? 3 : 2;
                val -= di >= 0 ? Rp[sd][di >= 0 ? di : 0] : Rn[sd][di < 0 ? -di : 0];
            }
            if (i2 == I && I != 1 && j2 == j && j != 1) val += Cq[(I == 0 ? 2 : 0) + (j == 0 ? 1 : 0)];
            if (lane < C) st[9 * lane + ij2] = val;
        }
        __builtin_amdgcn_wave_barrier();       // LDS serves a wavefront's accesses in order: the reads below see the row
        float *row = pr.F + (long)(9 * c + 3 * I + j) * dF;
#pragma unroll
        for (int k = 0; k < 9; ++k)
            if (lane + 64 * k < d) row[lane + 64 * k] = decay * old[j][k] + wnew * st[lane + 64 * k];
        if (pr.has_bias && lane == 0) row[d] = oldb[j];
        __builtin_amdgcn_wave_barrier();
    }
}

__global__ __launch_bounds__(256) void corr3_assemble_kernel(const CorrTable tab)
{
    __shared__ float strip[C3_ARW][9 * 64 + 4];
    const CorrProb &pr = tab.p[corr_locate(tab, blockIdx.x)];
    const int C = pr.C, d = 9 * C, dF = d + pr.has_bias;
    const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int rt = C3_ARW * (blockIdx.x - pr.blk_start) + w;         // row triple: the same for the whole wavefront
    const int c = rt / 3, i = rt - 3 * c;
    if (c > C || (c == C && (i > 0 || !pr.has_bias))) return;
    if (c == C) {
        const float *Ts = pr.Fs + (long)C3_LAGS * C * C, *Bv = pr.Bs + (long)C3_BQ * C * C;
        const float wnew = (1.0f - pr.decay) * pr.scale;
        float *row = pr.F + (long)d * dF;
        for (int x = lane; x < dF; x += 64) {
            float val;
            if (x == d) {
                val = (float)((long)pr.B * pr.H * pr.W);
            } else {
                const int cc = x / 9, ij = x - 9 * cc, ii = ij / 3, jj = ij - 3 * ii;
                val = Ts[cc];
                if (ii != 1) val -= Bv[(ii == 0 ? 1 : 0) * C + cc];
                if (jj != 1) val -= Bv[(jj == 0 ? 3 : 2) * C + cc];
                if (ii != 1 && jj != 1) val += Bv[(4 + (ii == 0 ? 2 : 0) + (jj == 0 ? 1 : 0)) * C + cc];
            }
            row[x] = pr.decay * row[x] + wnew * val;
        }
        return;
    }
    if (i == 0) corr3_assemble_rows<0>(pr, c, lane, strip[w]);
    else if (i == 1) corr3_assemble_rows<1>(pr, c, lane, strip[w]);
    else corr3_assemble_rows<2>(pr, c, lane, strip[w]);
}

}  // namespace kfac

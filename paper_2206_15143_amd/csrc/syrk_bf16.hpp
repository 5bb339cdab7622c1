// X^T X partial products for row-major bf16 X (bf16 patch matrices, token rows
// of linear layers) on the bf16 MFMA units: v_mfma_f32_32x32x16_bf16, products
// exact in fp32, fp32 accumulation (Eq. 4 of the DP-KFAC paper with bf16
// inputs; the factors themselves stay fp32).
//
// A workgroup of eight wavefronts owns a 256 x 256 block tile of the lower
// triangle; wave (wm, wn) owns 128 x 64 of it (4 x 2 MFMA tiles, 128
// accumulator registers).  K is walked in stages of 32 rows.  A stage is two
// panels [32 rows][256 columns] of bf16 copied from global memory straight into
// LDS by buffer_load_dwordx4 ... lds (no staging registers, three-stage ring,
// two stages in flight); rows past K and columns past the row length arrive as
// zeros through the buffer range check.
//
// The MFMA wants, per lane, eight consecutive k of one column, while the panel
// is stored as it lies in memory (k-major).  ds_read_b64_tr_b16 does that
// transposition on the way out of LDS: within 16 lanes, lane 4e+q supplies the
// address of four consecutive columns of row e, and lane i receives rows 0..3 of
// column i.  The row pitch is 288 elements (= 16 banks mod 64), so the four rows
// and two column halves a half-wave touches fall on disjoint banks.
//
// NCHW operands (1x1 convolution inputs, output gradients of every
// convolution) are k-contiguous already: their panels are staged [column][32 k]
// (pitch 80 bytes, conflict-free for 16-byte reads) and a lane's operand is one
// ds_read_b128.  A K stage never crosses an image; the k positions past the
// end of an image in its last stage are cleared in the A operand registers (the
// matching B values are finite neighbours and are multiplied by zero).
//
// On diagonal blocks the two waves whose tile lies wholly above the diagonal
// compute the column sums of the block (the bias border of A) as a product
// with a vector of ones instead of idling.
#pragma once

#include "syrk_wave.hpp"

namespace kfac {

constexpr int H_BM = 256;                    // block tile
constexpr int H_KT = 32;                     // rows per stage
constexpr int H_PITCH_B = 576;               // LDS row pitch in bytes (256 + 32 pad elements)
constexpr int H_SEGS = 36;                   // 16-byte pieces per LDS row (32 data + 4 pad)
constexpr int H_PANEL_B = H_KT * H_PITCH_B;  // 18432
constexpr int H_STAGE_B = 2 * H_PANEL_B;     // 36864
constexpr int H_NSTAGE = 3;
constexpr int H_PIECES = 2 * H_KT * H_SEGS;  // 2304 16-byte pieces per stage = 36 wave instructions
constexpr int H_LOADS = 5;                   // DMA instructions per wave and stage (8 waves x 5 = 40 >= 36)
constexpr int H_LDS_BYTES = H_NSTAGE * H_STAGE_B + 1024;
// NCHW staging: [256 columns][32 k] with an 80-byte column pitch, five 16-byte pieces per column
constexpr int HN_PITCH_B = 80;
constexpr int HN_PANEL_B = H_BM * HN_PITCH_B;   // 20480
constexpr int HN_STAGE_B = 2 * HN_PANEL_B;      // 40960 = 40 wave instructions
constexpr int HN_LDS_BYTES = H_NSTAGE * HN_STAGE_B + 1024;

typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ bf16x8 tr_frag(const unsigned char *lds, int byte)
{
    // rows k..k+3 and k+4..k+7 of the lane's column: two transposing reads
    const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) short4v *)(lds + byte));
    const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) short4v *)(lds + byte + 4 * H_PITCH_B));
    const short8v v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

__device__ __forceinline__ bf16x8 nchw_frag(const unsigned char *lds, int byte)
{
    const short8v v = *reinterpret_cast<const short8v *>(lds + byte);
    return __builtin_bit_cast(bf16x8, v);
}

// clears elements e >= nv of an operand fragment (nv may be <= 0 or >= 8)
__device__ __forceinline__ bf16x8 keep_first(bf16x8 x, int nv)
{
    typedef unsigned uint4v __attribute__((ext_vector_type(4)));
    uint4v u = __builtin_bit_cast(uint4v, x);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const unsigned m = (nv >= 2 * q + 2) ? 0xffffffffu : (nv == 2 * q + 1 ? 0x0000ffffu : 0u);
        u[q] &= m;
    }
    return __builtin_bit_cast(bf16x8, u);
}

struct HalfCtx {
    int4v rsrc;
    unsigned vo[H_LOADS];       // per-lane global byte offsets of this wave's pieces (W_OOB = none)
    unsigned dst[H_LOADS];      // LDS byte offset of each instruction inside a stage (or the landing zone)
    unsigned lds_base;
    unsigned tile_bytes;        // kRows: global bytes per K stage
    int nstages;
    // kNCHW: stage -> (image, k tile inside the image)
    int tpi, hw;                // K tiles per image, positions per image
    unsigned img_bytes;         // bytes from one image to the next
    int img0, kt0;              // image / tile of the split's first stage
};

// so: global byte offset of the stage (uniform)
template <int LAYOUT>
__device__ __forceinline__ void half_issue(const HalfCtx &c, int g, unsigned so_live)
{
    constexpr int STAGE_B = (LAYOUT == kRows) ? H_STAGE_B : HN_STAGE_B;
    const bool live = g < c.nstages;
    const unsigned buf = c.lds_base + (unsigned)((g % H_NSTAGE) * STAGE_B);
    const unsigned dummy = c.lds_base + (unsigned)(H_NSTAGE * STAGE_B);
    const unsigned so = live ? so_live : 0u;
#pragma unroll
    for (int i = 0; i < H_LOADS; ++i) {
        const bool piece = c.dst[i] != 0xffffffffu;
        dma16(piece ? buf + c.dst[i] : dummy, (live && piece) ? c.vo[i] : W_OOB, c.rsrc, so);
    }
}

// at most the loads of the stage issued last are still outstanding, then meet the other waves
__device__ __forceinline__ void half_sync()
{
    asm volatile("s_waitcnt vmcnt(5)\n\ts_barrier" ::: "memory");
}

enum HalfKind : int { kHFull = 0, kHOnes = 1, kHIdle = 2 };

// Walks the stages of a split: global byte offset of each stage and, for NCHW, the number of valid
// k positions in it.
template <int LAYOUT>
struct StageWalk {
    unsigned so;
    int img, kt, rem;
    __device__ __forceinline__ void start(const HalfCtx &c)
    {
        if (LAYOUT == kRows) { so = 0; rem = H_KT; }
        else { img = c.img0; kt = c.kt0; so = (unsigned)img * c.img_bytes + (unsigned)(kt * H_KT * 2); rem = c.hw - kt * H_KT; }
    }
    __device__ __forceinline__ void next(const HalfCtx &c)
    {
        if (LAYOUT == kRows) { so += c.tile_bytes; }
        else {
            ++kt;
            if (kt == c.tpi) { kt = 0; ++img; }
            so = (unsigned)img * c.img_bytes + (unsigned)(kt * H_KT * 2);
            rem = c.hw - kt * H_KT;
        }
    }
};

// The K loop of one wave.  KIND is uniform over a wavefront, so the MFMA chain is straight-line code.
template <int LAYOUT, int KIND>
__device__ __forceinline__ void half_loop(const HalfCtx &c, const unsigned char *lds, int a_byte, int b_byte,
                                          int lg, floatx16 (&acc)[8])
{
    constexpr int STAGE_B = (LAYOUT == kRows) ? H_STAGE_B : HN_STAGE_B;
    constexpr int JSTEP = (LAYOUT == kRows) ? 16 * H_PITCH_B : 32;      // bytes from one k16 step to the next
    constexpr int TSTEP = (LAYOUT == kRows) ? 64 : 32 * HN_PITCH_B;     // bytes from one 32-column tile to the next
    StageWalk<LAYOUT> wi, wc;     // stage being issued / stage being multiplied
    wi.start(c);
    wc.start(c);
    half_issue<LAYOUT>(c, 0, wi.so);
    wi.next(c);
    half_issue<LAYOUT>(c, 1, wi.so);
    wi.next(c);
    asm volatile("s_waitcnt vmcnt(5)\n\ts_barrier" ::: "memory");
    bf16x8 ones;
#pragma unroll
    for (int e = 0; e < 8; ++e) ones[e] = (__bf16)1.0f;
    for (int g = 0; g < c.nstages; ++g) {
        half_issue<LAYOUT>(c, g + 2, wi.so);
        wi.next(c);
        const unsigned char *buf = lds + (g % H_NSTAGE) * STAGE_B;
        const bool tail = (LAYOUT == kNCHW) && wc.rem < H_KT;
        if (KIND == kHFull) {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                bf16x8 a[4], b[2];
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    a[t] = (LAYOUT == kRows) ? tr_frag(buf, a_byte + j * JSTEP + t * TSTEP)
                                             : nchw_frag(buf, a_byte + j * JSTEP + t * TSTEP);
#pragma unroll
                for (int t = 0; t < 2; ++t)
                    b[t] = (LAYOUT == kRows) ? tr_frag(buf, b_byte + j * JSTEP + t * TSTEP)
                                             : nchw_frag(buf, b_byte + j * JSTEP + t * TSTEP);
                if (tail) {
                    const int nv = wc.rem - 16 * j - 8 * lg;
#pragma unroll
                    for (int t = 0; t < 4; ++t) a[t] = keep_first(a[t], nv);
                }
#pragma unroll
                for (int ti = 0; ti < 4; ++ti)
#pragma unroll
                    for (int tj = 0; tj < 2; ++tj)
                        acc[ti * 2 + tj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ti], b[tj], acc[ti * 2 + tj], 0, 0, 0);
            }
        } else if (KIND == kHOnes) {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                bf16x8 b[4];
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    b[t] = (LAYOUT == kRows) ? tr_frag(buf, b_byte + j * JSTEP + t * TSTEP)
                                             : nchw_frag(buf, b_byte + j * JSTEP + t * TSTEP);
                const bf16x8 o = tail ? keep_first(ones, wc.rem - 16 * j - 8 * lg) : ones;
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(o, b[t], acc[t], 0, 0, 0);
            }
        }
        wc.next(c);
        half_sync();
    }
    // the padding loads of the stages past the end may still be landing
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
}

template <int LAYOUT>
__global__ __launch_bounds__(512) void syrk_bf16_kernel(const SyrkTable tab)
{
    __shared__ __attribute__((aligned(16))) unsigned char lds[LAYOUT == kRows ? H_LDS_BYTES : HN_LDS_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = w >> 2, wn = w & 3;

    const int bid = xcd_block_id();
    int pi = 0;
    while (pi + 1 < tab.count && bid >= tab.p[pi + 1].blk_start) ++pi;
    const SyrkProb &pr = tab.p[pi];
    const int local = bid - pr.blk_start;
    const int nblk = pr.nb * (pr.nb + 1) / 2;
    const int split = local / nblk;
    const int blk = local - split * nblk;
    int bi, bj;
    tri_decode(blk, bi, bj);
    const bool diag = (bi == bj);

    // ---- K range of this split, buffer resource, per-lane piece offsets ----
    HalfCtx c;
    c.lds_base = (unsigned)(unsigned long)(__attribute__((address_space(3))) unsigned char *)lds;
    const long t0 = (long)split * pr.tiles_per_split;
    const int ld = (int)pr.ld;
    if (LAYOUT == kRows) {
        const long ktiles = (pr.K + H_KT - 1) / H_KT;
        const long t1 = (t0 + pr.tiles_per_split < ktiles) ? t0 + pr.tiles_per_split : ktiles;
        const long row0 = t0 * H_KT;
        const unsigned short *base = reinterpret_cast<const unsigned short *>(pr.x) + row0 * pr.ld;
        const long bytes_left = (pr.K - row0) * pr.ld * 2;
        const unsigned long ba = (unsigned long)base;
        c.rsrc.x = (int)(unsigned)ba;
        c.rsrc.y = (int)(unsigned)(ba >> 32);
        c.rsrc.z = bytes_left > 0x7fffffffl ? 0x7fffffff : (int)bytes_left;
        c.rsrc.w = 0x00020000;
        c.nstages = (int)(t1 - t0);
        c.tile_bytes = (unsigned)(H_KT * ld * 2);
        c.tpi = 1; c.hw = 0; c.img_bytes = 0; c.img0 = 0; c.kt0 = 0;
#pragma unroll
        for (int i = 0; i < H_LOADS; ++i) {
            const int inst = i * 8 + w;                 // wave instruction index inside the stage
            const int p = inst * 64 + lane;             // 16-byte piece
            const int panel = p / (H_KT * H_SEGS);
            const int r = p - panel * (H_KT * H_SEGS);
            const int row = r / H_SEGS, seg = r - row * H_SEGS;
            const int col = (panel == 0 ? bi : bj) * H_BM + seg * 8;
            const bool inst_ok = inst * 64 < H_PIECES && !(diag && inst * 64 >= H_KT * H_SEGS);
            const bool ok = inst_ok && p < H_PIECES && seg < 32 && col < ld;
            c.vo[i] = ok ? (unsigned)((row * ld + col) * 2) : W_OOB;
            c.dst[i] = inst_ok ? (unsigned)(inst * 1024) : 0xffffffffu;
        }
    } else {
        // x is [images][ctot][hw]; the buffer covers the whole tensor (the host checked it is below 2 GiB)
        const int hw = pr.hw;
        const int nimg = (int)(pr.K / hw);
        c.tpi = (hw + H_KT - 1) / H_KT;
        c.hw = hw;
        c.img_bytes = (unsigned)pr.ctot * (unsigned)hw * 2u;
        const long ktiles = (long)nimg * c.tpi;
        const long t1 = (t0 + pr.tiles_per_split < ktiles) ? t0 + pr.tiles_per_split : ktiles;
        c.nstages = (int)(t1 - t0);
        c.img0 = (int)(t0 / c.tpi);
        c.kt0 = (int)(t0 - (long)c.img0 * c.tpi);
        c.tile_bytes = 0;
        const unsigned long ba = (unsigned long)pr.x;
        c.rsrc.x = (int)(unsigned)ba;
        c.rsrc.y = (int)(unsigned)(ba >> 32);
        c.rsrc.z = (int)((long)nimg * c.img_bytes);
        c.rsrc.w = 0x00020000;
#pragma unroll
        for (int i = 0; i < H_LOADS; ++i) {
            const int inst = i * 8 + w;                 // 40 instructions: 20 per panel
            const int p = inst * 64 + lane;
            const int panel = p / (H_BM * 5);
            const int r = p - panel * (H_BM * 5);
            const int cl = r / 5, seg = r - cl * 5;
            const int col = (panel == 0 ? bi : bj) * H_BM + cl;
            const bool inst_ok = !(diag && panel == 1);
            const bool ok = inst_ok && seg < 4 && col < pr.d;
            c.vo[i] = ok ? (unsigned)((col * hw + seg * 8) * 2) : W_OOB;
            c.dst[i] = inst_ok ? (unsigned)(inst * 1024) : 0xffffffffu;
        }
    }

    floatx16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;

    const int lr = lane & 31, lg = lane >> 5;
    int lane_byte, a_byte, b_byte, o_byte;
    if (LAYOUT == kRows) {
        // per-lane part of the transposing read address: row 8*kgroup + e, column 16*colhalf + 4*q
        const int s16 = lane & 15, gi = lane >> 4;
        lane_byte = (8 * (gi >> 1) + (s16 >> 2)) * H_PITCH_B + (16 * (gi & 1) + 4 * (s16 & 3)) * 2;
        a_byte = lane_byte + wm * 128 * 2;
        b_byte = (diag ? 0 : H_PANEL_B) + lane_byte + wn * 64 * 2;
        o_byte = lane_byte + (wn - 2) * 128 * 2;
    } else {
        lane_byte = lr * HN_PITCH_B + 16 * lg;
        a_byte = lane_byte + wm * 128 * HN_PITCH_B;
        b_byte = (diag ? 0 : HN_PANEL_B) + lane_byte + wn * 64 * HN_PITCH_B;
        o_byte = lane_byte + (wn - 2) * 128 * HN_PITCH_B;
    }

    // wave roles: on diagonal blocks the tiles of waves (0, 2) and (0, 3) lie above the diagonal
    const bool upper = diag && wm == 0 && wn >= 2;
    const bool ones_duty = upper && pr.has_bias;
    if (!upper) {
        half_loop<LAYOUT, kHFull>(c, lds, a_byte, b_byte, lg, acc);
    } else if (ones_duty) {
        half_loop<LAYOUT, kHOnes>(c, lds, 0, o_byte, lg, acc);
    } else {
        half_loop<LAYOUT, kHIdle>(c, lds, 0, 0, lg, acc);
    }

    if (!upper) {
        float *dst = pr.partial + ((long)split * nblk + blk) * (H_BM * H_BM);
#pragma unroll
        for (int ti = 0; ti < 4; ++ti)
#pragma unroll
            for (int tj = 0; tj < 2; ++tj) {
                const int col = wn * 64 + tj * 32 + lr;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = wm * 128 + ti * 32 + 8 * (v >> 2) + 4 * lg + (v & 3);
                    dst[row * H_BM + col] = acc[ti * 2 + tj][v];
                }
            }
    } else if (ones_duty && lg == 0) {
        // every row of a ones-product tile holds the column sums: row 0 (v = 0 of lanes 0..31)
        float *csum = pr.partial + (long)pr.splits * nblk * (H_BM * H_BM);
#pragma unroll
        for (int t = 0; t < 4; ++t)
            csum[((long)split * pr.nb + bi) * H_BM + (wn - 2) * 128 + t * 32 + lr] = acc[t][0];
    }
}

}  // namespace kfac

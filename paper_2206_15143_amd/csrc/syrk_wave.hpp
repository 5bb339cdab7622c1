// Second-generation partial-product kernel for X^T X on row-major fp32 X
// (patch matrices, linear-layer inputs): "one wavefront = one 45-tile unit".
//
// The lower triangle is cut into 144 x 144 macro tiles (9 x 9 MFMA tiles of
// v_mfma_f32_16x16x4_f32).  A wavefront owns one unit of at most 45 MFMA tiles
// and keeps all 45 accumulators (180 registers) for the whole K range:
//   DIAG(i)     : the 45 lower tiles of macro tile (i, i); one operand set (a == b),
//   HALF(i,j,h) : rows of macro i x column tiles [0,5) (h=0) or [5,9) (h=1) of macro j < i.
// A workgroup is four wavefronts that share the staged column panels:
//   D block, full  : DIAG(a), DIAG(a+1), HALF(a+1,a,0), HALF(a+1,a,1)      panels a, a+1
//   D block, single: DIAG(a) only (last macro of an odd count): the four waves
//                    split K (each takes one k-step of four) over three staged
//                    K tiles and add their accumulators through LDS at the end
//   R block        : HALF(i,j,0), HALF(i,j,1), HALF(i,j+1,0), HALF(i,j+1,1)  panels i, j, j+1
// Every unit does 36-45 MFMAs per 9-14 LDS operand reads, and the waves of a
// block carry equal work (within 10 %), unlike square block tiles whose
// diagonal blocks leave a third of the waves idle.
//
// Panels ([16 rows][144 columns], pitch 144 = 16 mod 32: conflict-free operand
// reads) are filled by buffer_load_dwordx4 ... lds: each wave instruction
// copies 1 KB straight from global memory into LDS, nine per panel, with no
// staging registers; rows past K and columns past the row length read as zero
// through the buffer range check.  A ring of four stage buffers keeps three
// stages of loads in flight behind the MFMAs of the current one (a single CU
// must have ~60 KB outstanding to pull its share of HBM bandwidth).
#pragma once

#include "syrk_types.hpp"
#include "wave_common.hpp"

namespace kfac {

struct WaveCtx {
    int4v rsrc;
    unsigned vo[W_SLOTS][3];   // per-lane byte offsets of the 1 KB pieces q = w, w+4, w+8 of each panel slot
    unsigned tile_bytes;
    unsigned lds_base;         // LDS byte address of the stage ring
    int nslots, ntl, nstages;
    int w, lane, tid;
    int rslot, cslot, ctile0;
    bool single, owns_colsum;
    bool no_mfma, no_load;   // measurement switches
};

// Issue the loads of stage g into ring buffer g % 4: exactly nine instructions per wave, whatever
// the block kind (missing panels, pieces past the ninth and stages past the end become all-out-of-range
// loads, which move no data), so the vmcnt arithmetic of wave_sync is the same everywhere.
__device__ __forceinline__ void wave_issue(const WaveCtx &c, int g)
{
    const unsigned buf = c.lds_base + (unsigned)((g & (W_NSTAGE - 1)) * W_STAGE * 4);
    const unsigned dummy = c.lds_base + (unsigned)(W_NSTAGE * W_STAGE * 4);
#pragma unroll
    for (int s = 0; s < W_SLOTS; ++s) {
        const int tl = c.single ? 3 * g + s : g;       // K tile (relative to the split) this slot holds
        const bool live = (s < c.nslots) && (g < c.nstages) && (tl < c.ntl) && !c.no_load;
        const unsigned so = live ? (unsigned)tl * c.tile_bytes : 0u;
#pragma unroll
        for (int qi = 0; qi < 3; ++qi) {
            const int q = c.w + 4 * qi;
            const bool piece = q < W_NT;
            const unsigned v = (live && piece) ? c.vo[s][qi] : W_OOB;
            const unsigned dst = piece ? buf + (unsigned)((s * W_PANEL + q * 256) * 4) : dummy;
            dma16(dst, v, c.rsrc, so);
        }
    }
}

// The whole K loop of one wave, specialised on the kind of unit it owns so that the loop body is
// straight-line MFMA code accumulating in place.  All four specialisations execute the same number
// of barriers (nstages is uniform over the workgroup).
template <int KIND>
__device__ __forceinline__ void wave_loop(const WaveCtx &c, const float *lds, floatx4 (&acc)[45], float &cs0,
                                          float &cs1)
{
    wave_issue(c, 0);
    wave_issue(c, 1);
    wave_issue(c, 2);
    wave_sync();
    for (int g = 0; g < c.nstages; ++g) {
        wave_issue(c, g + 3);
        const float *buf = lds + (g & (W_NSTAGE - 1)) * W_STAGE;
        if (c.no_mfma) {
            // measurement only
        } else if (KIND == kSingle) {
            // wave w multiplies rows 4w..4w+3 of each of the three staged K tiles
#pragma unroll
            for (int st = 0; st < 3; ++st) unit_diag(buf + st * W_PANEL, 4 * c.w, c.lane, acc);
        } else if (KIND == kDiag) {
            const float *P = buf + c.rslot * W_PANEL;
#pragma unroll
            for (int st = 0; st < 4; ++st) unit_diag(P, 4 * st, c.lane, acc);
        } else {
            const float *Pr = buf + c.rslot * W_PANEL;
            const float *Pc = buf + c.cslot * W_PANEL + c.ctile0 * 16;
#pragma unroll
            for (int st = 0; st < 4; ++st) unit_half<KIND == kHalf5 ? 5 : 4>(Pr, Pc, 4 * st, c.lane, acc);
        }
        if (c.owns_colsum && c.tid < W_MT) {
            // column sums of the staged rows (rows past K are zero)
            const float *c0 = buf + c.tid;
            float s0 = 0.f, s1 = 0.f;
#pragma unroll
            for (int k = 0; k < W_KT; ++k) s0 += c0[k * W_MT];
#pragma unroll
            for (int k = 0; k < W_KT; ++k) s1 += c0[W_PANEL + k * W_MT];
            if (KIND == kSingle) {
                float s2 = 0.f;
#pragma unroll
                for (int k = 0; k < W_KT; ++k) s2 += c0[2 * W_PANEL + k * W_MT];
                cs0 += (s0 + s1) + s2;
            } else {
                cs0 += s0;
                cs1 += s1;
            }
        }
        wave_sync();
    }
    // the padding loads of the stages past the end may still be landing in the ring
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
}

// Which macro tiles the panels of a block hold and which unit each of its four waves owns.
struct BlockRole {
    int mac0, mac1, mac2;     // macro index per panel slot
    int nslots;
    bool single, owns_colsum;
    int kind;                 // WaveKind of this wave
    int rslot, cslot, ctile0; // panel slots of the row / column operand, first column tile
    int I, J;                 // macro tile this wave writes
};

__device__ __forceinline__ BlockRole decode_role(int m, int b, int w, bool has_bias)
{
    BlockRole r;
    r.mac0 = r.mac1 = r.mac2 = 0;
    r.single = false;
    r.owns_colsum = false;
    const int nds = (m + 1) / 2;
    if (b < nds) {
        const int a = 2 * b;
        r.owns_colsum = has_bias;
        if (a + 1 < m) {
            r.nslots = 2; r.mac0 = a; r.mac1 = a + 1;
            if (w == 0)      { r.kind = kDiag;  r.rslot = 0; r.cslot = 0; r.ctile0 = 0; r.I = a;     r.J = a; }
            else if (w == 1) { r.kind = kDiag;  r.rslot = 1; r.cslot = 1; r.ctile0 = 0; r.I = a + 1; r.J = a + 1; }
            else if (w == 2) { r.kind = kHalf5; r.rslot = 1; r.cslot = 0; r.ctile0 = 0; r.I = a + 1; r.J = a; }
            else             { r.kind = kHalf4; r.rslot = 1; r.cslot = 0; r.ctile0 = 5; r.I = a + 1; r.J = a; }
        } else {
            r.single = true;
            r.nslots = 3; r.mac0 = r.mac1 = r.mac2 = a;
            r.kind = kSingle; r.rslot = 0; r.cslot = 0; r.ctile0 = 0; r.I = a; r.J = a;
        }
    } else {
        int q = b - nds, i = 2;
        while (q >= i / 2) { q -= i / 2; ++i; }
        const int j = 2 * q;
        r.nslots = 3; r.mac0 = i; r.mac1 = j; r.mac2 = j + 1;
        r.rslot = 0; r.I = i;
        if (w == 0)      { r.kind = kHalf5; r.cslot = 1; r.ctile0 = 0; r.J = j; }
        else if (w == 1) { r.kind = kHalf4; r.cslot = 1; r.ctile0 = 5; r.J = j; }
        else if (w == 2) { r.kind = kHalf5; r.cslot = 2; r.ctile0 = 0; r.J = j + 1; }
        else             { r.kind = kHalf4; r.cslot = 2; r.ctile0 = 5; r.J = j + 1; }
    }
    return r;
}

// After the K loop: single blocks add the four waves' accumulators through LDS (fixed order
// w1, w2, w3), then every unit stores its partial tiles and the block its column sums.
// xch: at least 45*4*64 floats of LDS no load is in flight to.
__device__ __forceinline__ void wave_epilogue(const SyrkProb &pr, const BlockRole &r, int split, int w, int lane,
                                              int tid, int nrt, float *xch, floatx4 (&acc)[45], float cs0, float cs1)
{
    const int m = pr.nb;
    const int nblk = m * (m + 1) / 2;
    if (r.single) {
        for (int q = 1; q < 4; ++q) {
            __syncthreads();
            if (w == q) {
#pragma unroll
                for (int i = 0; i < 45; ++i)
#pragma unroll
                    for (int v = 0; v < 4; ++v) xch[(i * 4 + v) * 64 + lane] = acc[i][v];
            }
            __syncthreads();
            if (w == 0) {
#pragma unroll
                for (int i = 0; i < 45; ++i)
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc[i][v] += xch[(i * 4 + v) * 64 + lane];
            }
        }
    }
    if (!r.single || w == 0) {
        // tiles go out as they lie in the accumulators: 16 bytes per lane, 1 KB per tile, fully coalesced
        float *dst = pr.partial + ((long)split * nblk + (r.I * (r.I + 1) / 2 + r.J)) * (W_MT * W_MT);
        floatx4 *dst4 = reinterpret_cast<floatx4 *>(dst) + lane;
        if (r.kind == kSingle || r.kind == kDiag) {
#pragma unroll
            for (int ti = 0; ti < W_NT; ++ti) {
                if (ti < nrt) {
#pragma unroll
                    for (int tj = 0; tj <= ti; ++tj) dst4[(ti * W_NT + tj) * 64] = acc[ti * (ti + 1) / 2 + tj];
                }
            }
        } else {
            const int nc = (r.kind == kHalf5) ? 5 : 4;
#pragma unroll
            for (int ti = 0; ti < W_NT; ++ti) {
                if (ti < nrt) {
#pragma unroll
                    for (int tj = 0; tj < 5; ++tj) {
                        if (tj < nc) dst4[(ti * W_NT + r.ctile0 + tj) * 64] = acc[ti * 5 + tj];
                    }
                }
            }
        }
    }
    if (r.owns_colsum && tid < W_MT) {
        float *csum = pr.partial + (long)pr.splits * nblk * (W_MT * W_MT);
        csum[((long)split * m + r.mac0) * W_MT + tid] = cs0;
        if (!r.single) csum[((long)split * m + r.mac1) * W_MT + tid] = cs1;
    }
}

__global__ __launch_bounds__(256) void syrk_wave_kernel(const SyrkTable tab)
{
    __shared__ float lds[W_LDS_FLOATS];

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
    const int ntiles_last = (pr.d - (m - 1) * W_MT + 15) / 16;   // valid MFMA tiles of the last macro

    const BlockRole r = decode_role(m, b, w, pr.has_bias != 0);
    WaveCtx c;
    c.single = r.single; c.owns_colsum = r.owns_colsum; c.nslots = r.nslots;
    c.rslot = r.rslot; c.cslot = r.cslot; c.ctile0 = r.ctile0;
    const int nrt = (r.I == m - 1) ? ntiles_last : W_NT;   // valid row tiles of macro I (only the stores look at it)

    // ---- K range of this split, buffer resource over it ----
    const long ktiles = (pr.K + W_KT - 1) / W_KT;
    const long t0 = (long)split * pr.tiles_per_split;
    const long t1 = (t0 + pr.tiles_per_split < ktiles) ? t0 + pr.tiles_per_split : ktiles;
    c.ntl = (int)(t1 - t0);
    const long row0 = t0 * W_KT;
    const float *base = reinterpret_cast<const float *>(pr.x) + row0 * pr.ld;
    const long bytes_left = (pr.K - row0) * pr.ld * 4;
    const int nrec = bytes_left > 0x7fffffffl ? 0x7fffffff : (int)bytes_left;
    {   // raw buffer resource over the rows of this split: base, stride 0, byte count, dword format
        const unsigned long ba = (unsigned long)base;
        c.rsrc.x = (int)(unsigned)ba;
        c.rsrc.y = (int)(unsigned)(ba >> 32);
        c.rsrc.z = nrec;
        c.rsrc.w = 0x00020000;
    }
    c.lds_base = (unsigned)(unsigned long)(__attribute__((address_space(3))) float *)lds;
    c.w = w; c.lane = lane; c.tid = tid;
    c.no_mfma = (tab.debug & 1) != 0;
    c.no_load = (tab.debug & 2) != 0;
    const int ld = (int)pr.ld;
#pragma unroll
    for (int qi = 0; qi < 3; ++qi) {
        const int q = w + 4 * qi;
        const int f = 256 * q + 4 * lane;
        const int k = f / W_MT;
        const int col = f - k * W_MT;
        const bool qok = q < W_NT;
        const int g0 = r.mac0 * W_MT + col, g1 = r.mac1 * W_MT + col, g2 = r.mac2 * W_MT + col;
        c.vo[0][qi] = (qok && g0 < ld) ? (unsigned)((k * ld + g0) * 4) : W_OOB;
        c.vo[1][qi] = (qok && g1 < ld) ? (unsigned)((k * ld + g1) * 4) : W_OOB;
        c.vo[2][qi] = (qok && g2 < ld) ? (unsigned)((k * ld + g2) * 4) : W_OOB;
    }
    c.tile_bytes = (unsigned)(W_KT * ld * 4);
    c.nstages = (c.ntl + (c.single ? 3 : 1) - 1) / (c.single ? 3 : 1);

    floatx4 acc[45];
#pragma unroll
    for (int i = 0; i < 45; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
    float cs0 = 0.f, cs1 = 0.f;

    if (r.kind == kSingle)     wave_loop<kSingle>(c, lds, acc, cs0, cs1);
    else if (r.kind == kDiag)  wave_loop<kDiag>(c, lds, acc, cs0, cs1);
    else if (r.kind == kHalf5) wave_loop<kHalf5>(c, lds, acc, cs0, cs1);
    else                       wave_loop<kHalf4>(c, lds, acc, cs0, cs1);

    wave_epilogue(pr, r, split, w, lane, tid, nrt, lds, acc, cs0, cs1);
}

// ---------------------------------------------------------------------------------------------
// NCHW fp32 operands (inputs of 1x1 convolutions, output gradients of convolutions with more than 64
// channels): X^T is stored [image][channel][position], so a channel's K values are contiguous.  The
// panels are staged [144 channels][16 positions] with a pitch of 20 floats (16-byte pieces stay
// aligned, and the operand read "channel lr, position lk" of 64 lanes spreads two lanes per bank);
// a K stage never crosses an image, and the positions past the end of an image in its last stage
// are cleared in the operand registers.  Units, roles, ring and epilogue are those of the row-major
// kernel above.
constexpr int WN_PITCH = 20;
constexpr int WN_PANEL = 12 * 256;                       // floats per panel slot: 12 DMA instructions of 1 KB
constexpr int WN_STAGE = W_SLOTS * WN_PANEL;
constexpr int WN_LDS_FLOATS = W_NSTAGE * WN_STAGE + 256;

// one k-step of a DIAG unit; nv = valid positions left in this stage's K tile
__device__ __forceinline__ void unit_diag_nchw(const float *P, int kk, int lane, int nv, floatx4 (&acc)[45])
{
    const int lr = lane & 15, lk = lane >> 4;
    const float *src = P + lr * WN_PITCH + kk + lk;
    const bool ok = kk + lk < nv;
    float a[W_NT];
#pragma unroll
    for (int t = 0; t < W_NT; ++t) {
        const float v = src[t * 16 * WN_PITCH];
        a[t] = ok ? v : 0.f;
    }
#pragma unroll
    for (int ti = 0; ti < W_NT; ++ti)
#pragma unroll
        for (int tj = 0; tj <= ti; ++tj)
            acc[ti * (ti + 1) / 2 + tj] =
                __builtin_amdgcn_mfma_f32_16x16x4f32(a[ti], a[tj], acc[ti * (ti + 1) / 2 + tj], 0, 0, 0);
}

template <int NC>
__device__ __forceinline__ void unit_half_nchw(const float *Pr, const float *Pc, int kk, int lane, int nv,
                                               floatx4 (&acc)[45])
{
    const int lr = lane & 15, lk = lane >> 4;
    const float *sr = Pr + lr * WN_PITCH + kk + lk;
    const float *sc = Pc + lr * WN_PITCH + kk + lk;      // Pc already points at the first column tile
    const bool ok = kk + lk < nv;
    float a[W_NT], b[NC];
#pragma unroll
    for (int t = 0; t < W_NT; ++t) {
        const float v = sr[t * 16 * WN_PITCH];
        a[t] = ok ? v : 0.f;                             // clearing one operand is enough
    }
#pragma unroll
    for (int t = 0; t < NC; ++t) b[t] = sc[t * 16 * WN_PITCH];
#pragma unroll
    for (int ti = 0; ti < W_NT; ++ti)
#pragma unroll
        for (int tj = 0; tj < NC; ++tj)
            acc[ti * 5 + tj] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[ti], b[tj], acc[ti * 5 + tj], 0, 0, 0);
}

struct WaveNCtx {
    int4v rsrc;
    unsigned vo[W_SLOTS][3];
    unsigned lds_base;
    unsigned img_bytes;          // bytes from one image to the next
    int tpi, hw;                 // K tiles per image, positions per image
    int img, kt;                 // (image, tile) of the next K tile to be issued
    int nslots, ntl, nstages;
    int w, lane, tid;
    int rslot, cslot, ctile0;
    bool single, owns_colsum;
};

// Issue the loads of ring step g (always nine instructions per wave).  K tiles are issued in order,
// so the (image, tile) walk advances by one per live slot of a single block, by one per step otherwise.
__device__ __forceinline__ void waven_issue(WaveNCtx &c, int g)
{
    const unsigned buf = c.lds_base + (unsigned)((g & (W_NSTAGE - 1)) * WN_STAGE * 4);
    const unsigned dummy = c.lds_base + (unsigned)(W_NSTAGE * WN_STAGE * 4);
#pragma unroll
    for (int s = 0; s < W_SLOTS; ++s) {
        const int tl = c.single ? 3 * g + s : g;
        const bool live = (s < c.nslots) && (g < c.nstages) && (tl < c.ntl);
        const unsigned so = live ? (unsigned)c.img * c.img_bytes + (unsigned)(c.kt * W_KT * 4) : 0u;
#pragma unroll
        for (int qi = 0; qi < 3; ++qi) {
            const int q = c.w + 4 * qi;                  // 12 instructions per panel: all of them carry pieces
            const unsigned v = live ? c.vo[s][qi] : W_OOB;
            dma16(buf + (unsigned)((s * WN_PANEL + q * 256) * 4), v, c.rsrc, so);
        }
        const bool adv = c.single ? live : (s == W_SLOTS - 1 && g < c.nstages);
        if (adv) {
            if (++c.kt == c.tpi) { c.kt = 0; ++c.img; }
        }
    }
    (void)dummy;
}

template <int KIND>
__device__ __forceinline__ void waven_loop(WaveNCtx &c, const float *lds, int img0, int kt0, floatx4 (&acc)[45],
                                           float &cs0, float &cs1)
{
    waven_issue(c, 0);
    waven_issue(c, 1);
    waven_issue(c, 2);
    wave_sync();
    // (image, tile) of the K tile being multiplied: only the tile index matters (valid positions)
    int kt = kt0;
    auto rem_and_next = [&]() {
        const int nv = c.hw - kt * W_KT;
        if (++kt == c.tpi) kt = 0;
        return nv;
    };
    (void)img0;
    for (int g = 0; g < c.nstages; ++g) {
        waven_issue(c, g + 3);
        const float *buf = lds + (g & (W_NSTAGE - 1)) * WN_STAGE;
        int nvs[3];
        if (KIND == kSingle) {
#pragma unroll
            for (int st = 0; st < 3; ++st) nvs[st] = (3 * g + st < c.ntl) ? rem_and_next() : 0;
#pragma unroll
            for (int st = 0; st < 3; ++st) unit_diag_nchw(buf + st * WN_PANEL, 4 * c.w, c.lane, nvs[st], acc);
        } else {
            nvs[0] = rem_and_next();
            nvs[1] = nvs[2] = nvs[0];
            if (KIND == kDiag) {
                const float *P = buf + c.rslot * WN_PANEL;
#pragma unroll
                for (int st = 0; st < 4; ++st) unit_diag_nchw(P, 4 * st, c.lane, nvs[0], acc);
            } else {
                const float *Pr = buf + c.rslot * WN_PANEL;
                const float *Pc = buf + c.cslot * WN_PANEL + c.ctile0 * 16 * WN_PITCH;
#pragma unroll
                for (int st = 0; st < 4; ++st)
                    unit_half_nchw<KIND == kHalf5 ? 5 : 4>(Pr, Pc, 4 * st, c.lane, nvs[0], acc);
            }
        }
        if (c.owns_colsum && c.tid < W_MT) {
            // column sums of the staged positions (positions past the image end are not counted)
            const float *c0 = buf + c.tid * WN_PITCH;
            auto sum16 = [&](const float *p, int nv) {
                float s = 0.f;
#pragma unroll
                for (int k = 0; k < W_KT; ++k) s += (k < nv) ? p[k] : 0.f;
                return s;
            };
            if (KIND == kSingle) {
                cs0 += (sum16(c0, nvs[0]) + sum16(c0 + WN_PANEL, nvs[1])) + sum16(c0 + 2 * WN_PANEL, nvs[2]);
            } else {
                cs0 += sum16(c0, nvs[0]);
                cs1 += sum16(c0 + WN_PANEL, nvs[0]);
            }
        }
        wave_sync();
    }
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
}

__global__ __launch_bounds__(256) void syrk_wave_nchw_kernel(const SyrkTable tab)
{
    __shared__ float lds[WN_LDS_FLOATS];

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
    const int ntiles_last = (pr.d - (m - 1) * W_MT + 15) / 16;

    const BlockRole r = decode_role(m, b, w, pr.has_bias != 0);
    WaveNCtx c;
    c.single = r.single; c.owns_colsum = r.owns_colsum; c.nslots = r.nslots;
    c.rslot = r.rslot; c.cslot = r.cslot; c.ctile0 = r.ctile0;
    const int nrt = (r.I == m - 1) ? ntiles_last : W_NT;

    const int hw = pr.hw;
    const long nimg = pr.K / hw;
    c.hw = hw;
    c.tpi = (hw + W_KT - 1) / W_KT;
    c.img_bytes = (unsigned)pr.ctot * (unsigned)hw * 4u;
    const long ktiles = nimg * c.tpi;
    const long t0 = (long)split * pr.tiles_per_split;
    const long t1 = (t0 + pr.tiles_per_split < ktiles) ? t0 + pr.tiles_per_split : ktiles;
    c.ntl = (int)(t1 - t0);
    c.img = (int)(t0 / c.tpi);
    c.kt = (int)(t0 - (long)c.img * c.tpi);
    const int img0 = c.img, kt0 = c.kt;
    {   // the buffer covers the whole tensor (below 2 GiB, checked on the host)
        const unsigned long ba = (unsigned long)pr.x;
        c.rsrc.x = (int)(unsigned)ba;
        c.rsrc.y = (int)(unsigned)(ba >> 32);
        c.rsrc.z = (int)(nimg * (long)c.img_bytes);
        c.rsrc.w = 0x00020000;
    }
    c.lds_base = (unsigned)(unsigned long)(__attribute__((address_space(3))) float *)lds;
    c.w = w; c.lane = lane; c.tid = tid;
#pragma unroll
    for (int qi = 0; qi < 3; ++qi) {
        const int q = w + 4 * qi;
        const int p = q * 64 + lane;                 // 16-byte piece: channel p / 5, positions 4*(p % 5)..+3
        const int ch = p / 5, kq = p - ch * 5;
        const bool pok = ch < W_MT && kq < 4;
        const int g0 = r.mac0 * W_MT + ch, g1 = r.mac1 * W_MT + ch, g2 = r.mac2 * W_MT + ch;
        c.vo[0][qi] = (pok && g0 < pr.d) ? (unsigned)((g0 * hw + kq * 4) * 4) : W_OOB;
        c.vo[1][qi] = (pok && g1 < pr.d) ? (unsigned)((g1 * hw + kq * 4) * 4) : W_OOB;
        c.vo[2][qi] = (pok && g2 < pr.d) ? (unsigned)((g2 * hw + kq * 4) * 4) : W_OOB;
    }
    c.nstages = (c.ntl + (c.single ? 3 : 1) - 1) / (c.single ? 3 : 1);

    floatx4 acc[45];
#pragma unroll
    for (int i = 0; i < 45; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
    float cs0 = 0.f, cs1 = 0.f;

    if (r.kind == kSingle)     waven_loop<kSingle>(c, lds, img0, kt0, acc, cs0, cs1);
    else if (r.kind == kDiag)  waven_loop<kDiag>(c, lds, img0, kt0, acc, cs0, cs1);
    else if (r.kind == kHalf5) waven_loop<kHalf5>(c, lds, img0, kt0, acc, cs0, cs1);
    else                       waven_loop<kHalf4>(c, lds, img0, kt0, acc, cs0, cs1);

    wave_epilogue(pr, r, split, w, lane, tid, nrt, lds, acc, cs0, cs1);
}

}  // namespace kfac

// fp32 MFMA tile engine for products of the form  C = U^T V  where both
// operands are stored K-major (element (k, column)) or NCHW-like.
//
// A workgroup of NW x NW wavefronts owns a BM x BM output tile; each wavefront
// owns a (16*WT) x (16*WT) sub-tile made of WT x WT v_mfma_f32_16x16x4_f32
// accumulators.  K is walked in stages of KT = 16 rows that are staged through
// LDS (double buffered, one barrier per stage).
//
// Operand mapping of v_mfma_f32_16x16x4_f32 (lane l, lr = l & 15, lk = l >> 4):
//   A operand: A[i = lr][k = lk]      B operand: B[k = lk][j = lr]
//   D[v] (v = 0..3):  D[i = 4*lk + v][j = lr]
// For C = U^T V both operands are "row k of the staged panel, 16 consecutive
// columns", so with the LDS layout [k][column] every operand read is 16
// consecutive floats per k: conflict free when the row pitch is 16 mod 32.
#pragma once

#include "common.hpp"

namespace kfac {

template <int WT_, int NW_>
struct Tile {
    static constexpr int WT = WT_;
    static constexpr int NW = NW_;
    static constexpr int BM = WT_ * 16 * NW_;
    static constexpr int NT = NW_ * NW_ * 64;
    static constexpr int KT = 16;
    static constexpr int PITCH = (BM % 32 == 0) ? BM + 16 : BM;  // [k][col] layout, pitch = 16 (mod 32)
    static constexpr int PK = KT + 1;                            // [col][k] layout (NCHW operands)
    static constexpr int PANEL = (KT * PITCH > BM * PK) ? KT * PITCH : BM * PK;
    static constexpr int V4 = KT * BM / 4;                       // float4 slots per staged panel
    static constexpr int PASSES = (V4 + NT - 1) / NT;
};

struct Operand {
    const void *x;   // fp32 or bf16 elements (bf16 is widened to fp32 on load)
    long K;       // rows
    long ld;      // kRows: row pitch
    int d;        // valid columns
    int hw, ctot; // kNCHW addressing
    int vec;      // aligned 4-element loads allowed
};

// ---- global -> registers ---------------------------------------------------
template <int DT>
__device__ __forceinline__ float load1(const void *x, long off)
{
    if (DT == 0) return reinterpret_cast<const float *>(x)[off];
    return __uint_as_float((unsigned)reinterpret_cast<const unsigned short *>(x)[off] << 16);
}

template <int DT>
__device__ __forceinline__ floatx4 load4(const void *x, long off)
{
    if (DT == 0) return *reinterpret_cast<const floatx4 *>(reinterpret_cast<const float *>(x) + off);
    const uint2 b = *reinterpret_cast<const uint2 *>(reinterpret_cast<const unsigned short *>(x) + off);
    floatx4 v;
    v.x = __uint_as_float(b.x << 16);
    v.y = __uint_as_float(b.x & 0xffff0000u);
    v.z = __uint_as_float(b.y << 16);
    v.w = __uint_as_float(b.y & 0xffff0000u);
    return v;
}

template <class T, int LAYOUT, int DT>
__device__ __forceinline__ void fetch_panel(floatx4 (&st)[T::PASSES], const Operand &op, long k0, int col0,
                                            int tid)
{
#pragma unroll
    for (int p = 0; p < T::PASSES; ++p) {
        const int idx = tid + p * T::NT;
        floatx4 v = {0.f, 0.f, 0.f, 0.f};
        if (idx < T::V4) {
            if (LAYOUT == kRows) {
                const int r = idx / (T::BM / 4);
                const int c = (idx % (T::BM / 4)) * 4;
                const long k = k0 + r;
                const int col = col0 + c;
                if (k < op.K && col < op.d) {
                    const long off = k * op.ld + col;
                    if (op.vec && col + 3 < op.d) {
                        v = load4<DT>(op.x, off);
                    } else {
                        v.x = load1<DT>(op.x, off);
                        if (col + 1 < op.d) v.y = load1<DT>(op.x, off + 1);
                        if (col + 2 < op.d) v.z = load1<DT>(op.x, off + 2);
                        if (col + 3 < op.d) v.w = load1<DT>(op.x, off + 3);
                    }
                }
            } else {
                const int c = idx / (T::KT / 4);
                const int kq = idx % (T::KT / 4);
                const long k = k0 + kq * 4;
                const int ch = col0 + c;
                if (ch < op.d && k < op.K) {
                    if (op.vec) {   // hw % 4 == 0: the four k stay inside one image
                        const long n = k / op.hw;
                        const long p0 = k - n * op.hw;
                        v = load4<DT>(op.x, (n * op.ctot + ch) * (long)op.hw + p0);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const long kk = k + e;
                            if (kk < op.K) {
                                const long n = kk / op.hw;
                                const long p0 = kk - n * op.hw;
                                v[e] = load1<DT>(op.x, (n * op.ctot + ch) * (long)op.hw + p0);
                            }
                        }
                    }
                }
            }
        }
        st[p] = v;
    }
}

// Row-major panels for a prefetch ring: every load is issued unconditionally, from an address clamped into
// the operand, and what lies outside is zeroed when the panel is written to LDS (commit_rows_masked).  A
// load under a condition cannot be counted as in flight by the compiler, which then waits for every
// outstanding load wherever it needs one of them, and a ring of register sets is left without effect.
// VEC (aligned 4-element loads) is a template argument for the same reason: both shapes of load in one
// loop, chosen at run time, would again leave the count open.
template <class T, int DT, bool VEC>
__device__ __forceinline__ void fetch_rows_clamped(floatx4 (&st)[T::PASSES], const Operand &op, long k0, int col0,
                                                   int tid)
{
#pragma unroll
    for (int p = 0; p < T::PASSES; ++p) {
        int idx = tid + p * T::NT;
        if (T::V4 % T::NT != 0 && idx >= T::V4) idx = T::V4 - 1;      // threads without a slot in the last pass
        const int r = idx / (T::BM / 4);
        const int c = (idx % (T::BM / 4)) * 4;
        long k = k0 + r;
        if (k >= op.K) k = op.K - 1;
        const int col = col0 + c;
        if (VEC) {
            // col0 is a tile origin inside the operand and a multiple of 4; the row pitch is a multiple of 4
            // and at least d, so the four elements from any aligned column below d lie inside the row
            st[p] = load4<DT>(op.x, k * op.ld + (col < op.d ? col : col0));
        } else {
            const int last = op.d - 1;
            floatx4 v;
            v.x = load1<DT>(op.x, k * op.ld + (col < last ? col : last));
            v.y = load1<DT>(op.x, k * op.ld + (col + 1 < last ? col + 1 : last));
            v.z = load1<DT>(op.x, k * op.ld + (col + 2 < last ? col + 2 : last));
            v.w = load1<DT>(op.x, k * op.ld + (col + 3 < last ? col + 3 : last));
            st[p] = v;
        }
    }
}

// Zero what a clamped fetch read from outside the operand (in registers, before the panel is used).
template <class T>
__device__ __forceinline__ void mask_rows(floatx4 (&st)[T::PASSES], const Operand &op, long k0, int col0, int tid)
{
#pragma unroll
    for (int p = 0; p < T::PASSES; ++p) {
        const int idx = tid + p * T::NT;
        const int r = idx / (T::BM / 4);
        const int c = (idx % (T::BM / 4)) * 4;
        const bool row = idx < T::V4 && k0 + r < op.K;
        const int col = col0 + c;
        st[p].x = (row && col < op.d) ? st[p].x : 0.f;
        st[p].y = (row && col + 1 < op.d) ? st[p].y : 0.f;
        st[p].z = (row && col + 2 < op.d) ? st[p].z : 0.f;
        st[p].w = (row && col + 3 < op.d) ? st[p].w : 0.f;
    }
}

template <class T>
__device__ __forceinline__ void commit_rows_masked(const floatx4 (&st)[T::PASSES], const Operand &op, long k0,
                                                   int col0, float *lds, int tid)
{
#pragma unroll
    for (int p = 0; p < T::PASSES; ++p) {
        const int idx = tid + p * T::NT;
        if (idx < T::V4) {
            const int r = idx / (T::BM / 4);
            const int c = (idx % (T::BM / 4)) * 4;
            const bool row = k0 + r < op.K;
            const int col = col0 + c;
            floatx4 v;
            v.x = (row && col < op.d) ? st[p].x : 0.f;
            v.y = (row && col + 1 < op.d) ? st[p].y : 0.f;
            v.z = (row && col + 2 < op.d) ? st[p].z : 0.f;
            v.w = (row && col + 3 < op.d) ? st[p].w : 0.f;
            *reinterpret_cast<floatx4 *>(lds + r * T::PITCH + c) = v;
        }
    }
}

// ---- registers -> LDS --------------------------------------------------------
template <class T, int LAYOUT>
__device__ __forceinline__ void commit_panel(const floatx4 (&st)[T::PASSES], float *lds, int tid)
{
#pragma unroll
    for (int p = 0; p < T::PASSES; ++p) {
        const int idx = tid + p * T::NT;
        if (idx < T::V4) {
            if (LAYOUT == kRows) {
                const int r = idx / (T::BM / 4);
                const int c = (idx % (T::BM / 4)) * 4;
                *reinterpret_cast<floatx4 *>(lds + r * T::PITCH + c) = st[p];
            } else {
                const int c = idx / (T::KT / 4);
                const int kq = idx % (T::KT / 4);
                float *dst = lds + c * T::PK + kq * 4;
                dst[0] = st[p].x;
                dst[1] = st[p].y;
                dst[2] = st[p].z;
                dst[3] = st[p].w;
            }
        }
    }
}

// ---- one staged K step of the wave tile ---------------------------------------
// TRI: the wave tile sits on the diagonal of a symmetric product; sub-tiles
// strictly above the diagonal are skipped.
template <class T, int LAYOUT_U, int LAYOUT_V, bool TRI>
__device__ __forceinline__ void mma_stage(const float *Us, const float *Vs, int wm, int wn, int lane,
                                          floatx4 (&acc)[T::WT][T::WT])
{
    const int lr = lane & 15, lk = lane >> 4;
#pragma unroll
    for (int kk = 0; kk < T::KT; kk += 4) {
        float a[T::WT], b[T::WT];
#pragma unroll
        for (int t = 0; t < T::WT; ++t) {
            const int cu = (wm * T::WT + t) * 16 + lr;
            const int cv = (wn * T::WT + t) * 16 + lr;
            a[t] = (LAYOUT_U == kRows) ? Us[(kk + lk) * T::PITCH + cu] : Us[cu * T::PK + kk + lk];
            b[t] = (LAYOUT_V == kRows) ? Vs[(kk + lk) * T::PITCH + cv] : Vs[cv * T::PK + kk + lk];
        }
#pragma unroll
        for (int ti = 0; ti < T::WT; ++ti)
#pragma unroll
            for (int tj = 0; tj < T::WT; ++tj)
                if (!TRI || tj <= ti)
                    acc[ti][tj] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[ti], b[tj], acc[ti][tj], 0, 0, 0);
    }
}

// linear index of a lower-triangular block list -> (bi, bj), bi >= bj
__device__ __forceinline__ void tri_decode(int blk, int &bi, int &bj)
{
    int i = (int)((sqrtf(8.0f * (float)blk + 1.0f) - 1.0f) * 0.5f);
    while ((i + 1) * (i + 2) / 2 <= blk) ++i;
    while (i * (i + 1) / 2 > blk) --i;
    bi = i;
    bj = blk - i * (i + 1) / 2;
}

}  // namespace kfac

// Shared pieces of the wave-unit kernels (factor kernel syrk_wave.hpp, GEMM gemm_wave.hpp):
// 144-wide macro tiles of 9 x 9 v_mfma_f32_16x16x4_f32 tiles, units of at most 45 accumulator
// tiles per wavefront, [16 rows][144 columns] LDS panels filled by buffer_load_dwordx4 ... lds.
#pragma once

#include "tn_engine.hpp"

namespace kfac {

constexpr int W_MT = 144;           // macro tile order
constexpr int W_NT = 9;             // MFMA tiles per macro side
constexpr int W_KT = 16;            // rows per staged K tile
constexpr int W_PANEL = W_KT * W_MT;   // floats per panel stage
constexpr int W_SLOTS = 3;
constexpr unsigned W_OOB = 0x80000000u;

__host__ __device__ inline int wave_blocks_per_split(int m)
{
    int n = (m + 1) / 2;
    for (int i = 2; i < m; ++i) n += i / 2;
    return n;
}

// One k-step (4 rows) of a DIAG unit.  Straight-line code: all 45 tiles are always multiplied (tiles
// past the matrix edge see zero-filled operands), so every MFMA accumulates in place.
__device__ __forceinline__ void unit_diag(const float *P, int kk, int lane, floatx4 (&acc)[45])
{
    const int lr = lane & 15, lk = lane >> 4;
    const float *src = P + (kk + lk) * W_MT + lr;
    float a[W_NT];
#pragma unroll
    for (int t = 0; t < W_NT; ++t) a[t] = src[t * 16];
#pragma unroll
    for (int ti = 0; ti < W_NT; ++ti)
#pragma unroll
        for (int tj = 0; tj <= ti; ++tj)
            acc[ti * (ti + 1) / 2 + tj] =
                __builtin_amdgcn_mfma_f32_16x16x4f32(a[ti], a[tj], acc[ti * (ti + 1) / 2 + tj], 0, 0, 0);
}

// One k-step of a HALF unit: 9 row tiles x NC (5 or 4) column tiles.
template <int NC>
__device__ __forceinline__ void unit_half(const float *Pr, const float *Pc, int kk, int lane, floatx4 (&acc)[45])
{
    const int lr = lane & 15, lk = lane >> 4;
    const float *sr = Pr + (kk + lk) * W_MT + lr;
    const float *sc = Pc + (kk + lk) * W_MT + lr;     // Pc already points at the first column tile
    float a[W_NT], b[NC];
#pragma unroll
    for (int t = 0; t < W_NT; ++t) a[t] = sr[t * 16];
#pragma unroll
    for (int t = 0; t < NC; ++t) b[t] = sc[t * 16];
#pragma unroll
    for (int ti = 0; ti < W_NT; ++ti)
#pragma unroll
        for (int tj = 0; tj < NC; ++tj)
            acc[ti * 5 + tj] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[ti], b[tj], acc[ti * 5 + tj], 0, 0, 0);
}

enum WaveKind : int { kSingle = 0, kDiag = 1, kHalf5 = 2, kHalf4 = 3 };

constexpr int W_NSTAGE = 4;                              // ring of stage buffers (three stages in flight)
constexpr int W_STAGE = W_SLOTS * W_PANEL;               // floats per stage buffer
constexpr int W_LDS_FLOATS = W_NSTAGE * W_STAGE + 256;   // + 1 KB landing zone for the padding loads

typedef int int4v __attribute__((ext_vector_type(4)));

// One 1 KB global->LDS copy: lane l moves 16 bytes from (resource base + voff + soff) to LDS byte
// address lds_byte + 16*l.  Out-of-range offsets store zeros.  Issued through inline assembly so
// that the wait for its completion can be placed by hand (s_waitcnt vmcnt(N) in wave_sync): the
// loop keeps three stages of loads in flight behind the MFMAs.
__device__ __forceinline__ void dma16(unsigned lds_byte, unsigned voff, int4v rsrc, unsigned soff)
{
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_byte), "v"(voff), "s"(rsrc), "s"(soff)
                 : "memory");
}

// Wait until at most two stages of this wave's loads are outstanding, then meet the other waves.
__device__ __forceinline__ void wave_sync()
{
    asm volatile("s_waitcnt vmcnt(18)\n\ts_barrier" ::: "memory");
}

}  // namespace kfac

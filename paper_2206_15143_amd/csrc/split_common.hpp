// Shared pieces of the split-bf16 kernels (gemm_split.hpp, syrk_split.hpp): tile constants and the cut of fp32
// values into three bf16 pieces.
#pragma once

#include "wave_common.hpp"

namespace kfac {

constexpr int S_BM = 256;                     // rows of C per workgroup (columns of A)
constexpr int S_BN = 128;                     // columns of C per workgroup (columns of B)
constexpr int S_KT = 16;                      // rows of the operands per stage
constexpr int S_PANEL_A = S_KT * S_BM;        // floats
constexpr int S_PANEL_B = S_KT * S_BN;
constexpr int S_STAGE = S_PANEL_A + S_PANEL_B;   // 6144 floats = 24 KB
constexpr int S_NSTAGE = 3;
constexpr int S_LDS_FLOATS = S_NSTAGE * S_STAGE; // 72 KB

typedef __bf16 sbf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 sbf16x2 __attribute__((ext_vector_type(2)));
typedef float sfloat2 __attribute__((ext_vector_type(2)));
typedef unsigned suint4 __attribute__((ext_vector_type(4)));

// Eight fp32 values -> three packed bf16 pieces.  Each piece is the upper half of the fp32 word of what is left
// (truncation: the pieces have the sign of x and add up to x exactly, 8 + 8 + 8 significant bits), so a level
// costs one byte permute per two values and an AND and a subtraction per value, all full-rate operations (the
// rounding conversion v_cvt_pk_bf16_f32 measured at a quarter of that rate).
__device__ __forceinline__ void split_pieces(const float (&x)[8], suint4 &p1, suint4 &p2, suint4 &p3)
{
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const float a = x[2 * q], b = x[2 * q + 1];
        const unsigned ua = __builtin_bit_cast(unsigned, a), ub = __builtin_bit_cast(unsigned, b);
        p1[q] = __builtin_amdgcn_perm(ub, ua, 0x07060302u);
        const float ra = a - __builtin_bit_cast(float, ua & 0xffff0000u);
        const float rb = b - __builtin_bit_cast(float, ub & 0xffff0000u);
        const unsigned va = __builtin_bit_cast(unsigned, ra), vb = __builtin_bit_cast(unsigned, rb);
        p2[q] = __builtin_amdgcn_perm(vb, va, 0x07060302u);
        const float sa = ra - __builtin_bit_cast(float, va & 0xffff0000u);
        const float sb = rb - __builtin_bit_cast(float, vb & 0xffff0000u);
        p3[q] = __builtin_amdgcn_perm(__builtin_bit_cast(unsigned, sb), __builtin_bit_cast(unsigned, sa), 0x07060302u);
    }
}

}  // namespace kfac

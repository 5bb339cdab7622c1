// Problem descriptors of the factor (X^T X) kernels: one entry per factor in a grouped launch.
#pragma once

#include "common.hpp"

namespace kfac {

struct SyrkProb {
    const void *x;
    float *partial;   // [splits][nblk][BM*BM] tiles, then [splits][nb][BM] column sums
    float *F;
    long K;
    long ld;
    int d;            // core columns
    int hw, ctot;
    int nb;           // block tiles per side
    int splits;
    int tiles_per_split;
    int blk_start;    // first flattened block of this problem (partial kernel)
    int red_start;    // first flattened block of this problem (reduce kernel)
    int vec;
    int has_bias;
    float scale, decay;
};

struct SyrkTable {
    int count;
    int debug;   // measurement switches of the wave kernel (0 in normal use): 1 = no MFMAs, 2 = no data loads
    int starts[kMaxProblems];   // blk_start of every problem, compact: searched by bisection
    SyrkProb p[kMaxProblems];
};

}  // namespace kfac

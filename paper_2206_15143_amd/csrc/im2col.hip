// Patch extraction for convolution layers (the "convolution as a linear
// transformation" of the footnote in section 3 of the DP-KFAC paper):
//
//   out[(n, oh, ow)][(c, i, j)] = x[n, c, oh*stride - pad_h + i, ow*stride - pad_w + j]   (0 outside)
//
// NCHW in, row-major [B*Ho*Wo, ld] out, same element type.  The bias column is
// not written (the factor kernel derives its border from column sums), so rows
// stay 16-byte aligned and every store is a full 16-byte vector.
//
// One workgroup handles (image n, strip of SR output rows, chunk of CC input
// channels): the input slab it needs (with the zero halo) is staged once in
// LDS with coalesced reads, together with a small table of slab offsets per
// output column; then consecutive threads write consecutive 16-byte column
// groups of consecutive output rows.
#include "common.hpp"

#include <algorithm>

namespace kfac {

struct Im2colProb {
    const void *x;
    void *out;
    int B, C, H, W, kh, kw, stride, pad_h, pad_w, Ho, Wo;
    int ld;
    int SR, CC;         // output rows per strip, channels per chunk
    int nstrips, nchunks;
    int IR, WP;         // slab rows / row pitch
    int blk_start;
};

struct Im2colTable {
    int count;
    Im2colProb p[kMaxProblems];
};

template <typename E> struct VecOf;
template <> struct VecOf<float> { typedef floatx4 type; static constexpr int N = 4; };
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
template <> struct VecOf<unsigned short> { typedef uintx4 type; static constexpr int N = 8; };

template <typename E>
__global__ __launch_bounds__(256) void im2col_kernel(const Im2colTable tab)
{
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int VEC = VecOf<E>::N;

    int pi = 0;
    while (pi + 1 < tab.count && (int)blockIdx.x >= tab.p[pi + 1].blk_start) ++pi;
    const Im2colProb &pr = tab.p[pi];
    int local = blockIdx.x - pr.blk_start;
    const int chunk = local % pr.nchunks; local /= pr.nchunks;
    const int strip = local % pr.nstrips;
    const int n = local / pr.nstrips;

    const int kk = pr.kh * pr.kw;
    const int c0 = chunk * pr.CC;
    const int cc = min(pr.CC, pr.C - c0);
    const int oh0 = strip * pr.SR;
    const int sr = min(pr.SR, pr.Ho - oh0);
    const int plane = pr.IR * pr.WP;
    const int slab_elems = pr.CC * plane;       // + 1 zero cell
    const int col0 = c0 * kk;                    // first output column of this chunk
    const bool last = (chunk == pr.nchunks - 1);
    const int ncols_valid = cc * kk;
    const int ncols_out = last ? (pr.ld - col0) : ncols_valid;   // the last chunk also writes the pad columns
    const int ncg = ncols_out / VEC;

    E *slab = reinterpret_cast<E *>(smem);
    int *offs = reinterpret_cast<int *>(smem + ((size_t)(slab_elems + 1) * sizeof(E) + 15) / 16 * 16);

    // ---- stage the input slab (zero halo): one wave per slab row, lanes along x, so the only
    // integer division is a scalar one per row ----
    const E *xin = reinterpret_cast<const E *>(pr.x) + ((long)n * pr.C + c0) * pr.H * pr.W;
    const int ir_used = (sr - 1) * pr.stride + pr.kh;
    // lanes of a wave cover rpp slab rows at a time (rpp = 64 / WP, at least 1), so narrow images
    // keep all lanes busy; (channel, row) advance incrementally
    {
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        const int rpp = pr.WP >= 64 ? 1 : 64 / pr.WP;
        const int lrow = (rpp == 1) ? 0 : lane / pr.WP;
        const int lx = (rpp == 1) ? lane : lane - lrow * pr.WP;
        const int nrows = cc * ir_used;
        const int stride_rows = 4 * rpp;
        int rowid = wave * rpp + lrow;
        int c = rowid / ir_used;
        int r = rowid - c * ir_used;
        const int dc = stride_rows / ir_used, dr = stride_rows - dc * ir_used;
        const bool lane_ok = lrow < rpp;
        for (; rowid < nrows; rowid += stride_rows) {
            if (lane_ok) {
                const int ih = oh0 * pr.stride - pr.pad_h + r;
                const bool rok = ih >= 0 && ih < pr.H;
                const E *src = xin + ((long)c * pr.H + ih) * pr.W - pr.pad_w;
                E *dst = slab + c * plane + r * pr.WP;
                for (int xx = lx; xx < pr.WP; xx += 64) {
                    const int iw = xx - pr.pad_w;
                    E v = 0;
                    if (rok && iw >= 0 && iw < pr.W) v = src[xx];
                    dst[xx] = v;
                }
            }
            c += dc;
            r += dr;
            if (r >= ir_used) { r -= ir_used; ++c; }
        }
    }
    if (threadIdx.x == 0) slab[slab_elems] = 0;
    for (int col = threadIdx.x; col < ncg * VEC; col += 256) {
        int off = slab_elems;                    // pad column -> the zero cell
        if (col < ncols_valid) {
            const int c = col / kk;
            const int rem = col - c * kk;
            const int i = rem / pr.kw;
            const int j = rem - i * pr.kw;
            off = c * plane + i * pr.WP + j;
        }
        offs[col] = off;
    }
    __syncthreads();

    // ---- write the rows: item = (row, 16-byte column group).  Thread t keeps ONE column group
    // (t mod ncg) for the whole strip and walks rows t / ncg, t / ncg + rows_per_pass, ...: its VEC slab
    // offsets are read from the table once and stay in registers, and consecutive threads still write
    // consecutive 16-byte groups of a row.  (The 256 mod ncg threads past the last whole row idle.) ----
    E *out = reinterpret_cast<E *>(pr.out);
    const long row0 = ((long)n * pr.Ho + oh0) * pr.Wo;
    const int nrows = sr * pr.Wo;
    if (ncg <= 256) {
        const int rows_per_pass = 256 / ncg;
        int rowl = threadIdx.x / ncg;
        const int cg = threadIdx.x - rowl * ncg;
        if (rowl >= rows_per_pass) return;
        int o[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) o[e] = offs[cg * VEC + e];
        int ohl = rowl / pr.Wo;
        int ow = rowl - ohl * pr.Wo;
        const int d_oh = rows_per_pass / pr.Wo, d_ow = rows_per_pass - d_oh * pr.Wo;
        for (; rowl < nrows; rowl += rows_per_pass) {
            const int base = ohl * pr.stride * pr.WP + ow * pr.stride;
            E vals[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) vals[e] = slab[o[e] == slab_elems ? o[e] : o[e] + base];
            typename VecOf<E>::type v;
            __builtin_memcpy(&v, vals, sizeof(v));
            *reinterpret_cast<typename VecOf<E>::type *>(out + (row0 + rowl) * pr.ld + col0 + cg * VEC) = v;
            ohl += d_oh;
            ow += d_ow;
            if (ow >= pr.Wo) { ow -= pr.Wo; ++ohl; }
        }
        return;
    }
    // more column groups than threads: every thread walks several groups of each row
    for (int rowl = 0; rowl < nrows; ++rowl) {
        const int ohl = rowl / pr.Wo, ow = rowl - ohl * pr.Wo;
        const int base = ohl * pr.stride * pr.WP + ow * pr.stride;
        for (int cg = threadIdx.x; cg < ncg; cg += 256) {
            E vals[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const int o = offs[cg * VEC + e];
                vals[e] = slab[o == slab_elems ? o : o + base];
            }
            typename VecOf<E>::type v;
            __builtin_memcpy(&v, vals, sizeof(v));
            *reinterpret_cast<typename VecOf<E>::type *>(out + (row0 + rowl) * pr.ld + col0 + cg * VEC) = v;
        }
    }
}

namespace {

int gcd(int a, int b) { return b ? gcd(b, a % b) : a; }

size_t smem_bytes(const Im2colProb &p, int esz)
{
    const size_t slab = ((size_t)(p.CC * p.IR * p.WP + 1) * esz + 15) / 16 * 16;
    return slab + (size_t)(p.CC * p.kh * p.kw + 16) * sizeof(int);
}

// Strip height SR and channel chunk CC of a layer.  Measured over the 3x3 / 7x7, stride 1 / 2 shapes of
// the workloads, alone and inside the grouped factor update: the slab of a workgroup should stay near
// 20 KB (several workgroups per CU, so the load phase of one hides behind the stores of others) and the
// channel chunk narrow (pieces of ~128 elements per output row), which leaves the slab to a taller
// strip: the halo rows are re-read once per strip.
void plan_enough_blocks(Im2colProb &p, int esz)
{
    const Tuning &t = tuning();
    const int vec = 16 / esz;
    const int kk = p.kh * p.kw;
    const int g = vec / gcd(kk, vec);             // CC must be a multiple of g (or the whole of C)
    p.WP = (p.Wo - 1) * p.stride + p.kw;
    auto set = [&](int sr, int cc) {
        p.SR = sr;
        p.IR = (sr - 1) * p.stride + p.kh;
        p.CC = cc;
        p.nstrips = (p.Ho + sr - 1) / sr;
        p.nchunks = (p.C + cc - 1) / cc;
    };
    auto slab = [&](int sr, int cc) { return (size_t)cc * ((sr - 1) * p.stride + p.kh) * p.WP * esz + (size_t)cc * kk * 4 + 512; };
    const size_t lds = (size_t)std::min(60l * 1024, std::max(2048l, t.im2col_lds_bytes));   // <= kIm2colLdsCap
    long cc = ((t.im2col_piece_elems + kk - 1) / kk + g - 1) / g * g;
    if (cc >= p.C) cc = p.C;
    while (cc > g && cc != p.C && slab(1, (int)cc) > lds) cc -= g;
    if (cc == p.C && slab(1, (int)cc) > lds) cc = std::max<long>(g, (long)(p.C / g) * g);
    while (cc > g && slab(1, (int)cc) > lds) cc -= g;
    const long row_bytes = (long)p.Wo * cc * kk * esz;      // output of one strip row of the chunk
    int sr = (int)std::max(1l, std::min<long>(p.Ho, t.im2col_block_bytes / std::max(1l, row_bytes)));
    while (sr > 1 && slab(sr, (int)cc) > lds) --sr;
    set(sr, (int)cc);
    while (sr > 1 && (long)p.B * p.nstrips * p.nchunks < t.im2col_min_blocks) set(--sr, (int)cc);
    set((p.Ho + p.nstrips - 1) / p.nstrips, (int)cc);   // same number of strips, equal heights
}

constexpr long kIm2colLdsCap = 60l * 1024;   // what plan_enough_blocks may give a workgroup

int min_chunk(int kk, int esz)
{
    const int vec = 16 / esz;
    return vec / gcd(kk, vec);
}

}  // namespace

bool im2col_fits(int kh, int kw, int stride, int Wo, int esz)
{
    const long g = min_chunk(kh * kw, esz);
    const long WP = (long)(Wo - 1) * stride + kw;
    return g * kh * WP * esz + g * kh * kw * 4 + 512 <= kIm2colLdsCap;
}

hipError_t im2col_launch(const Im2colJob *jobs, int n, hipStream_t s)
{
    for (int dt = 0; dt < 2; ++dt) {
        Im2colTable tab;
        tab.count = 0;
        int blocks = 0;
        size_t smem = 0;
        auto flush = [&]() -> hipError_t {
            if (tab.count == 0) return hipSuccess;
            if (smem > 64 * 1024) return hipErrorInvalidValue;   // cannot happen for shapes im2col_fits() accepts
            if (dt == 0)
                KFAC_LAUNCH(KFAC_K_IM2COL, s, (im2col_kernel<float>), dim3(blocks), dim3(256), smem, tab);
            else
                KFAC_LAUNCH(KFAC_K_IM2COL, s, (im2col_kernel<unsigned short>), dim3(blocks), dim3(256), smem, tab);
            tab.count = 0;
            blocks = 0;
            smem = 0;
            return hipGetLastError();
        };
        for (int i = 0; i < n; ++i) {
            if (jobs[i].dtype != dt) continue;
            const Im2colJob &j = jobs[i];
            Im2colProb &p = tab.p[tab.count++];
            p.x = j.x; p.out = j.out;
            p.B = j.B; p.C = j.C; p.H = j.H; p.W = j.W; p.kh = j.kh; p.kw = j.kw;
            p.stride = j.stride; p.pad_h = j.pad_h; p.pad_w = j.pad_w; p.Ho = j.Ho; p.Wo = j.Wo; p.ld = j.ld;
            plan_enough_blocks(p, dt == 0 ? 4 : 2);
            p.blk_start = blocks;
            blocks += p.B * p.nstrips * p.nchunks;
            smem = std::max(smem, smem_bytes(p, dt == 0 ? 4 : 2));
            if (tab.count == kMaxProblems) {
                hipError_t e = flush();
                if (e != hipSuccess) return e;
            }
        }
        hipError_t e = flush();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace kfac

// fp32 MFMA GEMM of the form  C = A^T B  (both operands stored K-major), used
// for the two-sided preconditioning  P = G_inv * grad * A_inv  (Eq. 5 / rhs of
// Eq. 12 of the DP-KFAC paper): U^T = grad^T G_inv, then P = (U^T)^T A_inv, both
// with row-major outputs, no operand is ever read with a strided K; and for the
// panel products and rank-k updates of the blocked inversion.  Wide products
// go to the wave-unit kernel (gemm_wave.hpp), the rest to the block-tile kernel
// below.
#include <type_traits>
#include "gemm_wave.hpp"
#include "gemm_split.hpp"

#include <algorithm>
#include <vector>

namespace kfac {

struct GemmProb {
    const float *A;
    const float *B;
    float *C;
    long lda, ldb, ldc;
    int M, N, K;
    int tm, tn;       // tiles per side
    int blk_start;
    int mode;
    int p0, p1;
    long doff;
    int vecA, vecB;
    const float *rv, *cv;   // kStoreDiv
    float gamma;
    const int *gate;        // null, or two float bit patterns: leave C alone unless their product exceeds gate_cond
    float gate_cond;
    const float *D;         // kSubFrom
    long ldd;
};

// A launch covers up to kMaxGemmProblems products (a 14 KB kernel argument): the preconditioning of a whole
// network is then two launches, and the k-loop latency of a small product is paid once, not once per group of
// layers.  The first block of every product sits in a compact array of its own, searched by bisection.
constexpr int kMaxGemmProblems = 128;

struct GemmTable {
    int count;
    int starts[kMaxGemmProblems];
    GemmProb p[kMaxGemmProblems];
};

template <class T>
__global__ __launch_bounds__(T::NT) void gemm_tn_kernel(const GemmTable tab)
{
    __shared__ float lds[2][2][T::PANEL];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / T::NW, wn = wave % T::NW;

    int pi = 0, hi = tab.count - 1;
    while (pi < hi) {
        const int mid = (pi + hi + 1) >> 1;
        if ((int)blockIdx.x >= tab.starts[mid]) pi = mid;
        else hi = mid - 1;
    }
    const GemmProb &pr = tab.p[pi];
    if (pr.gate && !(__int_as_float(pr.gate[0]) * __int_as_float(pr.gate[1]) > pr.gate_cond)) return;   // uniform
    const int local = blockIdx.x - pr.blk_start;
    int bi, bj;
    if (pr.mode == kSubLowerSkip) {
        tri_decode(local, bi, bj);
    } else {
        bi = local / pr.tn;
        bj = local - bi * pr.tn;
    }
    const int m0 = bi * T::BM, n0 = bj * T::BM;

    Operand opA, opB;
    opA.x = pr.A; opA.K = pr.K; opA.ld = pr.lda; opA.d = pr.M; opA.hw = 1; opA.ctot = 0; opA.vec = pr.vecA;
    opB.x = pr.B; opB.K = pr.K; opB.ld = pr.ldb; opB.d = pr.N; opB.hw = 1; opB.ctot = 0; opB.vec = pr.vecB;

    floatx4 acc[T::WT][T::WT];
#pragma unroll
    for (int i = 0; i < T::WT; ++i)
#pragma unroll
        for (int j = 0; j < T::WT; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};

    // The panels are fetched D stages ahead into a ring of register sets, so that a stage waits for loads
    // issued D stages earlier: the short, latency-bound products (a few workgroups per matrix, each walking
    // the whole depth) live on that.  Set r holds stage t with t mod D = r; it is free again once that stage
    // has been written to LDS.  The large tiles keep one set (registers).
    constexpr int D = T::BM <= 64 ? 3 : 1;
    const long ktiles = (pr.K + T::KT - 1) / T::KT;
    auto k_loop = [&](auto vec_a, auto vec_b) {
        constexpr bool VA = decltype(vec_a)::value, VB = decltype(vec_b)::value;
        floatx4 sa[D][T::PASSES], sb[D][T::PASSES];
#pragma unroll
        for (int r = 0; r < D; ++r) {       // stages past the depth re-read the last rows and are never written to LDS
            fetch_rows_clamped<T, 0, VA>(sa[r], opA, (long)r * T::KT, m0, tid);
            fetch_rows_clamped<T, 0, VB>(sb[r], opB, (long)r * T::KT, n0, tid);
            __builtin_amdgcn_sched_barrier(0);      // issued in the order the loop consumes them
        }
        commit_rows_masked<T>(sa[0], opA, 0, m0, lds[0][0], tid);
        commit_rows_masked<T>(sb[0], opB, 0, n0, lds[0][1], tid);
        __syncthreads();
        for (long t0 = 0; t0 < ktiles; t0 += D) {
#pragma unroll
            for (int r = 0; r < D; ++r) {
                const long t = t0 + r;
                if (t >= ktiles) break;
                const int cur = (int)(t & 1);
                fetch_rows_clamped<T, 0, VA>(sa[r], opA, (t + D) * T::KT, m0, tid);
                fetch_rows_clamped<T, 0, VB>(sb[r], opB, (t + D) * T::KT, n0, tid);
                mma_stage<T, kRows, kRows, false>(lds[cur][0], lds[cur][1], wm, wn, lane, acc);
                if (t + 1 < ktiles) {
                    commit_rows_masked<T>(sa[(r + 1) % D], opA, (t + 1) * T::KT, m0, lds[cur ^ 1][0], tid);
                    commit_rows_masked<T>(sb[(r + 1) % D], opB, (t + 1) * T::KT, n0, lds[cur ^ 1][1], tid);
                }
                __syncthreads();
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    if (opA.vec) {
        if (opB.vec) k_loop(std::true_type{}, std::true_type{});
        else k_loop(std::true_type{}, std::false_type{});
    } else {
        if (opB.vec) k_loop(std::false_type{}, std::true_type{});
        else k_loop(std::false_type{}, std::false_type{});
    }

    const int lr = lane & 15, lk = lane >> 4;
#pragma unroll
    for (int ti = 0; ti < T::WT; ++ti)
#pragma unroll
        for (int tj = 0; tj < T::WT; ++tj) {
            const int n = n0 + (wn * T::WT + tj) * 16 + lr;
            if (n >= pr.N) continue;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int m = m0 + (wm * T::WT + ti) * 16 + 4 * lk + v;
                if (m >= pr.M) continue;
                const float val = acc[ti][tj][v];
                if (pr.mode == kStore) {
                    pr.C[(long)m * pr.ldc + n] = val;
                } else if (pr.mode == kStoreT) {
                    pr.C[(long)n * pr.ldc + m] = val;
                } else if (pr.mode == kStoreDiv) {
                    pr.C[(long)m * pr.ldc + n] = val / (pr.rv[m] * pr.cv[n] + pr.gamma);
                } else if (pr.mode == kSubFrom) {
                    pr.C[(long)m * pr.ldc + n] = pr.D[(long)m * pr.ldd + n] - val;
                } else if (pr.mode == kSubRect || pr.mode == kAddRect) {
                    const bool skip = ((long)n > (long)m + pr.doff) || (n >= pr.p0 && n < pr.p1);
                    if (!skip) pr.C[(long)m * pr.ldc + n] += pr.mode == kAddRect ? val : -val;
                } else {
                    const bool skip = (n > m) || (m >= pr.p0 && m < pr.p1) || (n >= pr.p0 && n < pr.p1);
                    if (!skip) pr.C[(long)m * pr.ldc + n] -= val;
                }
            }
        }
}

namespace {

const int kBms[] = {128, 144, 64, 32};

int choose_bm(int M, int N, bool square_lower)
{
    const long force = square_lower ? tuning().update_bm : tuning().gemm_bm;
    if (force)
        for (int i = 0; i < 4; ++i)
            if (kBms[i] == force) return i;
    int best = 0;
    double best_cost = 1e300;
    for (int i = 0; i < 4; ++i) {
        const long bm = kBms[i];
        const long tm = (M + bm - 1) / bm, tn = (N + bm - 1) / bm;
        const double tiles = square_lower ? (double)tm * (tm + 1) / 2 : (double)tm * tn;
        const double penalty = bm >= 128 ? 1.0 : (bm >= 64 ? 1.15 : 1.4);
        const double cost = tiles * bm * bm * penalty;
        if (cost < best_cost - 1e-9) { best_cost = cost; best = i; }
    }
    return best;
}

template <class T>
hipError_t launch_one(const GemmTable &tab, int blocks, hipStream_t s)
{
    KFAC_LAUNCH(KFAC_K_GEMM, s, (gemm_tn_kernel<T>), dim3(blocks), dim3(T::NT), 0, tab);
    double flops = 0.0;
    for (int k = 0; k < tab.count; ++k) {
        const GemmProb &p = tab.p[k];
        if (p.gate) continue;       // may be skipped on the device: not counted
        if (p.mode != kSubLowerSkip) { flops += 2.0 * p.M * p.N * p.K; continue; }
        const double live = (double)p.M - (double)(std::min(p.p1, p.M) - p.p0);
        flops += live * (live + 1.0) * p.K;
    }
    timing_work(flops, flops);
    return hipGetLastError();
}

}  // namespace

namespace {
// flops of the definition of a product (the lower-triangle update counts the entries it touches)
double gemm_job_flops(const GemmJob &j)
{
    if (j.mode == kSubRect || j.mode == kAddRect) {
        // rows m = 0..M-1 touch the columns n <= min(N - 1, m + doff) outside [p0, p1)
        double cnt = 0.0;
        for (int m = 0; m < j.M; ++m) {
            const long hi = std::min<long>(j.N - 1, m + j.doff);
            if (hi < 0) continue;
            long c = hi + 1;
            const long a = std::max<long>(0, j.p0), b = std::min<long>(hi + 1, j.p1);
            if (b > a) c -= b - a;
            cnt += (double)c;
        }
        return 2.0 * cnt * j.K;
    }
    if (j.mode != kSubLowerSkip) return 2.0 * j.M * j.N * j.K;
    const double live = (double)j.M - (double)(std::min(j.p1, j.M) - j.p0);
    return live * (live + 1.0) * j.K;
}

// Products wide enough to fill 144-wide macro tiles go to the wave-unit kernel.  A lower-triangular
// update qualifies only when its untouched band starts and ends on macro-tile boundaries.
bool wave_gemm_eligible(const GemmJob &j)
{
    if (!tuning().use_wave_gemm || j.mode == kStoreT || j.mode == kStoreDiv || j.mode == kSubRect || j.mode == kAddRect ||
        j.mode == kSubFrom || j.gate)
        return false;
    if (j.M < 100 || j.N < 100 || j.K < 16) return false;
    if ((long)j.K * j.lda * 4 > 0x7fffffffl || (long)j.K * j.ldb * 4 > 0x7fffffffl) return false;
    if (((uintptr_t)j.A) % 4 || ((uintptr_t)j.B) % 4) return false;
    if (j.mode == kSubLowerSkip)
        return j.M == j.N && j.p0 % W_MT == 0 && (j.p1 % W_MT == 0 || j.p1 >= j.M);
    return true;
}

hipError_t wave_gemm_launch(const GemmJob *jobs, const std::vector<int> &idx, hipStream_t s)
{
    GemmWTable tab;
    tab.count = 0;
    long blocks = 0;
    double wflops = 0.0;
    auto flush = [&]() -> hipError_t {
        if (tab.count == 0) return hipSuccess;
        // Contiguous tile ranges per XCD pay when a launch spans many problems of similar depth (each XCD
        // then works on a few matrices).  With mixed depths the long workgroups would pile up on one
        // XCD, and with a handful of problems the round-robin order measured as good or better.
        int kmin = tab.p[0].K, kmax = tab.p[0].K;
        for (int k = 1; k < tab.count; ++k) {
            kmin = std::min(kmin, tab.p[k].K);
            kmax = std::max(kmax, tab.p[k].K);
        }
        tab.xcd_remap = (tab.count >= tuning().gemm_xcd_remap_min && 2 * kmax <= 3 * kmin) ? 1 : 0;
        KFAC_LAUNCH(KFAC_K_GEMM_WAVE, s, gemm_wave_kernel, dim3((unsigned)blocks), dim3(256), 0, tab);
        timing_work(wflops, wflops);
        wflops = 0.0;
        tab.count = 0;
        blocks = 0;
        return hipGetLastError();
    };
    for (int i : idx) {
        const GemmJob &j = jobs[i];
        GemmWProb &p = tab.p[tab.count++];
        p.A = j.A; p.B = j.B; p.C = j.C;
        p.lda = (int)j.lda; p.ldb = (int)j.ldb; p.ldc = (int)j.ldc;
        p.M = j.M; p.N = j.N; p.K = j.K;
        p.mI = (j.M + W_MT - 1) / W_MT;
        const int nJ = (j.N + W_MT - 1) / W_MT;
        p.nJ2 = (nJ + 1) / 2;
        p.mode = j.mode; p.p0 = j.p0; p.p1 = j.p1;
        p.blk_start = (int)blocks;
        wflops += gemm_job_flops(j);
        if (j.mode == kSubLowerSkip) {
            for (int I = 0; I < p.mI; ++I) blocks += I / 2 + 1;
        } else {
            blocks += (long)p.mI * p.nJ2;
        }
        if (tab.count == kMaxProblems) {
            hipError_t e = flush();
            if (e != hipSuccess) return e;
        }
    }
    return flush();
}
}  // namespace

namespace {
// Products that fill 256 x 128 tiles reasonably go to the split-bf16 kernel (gemm_split.hpp).
bool split_gemm_eligible(const GemmJob &j)
{
    if (!tuning().use_split_gemm || (j.mode != kStore && j.mode != kSubLowerSkip && j.mode != kSubRect && j.mode != kAddRect))
        return false;
    if (j.M < tuning().split_gemm_min_m || j.N < 64 || j.K < 16) return false;
    // a product of a tile or two is bound by the latency of one tile's K loop and read-modify-write (55 us at
    // K = 256): the 64-wide tiles of the block-tile kernel spread it over many CUs and finish in 10-15 us
    if ((long)j.M * j.N < 4l * S_BM * S_BN) return false;
    if (j.mode == kStore && !j.wide_tiles) {
        if (j.K < tuning().split_gemm_min_k) return false;
        // 256 x 128 tiles: products that fill them badly (a 257-row or 65-column operand) stay with the 144-wide
        // tiles of the fp32 kernel
        const double tiles = (double)((j.M + S_BM - 1) / S_BM) * ((j.N + S_BN - 1) / S_BN);
        if ((double)j.M * j.N < 0.01 * tuning().split_gemm_min_fill * tiles * S_BM * S_BN) return false;
    }
    if ((long)j.K * j.lda * 4 > 0x7fffffffl || (long)j.K * j.ldb * 4 > 0x7fffffffl) return false;
    if ((long)j.M * j.ldc * 4 > 0x7fffffffl) return false;
    if (((uintptr_t)j.A) % 4 || ((uintptr_t)j.B) % 4) return false;
    if (j.mode == kSubLowerSkip) return j.M == j.N;
    return true;
}

hipError_t split_gemm_launch(const GemmJob *jobs, const std::vector<int> &idx, hipStream_t s)
{
    GemmSTable tab;
    tab.count = 0;
    tab.debug = (int)tuning().wave_debug;
    long blocks = 0;
    double flops = 0.0;
    auto flush = [&]() -> hipError_t {
        if (tab.count == 0) return hipSuccess;
        KFAC_LAUNCH(KFAC_K_GEMM_SPLIT, s, gemm_split_kernel, dim3((unsigned)blocks), dim3(256), 0, tab);
        timing_work(flops, 6.0 * flops);
        tab.count = 0;
        blocks = 0;
        flops = 0.0;
        return hipGetLastError();
    };
    for (int i : idx) {
        const GemmJob &j = jobs[i];
        GemmSProb &p = tab.p[tab.count++];
        p.A = j.A; p.B = j.B; p.C = j.C;
        p.lda = (int)j.lda; p.ldb = (int)j.ldb; p.ldc = (int)j.ldc;
        p.M = j.M; p.N = j.N; p.K = j.K;
        p.tI = (j.M + S_BM - 1) / S_BM;
        p.tJ = (j.N + S_BN - 1) / S_BN;
        p.mode = j.mode; p.p0 = j.p0; p.p1 = j.p1;
        p.doff = (int)std::min<long>(j.doff, 1l << 30);
        if (j.mode == kSubLowerSkip) p.doff = 0;
        p.gate = j.gate; p.gate_cond = j.gate_cond;
        p.blk_start = (int)blocks;
        for (int I = 0; I < p.tI; ++I) blocks += split_row_len(p.mode, p.tJ, p.doff, I);
        if (!j.gate) flops += gemm_job_flops(j);       // a gated product may be skipped on the device: not counted
        if (tab.count == kMaxProblems) {
            hipError_t e = flush();
            if (e != hipSuccess) return e;
        }
    }
    return flush();
}
}  // namespace

namespace {
// K slices of deep products.  A call with few 256 x 128 tiles, some of them hundreds of K stages deep, leaves most
// compute units with one long workgroup and nothing to pack beside it (three 512 x 4609 x 4609 products: 222 tiles
// of 289 stages on 256 units).  Such a product is cut into K slices: slice 0 stores into C, the others into
// partial matrices in the workspace, and a reduction adds them to C in slice order (a fixed order: the result
// does not depend on the schedule).  The partials are M x N, small beside the K x N operand that is read.
constexpr int kMaxKSlices = 8;

int kslice_count(const GemmJob &j, long split_tiles)
{
    const long cap = tuning().gemm_kslice_stages;
    if (cap <= 0 || split_tiles >= 1024) return 1;     // enough tiles to keep every unit busy as it is
    if (j.mode != kStore || j.gate || j.wide_tiles) return 1;
    const long stages = (j.K + S_KT - 1) / S_KT;
    if (2 * stages <= 3 * cap) return 1;
    return (int)std::min<long>(kMaxKSlices, (stages + cap - 1) / cap);
}

// slices per job (1 = as it is); returns the floats of partial matrices needed
size_t plan_kslices(const GemmJob *jobs, int n, std::vector<int> &ks)
{
    ks.assign(n, 1);
    long tiles = 0;
    for (int i = 0; i < n; ++i)
        if (jobs[i].M > 0 && jobs[i].N > 0 && jobs[i].K > 0 && split_gemm_eligible(jobs[i]))
            tiles += (long)((jobs[i].M + S_BM - 1) / S_BM) * ((jobs[i].N + S_BN - 1) / S_BN);
    size_t floats = 0;
    for (int i = 0; i < n; ++i) {
        if (!(jobs[i].M > 0 && jobs[i].N > 0 && jobs[i].K > 0) || !split_gemm_eligible(jobs[i])) continue;
        ks[i] = kslice_count(jobs[i], tiles);
        floats += (size_t)(ks[i] - 1) * align_up((size_t)jobs[i].M * jobs[i].N, 64);
    }
    return floats;
}

struct KRedProb {
    float *C;
    const float *P;      // first partial; the next ones follow at `stride` floats
    long ldc, stride;
    int M, N, parts;
    int blk_start;
};

struct KRedTable {
    int count;
    KRedProb p[kMaxProblems];
};

// C += P_1 + P_2 + ... (in this order); one thread per four consecutive entries of a row
__global__ __launch_bounds__(256) void gemm_kreduce_kernel(const KRedTable tab)
{
    int pi = 0;
    while (pi + 1 < tab.count && (int)blockIdx.x >= tab.p[pi + 1].blk_start) ++pi;
    const KRedProb &pr = tab.p[pi];
    const int n4 = (pr.N + 3) / 4;
    const long item = (long)(blockIdx.x - pr.blk_start) * 256 + threadIdx.x;
    if (item >= (long)pr.M * n4) return;
    const int m = (int)(item / n4), c0 = (int)(item - (long)m * n4) * 4;
    float *c = pr.C + (long)m * pr.ldc + c0;
    const float *q = pr.P + (long)m * pr.N + c0;
    const int cnt = min(4, pr.N - c0);
    float acc[4];
    for (int e = 0; e < cnt; ++e) acc[e] = c[e];
    for (int t = 0; t < pr.parts; ++t, q += pr.stride)
        for (int e = 0; e < cnt; ++e) acc[e] += q[e];
    for (int e = 0; e < cnt; ++e) c[e] = acc[e];
}

hipError_t gemm_launch_plain(const GemmJob *jobs, int n, hipStream_t s);
}  // namespace

size_t gemm_workspace_bytes(const GemmJob *jobs, int n)
{
    std::vector<int> ks;
    return plan_kslices(jobs, n, ks) * sizeof(float);
}

hipError_t gemm_launch(const GemmJob *jobs, int n, hipStream_t s, void *work, size_t work_bytes)
{
    std::vector<int> ks;
    const size_t need = (work != nullptr) ? plan_kslices(jobs, n, ks) * sizeof(float) : 0;
    if (need == 0 || need > work_bytes) return gemm_launch_plain(jobs, n, s);
    std::vector<GemmJob> v;
    std::vector<KRedProb> red;
    float *part = static_cast<float *>(work);
    for (int i = 0; i < n; ++i) {
        const GemmJob &j = jobs[i];
        if (ks[i] <= 1) {
            v.push_back(j);
            continue;
        }
        const long stages = (j.K + S_KT - 1) / S_KT;
        const long per = (stages + ks[i] - 1) / ks[i] * S_KT;      // rows of K per slice
        const size_t stride = align_up((size_t)j.M * j.N, 64);
        int made = 0;
        for (long k0 = 0; k0 < j.K; k0 += per, ++made) {
            GemmJob t = j;
            t.A = j.A + k0 * j.lda;
            t.B = j.B + k0 * j.ldb;
            t.K = (int)std::min<long>(per, j.K - k0);
            t.wide_tiles = true;            // a slice stays on the split-bf16 kernel whatever its depth
            if (made > 0) {
                t.C = part + (size_t)(made - 1) * stride;
                t.ldc = j.N;
            }
            v.push_back(t);
        }
        KRedProb r;
        r.C = j.C; r.P = part; r.ldc = j.ldc; r.stride = (long)stride; r.M = j.M; r.N = j.N; r.parts = made - 1;
        r.blk_start = 0;
        if (r.parts > 0) red.push_back(r);
        part += (size_t)(ks[i] - 1) * stride;
    }
    hipError_t e = gemm_launch_plain(v.data(), (int)v.size(), s);
    if (e != hipSuccess) return e;
    for (size_t g0 = 0; g0 < red.size(); g0 += kMaxProblems) {
        KRedTable tab;
        tab.count = (int)std::min<size_t>(kMaxProblems, red.size() - g0);
        long blocks = 0;
        for (int k = 0; k < tab.count; ++k) {
            tab.p[k] = red[g0 + k];
            tab.p[k].blk_start = (int)blocks;
            blocks += ((long)tab.p[k].M * ((tab.p[k].N + 3) / 4) + 255) / 256;
        }
        KFAC_LAUNCH(KFAC_K_GEMM, s, gemm_kreduce_kernel, dim3((unsigned)blocks), dim3(256), 0, tab);
        timing_work(0.0, 0.0);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

namespace {
hipError_t gemm_launch_plain(const GemmJob *jobs, int n, hipStream_t s)
{
    std::vector<int> cfg(n);
    std::vector<int> wave, split;
    for (int i = 0; i < n; ++i) {
        if (jobs[i].M > 0 && jobs[i].N > 0 && jobs[i].K > 0 && split_gemm_eligible(jobs[i])) {
            cfg[i] = -1;
            split.push_back(i);
        } else if (jobs[i].M > 0 && jobs[i].N > 0 && jobs[i].K > 0 && wave_gemm_eligible(jobs[i])) {
            cfg[i] = -1;
            wave.push_back(i);
        } else {
            cfg[i] = choose_bm(jobs[i].M, jobs[i].N, jobs[i].mode == kSubLowerSkip);
        }
    }
    {   // a small call is bound by its launches, not by its flops: one tile shape for all its products then
        double flops = 0.0, cost[4] = {0.0, 0.0, 0.0, 0.0};
        int used = 0;
        for (int i = 0; i < n; ++i) {
            const GemmJob &j = jobs[i];
            if (cfg[i] < 0 || j.mode == kSubLowerSkip) continue;      // the update products keep their own tile
            if (j.M <= 0 || j.N <= 0 || j.K <= 0) continue;
            used |= 1 << cfg[i];
            flops += 2.0 * j.M * j.N * j.K;
            for (int c = 0; c < 4; ++c) {
                const long bm = kBms[c];
                const long tm = (j.M + bm - 1) / bm, tn = (j.N + bm - 1) / bm;
                cost[c] += (double)tm * tn * bm * bm * (bm >= 128 ? 1.0 : (bm >= 64 ? 1.15 : 1.4)) * j.K;
            }
        }
        if (!tuning().gemm_bm && (used & (used - 1)) != 0 && flops < 8e9) {
            int best = 0;
            for (int c = 1; c < 4; ++c)
                if (cost[c] < cost[best]) best = c;
            for (int i = 0; i < n; ++i)
                if (cfg[i] >= 0 && jobs[i].mode != kSubLowerSkip) cfg[i] = best;
        }
    }
    if (!tuning().gemm_bm) {
        // a call whose block-tile products would not even give every CU a workgroup is bound by the K loop of one
        // tile: the 64-wide tiles spread it over four times as many CUs
        long wgs = 0;
        for (int i = 0; i < n; ++i) {
            const GemmJob &j = jobs[i];
            if (cfg[i] < 0 || j.mode == kSubLowerSkip || j.M <= 0 || j.N <= 0 || j.K <= 0) continue;
            const long bm = kBms[cfg[i]];
            wgs += ((j.M + bm - 1) / bm) * ((j.N + bm - 1) / bm);
        }
        if (wgs > 0 && wgs < 200)
            for (int i = 0; i < n; ++i)
                if (cfg[i] >= 0 && jobs[i].mode != kSubLowerSkip && kBms[cfg[i]] > 64) cfg[i] = 2;
    }
    if (!split.empty()) {
        std::stable_sort(split.begin(), split.end(), [&](int a, int b) { return jobs[a].K > jobs[b].K; });
        hipError_t e = split_gemm_launch(jobs, split, s);
        if (e != hipSuccess) return e;
    }
    if (!wave.empty()) {
        // deepest products first: launches of similar depth, and the long workgroups start early
        std::stable_sort(wave.begin(), wave.end(), [&](int a, int b) { return jobs[a].K > jobs[b].K; });
        hipError_t e = wave_gemm_launch(jobs, wave, s);
        if (e != hipSuccess) return e;
    }
    for (int c = 0; c < 4; ++c) {
        GemmTable tab;
        tab.count = 0;
        int blocks = 0;
        auto flush = [&]() -> hipError_t {
            if (tab.count == 0) return hipSuccess;
            hipError_t e;
            switch (c) {
                case 0: e = launch_one<Tile<4, 2>>(tab, blocks, s); break;
                case 1: e = launch_one<Tile<3, 3>>(tab, blocks, s); break;
                case 2: e = launch_one<Tile<2, 2>>(tab, blocks, s); break;
                default: e = launch_one<Tile<1, 2>>(tab, blocks, s); break;
            }
            tab.count = 0;
            blocks = 0;
            return e;
        };
        for (int i = 0; i < n; ++i) {
            if (cfg[i] != c) continue;
            const GemmJob &j = jobs[i];
            if (j.M <= 0 || j.N <= 0 || j.K <= 0) continue;
            GemmProb &p = tab.p[tab.count++];
            const int bm = kBms[c];
            p.A = j.A; p.B = j.B; p.C = j.C;
            p.lda = j.lda; p.ldb = j.ldb; p.ldc = j.ldc;
            p.M = j.M; p.N = j.N; p.K = j.K;
            p.tm = (j.M + bm - 1) / bm;
            p.tn = (j.N + bm - 1) / bm;
            p.blk_start = blocks;
            tab.starts[tab.count - 1] = blocks;
            p.mode = j.mode;
            p.p0 = j.p0; p.p1 = j.p1; p.doff = j.doff;
            p.rv = j.rv; p.cv = j.cv; p.gamma = j.gamma; p.gate = j.gate; p.gate_cond = j.gate_cond;
            p.D = j.D; p.ldd = j.ldd;
            p.vecA = (((uintptr_t)j.A) % 16 == 0 && j.lda % 4 == 0) ? 1 : 0;
            p.vecB = (((uintptr_t)j.B) % 16 == 0 && j.ldb % 4 == 0) ? 1 : 0;
            blocks += (j.mode == kSubLowerSkip) ? p.tm * (p.tm + 1) / 2 : p.tm * p.tn;
            if (tab.count == kMaxGemmProblems) {
                hipError_t e = flush();
                if (e != hipSuccess) return e;
            }
        }
        hipError_t e = flush();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace

}  // namespace kfac

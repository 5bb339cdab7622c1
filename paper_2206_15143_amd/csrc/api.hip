// C ABI of the library (see include/kfac.h): argument validation, workspace
// planning and the launch sequences.  No arithmetic happens on the host.
#include "../../include/kfac.h"

#include "common.hpp"

#include <cstring>
#include <mutex>
#include <string>
#include <tuple>
#include <vector>

// Intermediate product of kfac_precondition_static: device memory that belongs to the library image, one copy
// per GPU, held until the process ends.  In host code this name is only a handle for hipGetSymbolAddress.
static __device__ __align__(256) unsigned char scratch[KFAC_STATIC_SCRATCH_BYTES];

namespace kfac {

Tuning &tuning()
{
    static Tuning t;
    return t;
}

namespace {
struct TimingState {
    bool on = false;
    struct Rec { int cls; hipEvent_t a, b; double work, executed; };
    std::vector<Rec> recs;
    std::vector<hipEvent_t> pool;
    hipEvent_t get()
    {
        if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
        hipEvent_t e = nullptr;
        (void)hipEventCreate(&e);
        return e;
    }
};
TimingState &timing()
{
    static TimingState t;
    return t;
}
}  // namespace

bool timing_active() { return timing().on; }

void timing_begin(int cls, hipStream_t s)
{
    TimingState &t = timing();
    if (!t.on) return;
    TimingState::Rec r{cls, t.get(), t.get(), 0.0, 0.0};
    (void)hipEventRecord(r.a, s);
    t.recs.push_back(r);
}

void timing_end(hipStream_t s)
{
    TimingState &t = timing();
    if (!t.on || t.recs.empty()) return;
    (void)hipEventRecord(t.recs.back().b, s);
}

void timing_work(double work, double executed)
{
    TimingState &t = timing();
    if (!t.on || t.recs.empty()) return;
    t.recs.back().work = work;
    t.recs.back().executed = executed < 0.0 ? work : executed;
}

namespace {

struct Geo {
    int dA, dG, d_core;
    int Ho, Wo;
    int ph, pw;         // padding of the rows / columns of the map
    long R;             // rows of the patch matrix / samples
    bool conv, patches; // patches: the extractor has to run
    bool fused3;        // 3x3/s1/p1 fp32 conv whose A factor is built straight from the NCHW input
    int ld;             // patch leading dimension (elements)
    int esz;
    bool g_rows;        // bf16 output gradients on a map with an odd number of positions: through a row-major copy
    int ldg;            // its leading dimension (elements)
};

bool desc_ok(const kfac_layer_desc *d)
{
    if (!d) return false;
    if (d->kind != KFAC_LINEAR && d->kind != KFAC_CONV2D) return false;
    if (d->in_dtype != KFAC_F32 && d->in_dtype != KFAC_BF16) return false;
    return true;
}

kfac_status desc_check(const kfac_layer_desc *d)
{
    if (!d) return KFAC_ERR_NULL;
    if (!desc_ok(d)) return KFAC_ERR_DTYPE;
    if (d->d_in <= 0 || d->d_out <= 0) return KFAC_ERR_SHAPE;
    if (d->has_bias != 0 && d->has_bias != 1) return KFAC_ERR_SHAPE;
    if (d->kind == KFAC_CONV2D) {
        if (d->kh <= 0 || d->kw <= 0 || d->stride <= 0 || d->pad < 0 || d->pad_h < 0 || d->pad_w < 0)
            return KFAC_ERR_SHAPE;
        if ((long)d->d_in * d->kh * d->kw > (1l << 24)) return KFAC_ERR_SHAPE;
    }
    return KFAC_OK;
}

int core_dim(const kfac_layer_desc *d)
{
    return d->kind == KFAC_CONV2D ? d->d_in * d->kh * d->kw : d->d_in;
}

kfac_status geometry(const kfac_layer_desc *d, int batch, int h, int w, Geo &g)
{
    kfac_status st = desc_check(d);
    if (st != KFAC_OK) return st;
    if (batch <= 0) return KFAC_ERR_SHAPE;
    g.esz = d->in_dtype == KFAC_F32 ? 4 : 2;
    g.d_core = core_dim(d);
    g.dA = g.d_core + d->has_bias;
    g.dG = d->d_out;
    g.conv = d->kind == KFAC_CONV2D;
    const int vec = 16 / g.esz;
    g.ld = (g.d_core + vec - 1) / vec * vec;
    if (g.conv) {
        if (h <= 0 || w <= 0) return KFAC_ERR_SHAPE;
        const int ph = d->pad + d->pad_h, pw = d->pad + d->pad_w;   // rows, columns
        if (h + 2 * ph < d->kh || w + 2 * pw < d->kw) return KFAC_ERR_SHAPE;
        g.ph = ph;
        g.pw = pw;
        g.Ho = (h + 2 * ph - d->kh) / d->stride + 1;
        g.Wo = (w + 2 * pw - d->kw) / d->stride + 1;
        g.R = (long)batch * g.Ho * g.Wo;
        g.patches = !(d->kh == 1 && d->kw == 1 && d->stride == 1 && ph == 0 && pw == 0);
        g.fused3 = tuning().fuse_conv3 && d->in_dtype == KFAC_F32 && d->kh == 3 && d->kw == 3 && d->stride == 1 &&
                   ph == 1 && pw == 1 && d->d_in % 16 == 0 && d->d_in <= tuning().fuse_conv3_max_c && conv3_rows(h, w) > 0 &&
                   (long)batch * d->d_in * h * w * 4 < 0x7fff0000l;
        if (g.fused3) g.patches = false;
        // The bf16 MFMA kernel reads NCHW operands in 4-byte pieces along a channel row, which an odd number of
        // positions per channel (7 x 7 maps) misaligns; the fp32-widening kernel that would take such operands
        // runs at a tenth of its rate.  They are first copied into row-major form instead, [positions, channels],
        // by the patch kernel (a 1 x 1 "extraction" is that transposition): a few MB per layer.
        const bool bf = d->in_dtype == KFAC_BF16;
        if (bf && !g.patches && tuning().bf16_rows_copy && ((long)h * w) % 2 == 1 && d->d_in >= 96) g.patches = true;
        g.g_rows = bf && tuning().bf16_rows_copy && ((long)g.Ho * g.Wo) % 2 == 1 && d->d_out >= 96;
        g.ldg = (d->d_out + 7) / 8 * 8;
        // the patch kernel stages at least one output row of its narrowest channel chunk in LDS: a map too wide for
        // that is refused here, before anything is launched
        if (g.patches && !im2col_fits(d->kh, d->kw, d->stride, g.Wo, g.esz)) return KFAC_ERR_SHAPE;
    } else {
        g.Ho = g.Wo = 1;
        g.R = batch;
        g.patches = false;
        g.fused3 = false;
        g.g_rows = false;
        g.ldg = 0;
    }
    return KFAC_OK;
}

size_t a_patch_bytes(const Geo &g) { return g.patches ? align_up((size_t)g.R * g.ld * g.esz, 256) : 0; }
size_t patch_bytes(const Geo &g)
{
    return a_patch_bytes(g) + (g.g_rows ? align_up((size_t)g.R * g.ldg * g.esz, 256) : 0);
}

bool aligned(const void *p, size_t a) { return ((uintptr_t)p) % a == 0; }

// jobs of one layer; `patches` is where its patch matrix lives (if needed)
void layer_jobs(const kfac_layer_desc *d, const Geo &g, const void *act, const void *gout, int batch, int h,
                int w, float sA, float sG, float decay, float *A_run, float *G_run, void *patches,
                std::vector<Im2colJob> &ij, std::vector<FactorJob> &fj)
{
    FactorJob a{};
    a.dtype = d->in_dtype;
    a.has_bias = d->has_bias;
    a.scale = sA;
    a.decay = decay;
    a.F = A_run;
    a.d_core = g.d_core;
    a.K = g.R;
    if (!g.conv) {
        a.x = act; a.layout = kRows; a.ld = d->d_in; a.hw = 1; a.ctot = d->d_in;
    } else if (g.fused3) {
        a.x = act; a.layout = kConv3; a.ld = 0; a.hw = h * w; a.ctot = d->d_in; a.h = h; a.w = w;
    } else if (!g.patches) {
        a.x = act; a.layout = kNCHW; a.ld = 0; a.hw = h * w; a.ctot = d->d_in;
    } else {
        Im2colJob j{};
        j.x = act; j.out = patches; j.dtype = d->in_dtype;
        j.B = batch; j.C = d->d_in; j.H = h; j.W = w; j.kh = d->kh; j.kw = d->kw;
        j.stride = d->stride; j.pad_h = g.ph; j.pad_w = g.pw; j.Ho = g.Ho; j.Wo = g.Wo; j.ld = g.ld;
        ij.push_back(j);
        a.x = patches; a.layout = kRows; a.ld = g.ld; a.hw = 1; a.ctot = g.d_core;
    }
    fj.push_back(a);

    FactorJob q{};
    q.dtype = d->in_dtype;
    q.has_bias = 0;
    q.scale = sG;
    q.decay = decay;
    q.F = G_run;
    q.d_core = g.dG;
    q.K = g.R;
    q.x = gout;
    if (!g.conv) {
        q.layout = kRows; q.ld = d->d_out; q.hw = 1; q.ctot = d->d_out;
    } else if (g.g_rows) {
        Im2colJob j{};
        j.x = gout; j.out = patches ? static_cast<char *>(patches) + a_patch_bytes(g) : nullptr; j.dtype = d->in_dtype;
        j.B = batch; j.C = d->d_out; j.H = g.Ho; j.W = g.Wo; j.kh = 1; j.kw = 1;
        j.stride = 1; j.pad_h = 0; j.pad_w = 0; j.Ho = g.Ho; j.Wo = g.Wo; j.ld = g.ldg;
        ij.push_back(j);
        q.x = j.out; q.layout = kRows; q.ld = g.ldg; q.hw = 1; q.ctot = d->d_out;
    } else {
        q.layout = kNCHW; q.ld = 0; q.hw = g.Ho * g.Wo; q.ctot = d->d_out;
    }
    fj.push_back(q);
}

// Layers are processed in chunks whose patch matrices fit a byte budget, so
// that a chunk's patches are still in the last-level cache when the SYRK reads
// them.  Layers are independent, so the chunks need not follow the caller's
// order: layers of one shape are kept together (a grouped launch over equal
// problems has no imbalance between its workgroups) and a run of equal layers
// longer than a chunk is cut into equal parts.
struct Chunk { std::vector<int> idx; };

std::vector<Chunk> make_chunks(const std::vector<Geo> &geo, const kfac_layer_desc *descs, const int *batch,
                               const int *h, const int *w)
{
    const int n = (int)geo.size();
    const int cap = kMaxProblems;   // the A and the G factors of conv layers go to different kernels: one table each
    const size_t budget = (size_t)tuning().patch_chunk_bytes;
    auto key = [&](int i) {
        const kfac_layer_desc &d = descs[i];
        return std::make_tuple(geo[i].fused3 ? 0 : 1, d.kind, d.in_dtype, d.d_in, d.d_out, d.kh, d.kw, d.stride,
                               d.pad, d.pad_h, d.pad_w, d.has_bias, batch[i], h ? h[i] : 1, w ? w[i] : 1);
    };
    std::vector<int> order(n);
    for (int i = 0; i < n; ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return key(a) < key(b); });

    std::vector<Chunk> out;
    Chunk cur;
    size_t acc = 0;
    auto flush = [&]() {
        if (!cur.idx.empty()) out.push_back(cur);
        cur.idx.clear();
        acc = 0;
    };
    auto add = [&](int i) {
        const size_t pb = patch_bytes(geo[i]);
        if (!cur.idx.empty() && (acc + pb > budget || (int)cur.idx.size() >= cap)) flush();
        cur.idx.push_back(i);
        acc += pb;
    };
    int r0 = 0;
    while (r0 < n) {
        int r1 = r0;
        while (r1 < n && key(order[r1]) == key(order[r0])) ++r1;
        const int cnt = r1 - r0;
        if (cnt >= 8) {
            // a long run of equal layers gets chunks of its own, cut into equal parts
            flush();
            const size_t pb = patch_bytes(geo[order[r0]]);
            int per = cap;
            if (pb > 0) per = (int)std::max<size_t>(1, std::min<size_t>(cap, budget / pb));
            const int parts = (cnt + per - 1) / per;
            const int each = (cnt + parts - 1) / parts;
            for (int k = 0; k < cnt; ++k) {
                if (k > 0 && k % each == 0) flush();
                cur.idx.push_back(order[r0 + k]);
            }
            flush();
        } else {
            for (int k = r0; k < r1; ++k) add(order[k]);
        }
        r0 = r1;
    }
    flush();
    return out;
}

struct UpdatePlan {
    std::vector<Geo> geo;
    std::vector<Chunk> chunks;
    size_t patch_region = 0, syrk_region = 0;
};

kfac_status plan_update(int n, const kfac_layer_desc *descs, const int *batch, const int *h, const int *w,
                        UpdatePlan &pl)
{
    pl.geo.resize(n);
    for (int i = 0; i < n; ++i) {
        kfac_status st = geometry(&descs[i], batch[i], h ? h[i] : 1, w ? w[i] : 1, pl.geo[i]);
        if (st != KFAC_OK) return st;
    }
    pl.chunks = make_chunks(pl.geo, descs, batch, h, w);
    for (const Chunk &c : pl.chunks) {
        size_t pb = 0;
        std::vector<Im2colJob> ij;
        std::vector<FactorJob> fj;
        for (int i : c.idx) {
            // placeholder pointers: only shapes matter for the workspace plan (but alignment
            // decides nothing about sizes)
            layer_jobs(&descs[i], pl.geo[i], nullptr, nullptr, batch[i], h ? h[i] : 1, w ? w[i] : 1, 1.f, 1.f,
                       0.f, nullptr, nullptr, nullptr, ij, fj);
            pb += patch_bytes(pl.geo[i]);
        }
        pl.patch_region = std::max(pl.patch_region, pb);
        pl.syrk_region = std::max(pl.syrk_region, syrk_workspace_bytes(fj.data(), (int)fj.size()));
    }
    return KFAC_OK;
}

size_t invert_ws(int n, const kfac_layer_desc *descs)
{
    std::vector<InvertJob> jobs;
    for (int i = 0; i < n; ++i) {
        InvertJob a{}; a.n = core_dim(&descs[i]) + descs[i].has_bias; jobs.push_back(a);
        InvertJob g{}; g.n = descs[i].d_out; jobs.push_back(g);
    }
    return invert_workspace_bytes(jobs.data(), (int)jobs.size());
}

// the inversion workspace is followed by the 2n device-side damping terms of kfac_invert_pi
size_t invert_ws_total(int n, const kfac_layer_desc *descs)
{
    return align_up(invert_ws(n, descs), 256) + align_up((size_t)2 * n * sizeof(float), 256);
}

// the intermediates U^T [d_A, d_G] of kfac_precondition_batched, one per layer
size_t precond_ws_min(int n, const kfac_layer_desc *descs)
{
    size_t total = 0;
    for (int i = 0; i < n; ++i) {
        const size_t dA = core_dim(&descs[i]) + descs[i].has_bias, dG = descs[i].d_out;
        total += align_up(dA * dG * sizeof(float), 256);
    }
    return total;
}

// the two products of layer i: U^T = grad^T G_inv, P = (U^T)^T A_inv (pointers may be null: shapes only)
void precond_jobs(const kfac_layer_desc &d, const float *A_inv, const float *G_inv, const float *grad, float *out,
                  float *Ut, GemmJob &a, GemmJob &b)
{
    const int dA = core_dim(&d) + d.has_bias, dG = d.d_out;
    // U^T[dA, dG] = grad^T G_inv  (G_inv symmetric): A = grad, B = G_inv, both K-major over d_G
    a = GemmJob{};
    a.A = grad; a.B = G_inv; a.C = Ut;
    a.M = dA; a.N = dG; a.K = dG; a.lda = dA; a.ldb = dG; a.ldc = dG; a.mode = kStore; a.p0 = a.p1 = 0;
    // P[dG, dA] = (U^T)^T A_inv
    b = GemmJob{};
    b.A = Ut; b.B = A_inv; b.C = out;
    b.M = dG; b.N = dA; b.K = dA; b.lda = dG; b.ldb = dA; b.ldc = dA; b.mode = kStore; b.p0 = b.p1 = 0;
}

// ... plus room for the K-slice partials of the deeper of the two groups of products
size_t precond_ws(int n, const kfac_layer_desc *descs)
{
    std::vector<GemmJob> g1(n), g2(n);
    for (int i = 0; i < n; ++i) precond_jobs(descs[i], nullptr, nullptr, nullptr, nullptr, nullptr, g1[i], g2[i]);
    return precond_ws_min(n, descs) + align_up(std::max(gemm_workspace_bytes(g1.data(), n),
                                                        gemm_workspace_bytes(g2.data(), n)), 256);
}

std::vector<EigenJob> eigen_jobs(int n, const kfac_layer_desc *descs, const float *const *A, const float *const *G,
                                 float *const *QA, float *const *vA, float *const *QG, float *const *vG, int *info)
{
    std::vector<EigenJob> jobs;
    for (int i = 0; i < n; ++i) {
        EigenJob a{};
        a.n = core_dim(&descs[i]) + descs[i].has_bias;
        EigenJob g{};
        g.n = descs[i].d_out;
        if (A) {
            a.M = A[i]; a.Q = QA[i]; a.v = vA[i]; a.info = info + 2 * i;
            g.M = G[i]; g.Q = QG[i]; g.v = vG[i]; g.info = info + 2 * i + 1;
        }
        jobs.push_back(a);
        jobs.push_back(g);
    }
    return jobs;
}

size_t eigen_ws(int n, const kfac_layer_desc *descs)
{
    std::vector<EigenJob> jobs = eigen_jobs(n, descs, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr);
    return eigen_workspace_bytes(jobs.data(), (int)jobs.size());
}

// Eq. 13 workspace per layer: two d_A x d_G intermediates and the transposes of Q_A and Q_G
size_t precond_eigen_ws(int n, const kfac_layer_desc *descs)
{
    size_t total = 0;
    for (int i = 0; i < n; ++i) {
        const size_t dA = core_dim(&descs[i]) + descs[i].has_bias, dG = descs[i].d_out;
        total += 2 * align_up(dA * dG * sizeof(float), 256) + align_up(dA * dA * sizeof(float), 256) +
                 align_up(dG * dG * sizeof(float), 256);
    }
    return total;
}

}  // namespace
}  // namespace kfac

using namespace kfac;

extern "C" {

int kfac_dim_A(const kfac_layer_desc *d)
{
    if (desc_check(d) != KFAC_OK) return -1;
    return core_dim(d) + d->has_bias;
}

int kfac_dim_G(const kfac_layer_desc *d)
{
    if (desc_check(d) != KFAC_OK) return -1;
    return d->d_out;
}

int kfac_patch_ld(const kfac_layer_desc *d)
{
    if (desc_check(d) != KFAC_OK) return -1;
    const int vec = d->in_dtype == KFAC_F32 ? 4 : 8;
    return (core_dim(d) + vec - 1) / vec * vec;
}

size_t kfac_workspace_bytes_batched(int n, const kfac_layer_desc *descs, const int *batch, const int *h,
                                    const int *w)
{
    if (n <= 0 || !descs || !batch) return 0;
    UpdatePlan pl;
    if (plan_update(n, descs, batch, h, w, pl) != KFAC_OK) return 0;
    size_t need = pl.patch_region + pl.syrk_region;
    need = std::max(need, invert_ws_total(n, descs));
    need = std::max(need, precond_ws(n, descs));
    need = std::max(need, eigen_ws(n, descs));
    need = std::max(need, precond_eigen_ws(n, descs));
    return need + 256;
}

size_t kfac_workspace_bytes(const kfac_layer_desc *d, int batch, int h, int w)
{
    return kfac_workspace_bytes_batched(1, d, &batch, &h, &w);
}

kfac_status kfac_im2col(const kfac_layer_desc *d, const void *d_act, int batch, int h, int w, void *d_patches,
                        void *hip_stream)
{
    Geo g;
    kfac_status st = geometry(d, batch, h, w, g);
    if (st != KFAC_OK) return st;
    if (!g.conv) return KFAC_ERR_SHAPE;
    if (!d_act || !d_patches) return KFAC_ERR_NULL;
    if (!aligned(d_act, 16) || !aligned(d_patches, 16)) return KFAC_ERR_ALIGN;
    Im2colJob j{};
    j.x = d_act; j.out = d_patches; j.dtype = d->in_dtype;
    j.B = batch; j.C = d->d_in; j.H = h; j.W = w; j.kh = d->kh; j.kw = d->kw;
    j.stride = d->stride; j.pad_h = g.ph; j.pad_w = g.pw; j.Ho = g.Ho; j.Wo = g.Wo; j.ld = g.ld;
    return im2col_launch(&j, 1, (hipStream_t)hip_stream) == hipSuccess ? KFAC_OK : KFAC_ERR_HIP;
}

kfac_status kfac_update_factors_batched(int n, const kfac_layer_desc *descs, const void *const *d_act,
                                        const void *const *d_gout, const int *batch, const int *h,
                                        const int *w, const float *scale_A, const float *scale_G, float decay,
                                        float *const *d_A_run, float *const *d_G_run, void *d_work,
                                        size_t work_bytes, void *hip_stream)
{
    if (n <= 0) return KFAC_ERR_SHAPE;
    if (!descs || !d_act || !d_gout || !batch || !scale_A || !scale_G || !d_A_run || !d_G_run)
        return KFAC_ERR_NULL;
    if (!(decay >= 0.f && decay <= 1.f)) return KFAC_ERR_PARAM;
    UpdatePlan pl;
    kfac_status st = plan_update(n, descs, batch, h, w, pl);
    if (st != KFAC_OK) return st;
    for (int i = 0; i < n; ++i) {
        if (!d_act[i] || !d_gout[i] || !d_A_run[i] || !d_G_run[i]) return KFAC_ERR_NULL;
        if (!(scale_A[i] > 0.f) || !(scale_G[i] > 0.f)) return KFAC_ERR_PARAM;
        if (descs[i].kind == KFAC_CONV2D && (!h || !w)) return KFAC_ERR_NULL;
        if (!aligned(d_act[i], 16) || !aligned(d_gout[i], 16) ||
            !aligned(d_A_run[i], 4) || !aligned(d_G_run[i], 4))
            return KFAC_ERR_ALIGN;
    }
    const size_t need = pl.patch_region + pl.syrk_region;
    if (need > 0 && !d_work) return KFAC_ERR_NULL;
    if (work_bytes < need || !aligned(d_work, 256)) return d_work && !aligned(d_work, 256) ? KFAC_ERR_ALIGN
                                                                                           : KFAC_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)hip_stream;
    char *patch_base = static_cast<char *>(d_work);
    char *syrk_base = patch_base + pl.patch_region;
    for (const Chunk &c : pl.chunks) {
        std::vector<Im2colJob> ij;
        std::vector<FactorJob> fj;
        size_t poff = 0;
        for (int i : c.idx) {
            layer_jobs(&descs[i], pl.geo[i], d_act[i], d_gout[i], batch[i], h ? h[i] : 1, w ? w[i] : 1,
                       scale_A[i], scale_G[i], decay, d_A_run[i], d_G_run[i], patch_base + poff, ij, fj);
            poff += patch_bytes(pl.geo[i]);
        }
        if (!ij.empty() && im2col_launch(ij.data(), (int)ij.size(), s) != hipSuccess) return KFAC_ERR_HIP;
        if (syrk_launch(fj.data(), (int)fj.size(), syrk_base, pl.syrk_region, s) != hipSuccess)
            return KFAC_ERR_HIP;
    }
    return KFAC_OK;
}

kfac_status kfac_update_factors(const kfac_layer_desc *d, const void *d_act, const void *d_gout, int batch, int h,
                                int w, float scale_A, float scale_G, float decay, float *d_A_run,
                                float *d_G_run, void *d_work, size_t work_bytes, void *hip_stream)
{
    if (!d) return KFAC_ERR_NULL;
    return kfac_update_factors_batched(1, d, &d_act, &d_gout, &batch, &h, &w, &scale_A, &scale_G, decay,
                                       &d_A_run, &d_G_run, d_work, work_bytes, hip_stream);
}

kfac_status kfac_invert_batched(int n, const kfac_layer_desc *descs, const float *const *d_A_run,
                                const float *const *d_G_run, float damping_A, float damping_G,
                                float *const *d_A_inv, float *const *d_G_inv, int *d_info, void *d_work,
                                size_t work_bytes, void *hip_stream)
{
    if (n <= 0) return KFAC_ERR_SHAPE;
    if (!descs || !d_A_run || !d_G_run || !d_A_inv || !d_G_inv || !d_info || !d_work) return KFAC_ERR_NULL;
    if (!(damping_A >= 0.f) || !(damping_G >= 0.f)) return KFAC_ERR_PARAM;
    std::vector<InvertJob> jobs;
    for (int i = 0; i < n; ++i) {
        kfac_status st = desc_check(&descs[i]);
        if (st != KFAC_OK) return st;
        if (!d_A_run[i] || !d_G_run[i] || !d_A_inv[i] || !d_G_inv[i]) return KFAC_ERR_NULL;
        if (!aligned(d_A_run[i], 4) || !aligned(d_G_run[i], 4) || !aligned(d_A_inv[i], 4) ||
            !aligned(d_G_inv[i], 4))
            return KFAC_ERR_ALIGN;
        if (d_A_run[i] == d_A_inv[i] || d_G_run[i] == d_G_inv[i]) return KFAC_ERR_PARAM;
        InvertJob a{};
        a.M = d_A_run[i]; a.Minv = d_A_inv[i]; a.n = core_dim(&descs[i]) + descs[i].has_bias;
        a.damping = damping_A; a.info = d_info + 2 * i;
        jobs.push_back(a);
        InvertJob g{};
        g.M = d_G_run[i]; g.Minv = d_G_inv[i]; g.n = descs[i].d_out;
        g.damping = damping_G; g.info = d_info + 2 * i + 1;
        jobs.push_back(g);
    }
    if (!aligned(d_work, 256)) return KFAC_ERR_ALIGN;
    if (invert_workspace_bytes(jobs.data(), (int)jobs.size()) > work_bytes) return KFAC_ERR_WORKSPACE;
    return invert_launch(jobs.data(), (int)jobs.size(), d_work, work_bytes, (hipStream_t)hip_stream) == hipSuccess
               ? KFAC_OK
               : KFAC_ERR_HIP;
}

kfac_status kfac_invert_pi_batched(int n, const kfac_layer_desc *descs, const float *const *d_A_run,
                                   const float *const *d_G_run, float gamma, float *const *d_A_inv,
                                   float *const *d_G_inv, int *d_info, float *d_damping, void *d_work,
                                   size_t work_bytes, void *hip_stream)
{
    if (n <= 0) return KFAC_ERR_SHAPE;
    if (!descs || !d_A_run || !d_G_run || !d_A_inv || !d_G_inv || !d_info || !d_work) return KFAC_ERR_NULL;
    if (!(gamma >= 0.f)) return KFAC_ERR_PARAM;
    if (d_damping && !aligned(d_damping, 4)) return KFAC_ERR_ALIGN;
    if (!aligned(d_work, 256)) return KFAC_ERR_ALIGN;
    for (int i = 0; i < n; ++i) {
        kfac_status st = desc_check(&descs[i]);
        if (st != KFAC_OK) return st;
        if (!d_A_run[i] || !d_G_run[i] || !d_A_inv[i] || !d_G_inv[i]) return KFAC_ERR_NULL;
        if (!aligned(d_A_run[i], 4) || !aligned(d_G_run[i], 4) || !aligned(d_A_inv[i], 4) ||
            !aligned(d_G_inv[i], 4))
            return KFAC_ERR_ALIGN;
        if (d_A_run[i] == d_A_inv[i] || d_G_run[i] == d_G_inv[i]) return KFAC_ERR_PARAM;
    }
    if (invert_ws_total(n, descs) > work_bytes) return KFAC_ERR_WORKSPACE;
    const size_t inv_bytes = align_up(invert_ws(n, descs), 256);
    float *lam = d_damping ? d_damping : reinterpret_cast<float *>(static_cast<char *>(d_work) + inv_bytes);
    std::vector<InvertJob> jobs;
    std::vector<int> dA(n), dG(n);
    for (int i = 0; i < n; ++i) {
        dA[i] = core_dim(&descs[i]) + descs[i].has_bias;
        dG[i] = descs[i].d_out;
        InvertJob a{};
        a.M = d_A_run[i]; a.Minv = d_A_inv[i]; a.n = dA[i]; a.damping = 0.f; a.damping_dev = lam + 2 * i;
        a.info = d_info + 2 * i;
        jobs.push_back(a);
        InvertJob g{};
        g.M = d_G_run[i]; g.Minv = d_G_inv[i]; g.n = dG[i]; g.damping = 0.f; g.damping_dev = lam + 2 * i + 1;
        g.info = d_info + 2 * i + 1;
        jobs.push_back(g);
    }
    hipStream_t s = (hipStream_t)hip_stream;
    if (pi_damping_launch(d_A_run, d_G_run, dA.data(), dG.data(), n, gamma, lam, s) != hipSuccess)
        return KFAC_ERR_HIP;
    return invert_launch(jobs.data(), (int)jobs.size(), d_work, inv_bytes, s) == hipSuccess ? KFAC_OK : KFAC_ERR_HIP;
}

kfac_status kfac_invert_pi(const kfac_layer_desc *d, const float *d_A_run, const float *d_G_run, float gamma,
                           float *d_A_inv, float *d_G_inv, int *d_info, float *d_damping, void *d_work,
                           size_t work_bytes, void *hip_stream)
{
    if (!d) return KFAC_ERR_NULL;
    return kfac_invert_pi_batched(1, d, &d_A_run, &d_G_run, gamma, &d_A_inv, &d_G_inv, d_info, d_damping, d_work,
                                  work_bytes, hip_stream);
}

kfac_status kfac_invert(const kfac_layer_desc *d, const float *d_A_run, const float *d_G_run, float damping_A,
                        float damping_G, float *d_A_inv, float *d_G_inv, int *d_info, void *d_work,
                        size_t work_bytes, void *hip_stream)
{
    if (!d) return KFAC_ERR_NULL;
    return kfac_invert_batched(1, d, &d_A_run, &d_G_run, damping_A, damping_G, &d_A_inv, &d_G_inv, d_info,
                               d_work, work_bytes, hip_stream);
}

kfac_status kfac_precondition_batched(int n, const kfac_layer_desc *descs, const float *const *d_A_inv,
                                      const float *const *d_G_inv, const float *const *d_grad,
                                      float *const *d_out, void *d_work, size_t work_bytes, void *hip_stream)
{
    if (n <= 0) return KFAC_ERR_SHAPE;
    if (!descs || !d_A_inv || !d_G_inv || !d_grad || !d_out || !d_work) return KFAC_ERR_NULL;
    for (int i = 0; i < n; ++i) {
        kfac_status st = desc_check(&descs[i]);
        if (st != KFAC_OK) return st;
        if (!d_A_inv[i] || !d_G_inv[i] || !d_grad[i] || !d_out[i]) return KFAC_ERR_NULL;
        if (!aligned(d_A_inv[i], 4) || !aligned(d_G_inv[i], 4) || !aligned(d_grad[i], 4) || !aligned(d_out[i], 4))
            return KFAC_ERR_ALIGN;
    }
    if (!aligned(d_work, 256)) return KFAC_ERR_ALIGN;
    // the intermediates are required; the K-slice partials behind them are used when there is room for them
    if (precond_ws_min(n, descs) > work_bytes) return KFAC_ERR_WORKSPACE;
    std::vector<GemmJob> g1(n), g2(n);
    size_t off = 0;
    for (int i = 0; i < n; ++i) {
        const size_t dA = (size_t)core_dim(&descs[i]) + descs[i].has_bias, dG = descs[i].d_out;
        float *Ut = reinterpret_cast<float *>(static_cast<char *>(d_work) + off);
        off += align_up(dA * dG * sizeof(float), 256);
        precond_jobs(descs[i], d_A_inv[i], d_G_inv[i], d_grad[i], d_out[i], Ut, g1[i], g2[i]);
    }
    void *slices = static_cast<char *>(d_work) + off;
    const size_t slice_bytes = work_bytes - off;
    hipStream_t s = (hipStream_t)hip_stream;
    if (gemm_launch(g1.data(), n, s, slices, slice_bytes) != hipSuccess) return KFAC_ERR_HIP;
    if (gemm_launch(g2.data(), n, s, slices, slice_bytes) != hipSuccess) return KFAC_ERR_HIP;
    return KFAC_OK;
}

kfac_status kfac_precondition(const kfac_layer_desc *d, const float *d_A_inv, const float *d_G_inv,
                              const float *d_grad, float *d_out, void *d_work, size_t work_bytes,
                              void *hip_stream)
{
    if (!d) return KFAC_ERR_NULL;
    return kfac_precondition_batched(1, d, &d_A_inv, &d_G_inv, &d_grad, &d_out, d_work, work_bytes, hip_stream);
}

kfac_status kfac_eigen_batched(int n, const kfac_layer_desc *descs, const float *const *d_A_run,
                               const float *const *d_G_run, float *const *d_Q_A, float *const *d_v_A,
                               float *const *d_Q_G, float *const *d_v_G, int *d_info, void *d_work,
                               size_t work_bytes, void *hip_stream)
{
    if (n <= 0) return KFAC_ERR_SHAPE;
    if (!descs || !d_A_run || !d_G_run || !d_Q_A || !d_v_A || !d_Q_G || !d_v_G || !d_info || !d_work)
        return KFAC_ERR_NULL;
    for (int i = 0; i < n; ++i) {
        kfac_status st = desc_check(&descs[i]);
        if (st != KFAC_OK) return st;
        if (!d_A_run[i] || !d_G_run[i] || !d_Q_A[i] || !d_v_A[i] || !d_Q_G[i] || !d_v_G[i]) return KFAC_ERR_NULL;
        if (!aligned(d_A_run[i], 4) || !aligned(d_G_run[i], 4) || !aligned(d_Q_A[i], 4) || !aligned(d_v_A[i], 4) ||
            !aligned(d_Q_G[i], 4) || !aligned(d_v_G[i], 4))
            return KFAC_ERR_ALIGN;
        if (d_A_run[i] == d_Q_A[i] || d_G_run[i] == d_Q_G[i]) return KFAC_ERR_PARAM;
    }
    if (!aligned(d_work, 256)) return KFAC_ERR_ALIGN;
    std::vector<EigenJob> jobs = eigen_jobs(n, descs, d_A_run, d_G_run, d_Q_A, d_v_A, d_Q_G, d_v_G, d_info);
    if (eigen_workspace_bytes(jobs.data(), (int)jobs.size()) > work_bytes) return KFAC_ERR_WORKSPACE;
    return eigen_launch(jobs.data(), (int)jobs.size(), d_work, work_bytes, (hipStream_t)hip_stream) == hipSuccess
               ? KFAC_OK
               : KFAC_ERR_HIP;
}

kfac_status kfac_eigen(const kfac_layer_desc *d, const float *d_A_run, const float *d_G_run, float *d_Q_A,
                       float *d_v_A, float *d_Q_G, float *d_v_G, int *d_info, void *d_work, size_t work_bytes,
                       void *hip_stream)
{
    if (!d) return KFAC_ERR_NULL;
    return kfac_eigen_batched(1, d, &d_A_run, &d_G_run, &d_Q_A, &d_v_A, &d_Q_G, &d_v_G, d_info, d_work, work_bytes,
                              hip_stream);
}

kfac_status kfac_precondition_eigen_batched(int n, const kfac_layer_desc *descs, const float *const *d_Q_A,
                                            const float *const *d_v_A, const float *const *d_Q_G,
                                            const float *const *d_v_G, float gamma, const float *const *d_grad,
                                            float *const *d_out, void *d_work, size_t work_bytes,
                                            void *hip_stream)
{
    if (n <= 0) return KFAC_ERR_SHAPE;
    if (!descs || !d_Q_A || !d_v_A || !d_Q_G || !d_v_G || !d_grad || !d_out || !d_work) return KFAC_ERR_NULL;
    if (!(gamma >= 0.f)) return KFAC_ERR_PARAM;
    for (int i = 0; i < n; ++i) {
        kfac_status st = desc_check(&descs[i]);
        if (st != KFAC_OK) return st;
        if (!d_Q_A[i] || !d_v_A[i] || !d_Q_G[i] || !d_v_G[i] || !d_grad[i] || !d_out[i]) return KFAC_ERR_NULL;
        if (!aligned(d_Q_A[i], 4) || !aligned(d_v_A[i], 4) || !aligned(d_Q_G[i], 4) || !aligned(d_v_G[i], 4) ||
            !aligned(d_grad[i], 4) || !aligned(d_out[i], 4))
            return KFAC_ERR_ALIGN;
    }
    if (!aligned(d_work, 256)) return KFAC_ERR_ALIGN;
    if (precond_eigen_ws(n, descs) > work_bytes) return KFAC_ERR_WORKSPACE;
    // With Q = [eigenvectors in columns] and every product in the form C = X^T Y (both operands K-major):
    //   U   [dA, dG] = grad^T Q_G                      (= (Q_G^T grad)^T)
    //   T1  [dG, dA] = U^T Q_A  ./ (v_G v_A^T + gamma)   (division in the epilogue)
    //   T2t [dA, dG] = T1^T Q_G^T                      (= (Q_G T1)^T)
    //   P   [dG, dA] = T2t^T Q_A^T
    std::vector<GemmJob> g1(n), g2(n), g3(n), g4(n);
    std::vector<const float *> tsrc;
    std::vector<float *> tdst;
    std::vector<int> tn;
    size_t off = 0;
    auto take = [&](size_t floats) {
        float *p = reinterpret_cast<float *>(static_cast<char *>(d_work) + off);
        off += align_up(floats * sizeof(float), 256);
        return p;
    };
    for (int i = 0; i < n; ++i) {
        const int dA = core_dim(&descs[i]) + descs[i].has_bias, dG = descs[i].d_out;
        float *U = take((size_t)dA * dG), *T1 = take((size_t)dA * dG);
        float *QAt = take((size_t)dA * dA), *QGt = take((size_t)dG * dG);
        tsrc.push_back(d_Q_A[i]); tdst.push_back(QAt); tn.push_back(dA);
        tsrc.push_back(d_Q_G[i]); tdst.push_back(QGt); tn.push_back(dG);
        GemmJob &a = g1[i];
        a.A = d_grad[i]; a.B = d_Q_G[i]; a.C = U;
        a.M = dA; a.N = dG; a.K = dG; a.lda = dA; a.ldb = dG; a.ldc = dG; a.mode = kStore; a.p0 = a.p1 = 0;
        GemmJob &b = g2[i];
        b.A = U; b.B = d_Q_A[i]; b.C = T1;
        b.M = dG; b.N = dA; b.K = dA; b.lda = dG; b.ldb = dA; b.ldc = dA; b.mode = kStoreDiv; b.p0 = b.p1 = 0;
        b.rv = d_v_G[i]; b.cv = d_v_A[i]; b.gamma = gamma;
        GemmJob &c = g3[i];
        c.A = T1; c.B = QGt; c.C = U;
        c.M = dA; c.N = dG; c.K = dG; c.lda = dA; c.ldb = dG; c.ldc = dG; c.mode = kStore; c.p0 = c.p1 = 0;
        GemmJob &e = g4[i];
        e.A = U; e.B = QAt; e.C = d_out[i];
        e.M = dG; e.N = dA; e.K = dA; e.lda = dG; e.ldb = dA; e.ldc = dA; e.mode = kStore; e.p0 = e.p1 = 0;
    }
    hipStream_t s = (hipStream_t)hip_stream;
    if (transpose_launch(tsrc.data(), tdst.data(), tn.data(), (int)tn.size(), s) != hipSuccess) return KFAC_ERR_HIP;
    if (gemm_launch(g1.data(), n, s) != hipSuccess) return KFAC_ERR_HIP;
    if (gemm_launch(g2.data(), n, s) != hipSuccess) return KFAC_ERR_HIP;
    if (gemm_launch(g3.data(), n, s) != hipSuccess) return KFAC_ERR_HIP;
    if (gemm_launch(g4.data(), n, s) != hipSuccess) return KFAC_ERR_HIP;
    return KFAC_OK;
}

kfac_status kfac_precondition_eigen(const kfac_layer_desc *d, const float *d_Q_A, const float *d_v_A,
                                    const float *d_Q_G, const float *d_v_G, float gamma, const float *d_grad,
                                    float *d_out, void *d_work, size_t work_bytes, void *hip_stream)
{
    if (!d) return KFAC_ERR_NULL;
    return kfac_precondition_eigen_batched(1, d, &d_Q_A, &d_v_A, &d_Q_G, &d_v_G, gamma, &d_grad, &d_out, d_work,
                                           work_bytes, hip_stream);
}

// Device address of `scratch` on the current device, looked up once per device.
static kfac_status static_scratch_ptr(void **out)
{
    static std::mutex mu;
    static void *per_dev[64] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return KFAC_ERR_HIP;
    std::lock_guard<std::mutex> lock(mu);
    if (!per_dev[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return KFAC_ERR_HIP;
        per_dev[dev] = p;
    }
    *out = per_dev[dev];
    return KFAC_OK;
}

kfac_status kfac_precondition_static(const kfac_layer_desc *d, const float *d_A_inv, const float *d_G_inv,
                                     const float *d_grad, float *d_out, void *hip_stream)
{
    kfac_status st = desc_check(d);
    if (st != KFAC_OK) return st;
    const size_t dA = (size_t)core_dim(d) + d->has_bias, dG = (size_t)d->d_out;
    if (dA * dG * sizeof(float) > (size_t)KFAC_STATIC_SCRATCH_BYTES) return KFAC_ERR_TOO_LARGE;
    void *ptr = nullptr;
    st = static_scratch_ptr(&ptr);
    if (st != KFAC_OK) return st;
    // the intermediate U^T [d_A, d_G] is written in full by the first product before the second reads it:
    // nothing in the buffer has to start at zero
    // (the size passed is that of the intermediate alone: no K-slice partials, every product in one piece)
    return kfac_precondition_batched(1, d, &d_A_inv, &d_G_inv, &d_grad, &d_out, ptr,
                                     align_up(dA * dG * sizeof(float), 256), hip_stream);
}

const char *kfac_status_string(kfac_status s)
{
    switch (s) {
        case KFAC_OK: return "ok";
        case KFAC_ERR_NULL: return "null pointer";
        case KFAC_ERR_SHAPE: return "bad shape";
        case KFAC_ERR_DTYPE: return "bad dtype or layer kind";
        case KFAC_ERR_WORKSPACE: return "workspace too small";
        case KFAC_ERR_PARAM: return "bad parameter";
        case KFAC_ERR_HIP: return "HIP launch failed";
        case KFAC_ERR_ALIGN: return "misaligned pointer";
        case KFAC_ERR_TOO_LARGE: return "problem exceeds the library's static scratch buffer";
    }
    return "unknown status";
}

int kfac_version(void) { return 100; }

int kfac_timing_enable(int on)
{
    timing().on = on != 0;
    return 0;
}

int kfac_timing_collect_ex(double *ms, long *launches, double *work, double *executed)
{
    auto &t = timing();
    int rc = 0;
    for (auto &r : t.recs) {
        float e = 0.f;
        if (hipEventSynchronize(r.b) != hipSuccess || hipEventElapsedTime(&e, r.a, r.b) != hipSuccess) rc = 1;
        if (ms) ms[r.cls] += e;
        if (launches) launches[r.cls] += 1;
        if (work) work[r.cls] += r.work;
        if (executed) executed[r.cls] += r.executed;
        t.pool.push_back(r.a);
        t.pool.push_back(r.b);
    }
    t.recs.clear();
    return rc;
}

int kfac_timing_collect(double *ms, long *launches, double *work)
{
    return kfac_timing_collect_ex(ms, launches, work, nullptr);
}

const char *kfac_timing_class_name(int cls)
{
    static const char *names[KFAC_K_COUNT] = {"im2col", "syrk_partial", "syrk_reduce", "inv_init",
                                              "inv_pivot", "inv_panel", "inv_finish", "gemm_tn",
                                              "syrk_wave", "syrk_conv3", "syrk_small", "inv_step",
                                              "syrk_bf16", "gemm_wave", "eig_init", "eig_round", "eig_final",
                                              "syrk_corr3", "corr3_assemble", "gemm_split", "syrk_split"};
    return (cls >= 0 && cls < KFAC_K_COUNT) ? names[cls] : "?";
}

namespace {
__global__ __launch_bounds__(256) void calib_copy_kernel(float4 *__restrict__ dst, const float4 *__restrict__ src, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}
}  // namespace

int kfac_profile_copy(void *d_dst, const void *d_src, size_t bytes, void *hip_stream)
{
    if (!d_dst || !d_src || bytes == 0 || bytes % 16 || (reinterpret_cast<uintptr_t>(d_dst) & 15) ||
        (reinterpret_cast<uintptr_t>(d_src) & 15))
        return 1;
    const size_t n = bytes / 16;
    const int blocks = (int)std::min<size_t>((n + 255) / 256, 256 * 16);
    hipLaunchKernelGGL(calib_copy_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<float4 *>(d_dst), static_cast<const float4 *>(d_src), n);
    return hipGetLastError() == hipSuccess ? 0 : 2;
}

int kfac_profile_gemm(const float *d_A, const float *d_B, float *d_C, int M, int N, int K, long lda, long ldb,
                      long ldc, int mode, int p0, int p1, void *hip_stream)
{
    if (!d_A || !d_B || !d_C || M <= 0 || N <= 0 || K <= 0 || lda < M || ldb < N || ldc < N) return 1;
    if (mode != kStore && mode != kSubLowerSkip) return 1;
    if (mode == kSubLowerSkip && (M != N || p0 < 0 || p1 < p0)) return 1;
    GemmJob j{};
    j.A = d_A; j.B = d_B; j.C = d_C; j.M = M; j.N = N; j.K = K; j.lda = lda; j.ldb = ldb; j.ldc = ldc;
    j.mode = mode; j.p0 = p0; j.p1 = p1;
    return gemm_launch(&j, 1, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? 0 : 2;
}

/* Development knob: returns 0 when the key is known. */
int kfac_tune(const char *key, long value)
{
    Tuning &t = tuning();
    const std::string k(key ? key : "");
    if (k == "target_blocks") t.target_blocks = value;
    else if (k == "tile_max_splits") t.tile_max_splits = value < 1 ? 1 : value;
    else if (k == "small_blocks_x") t.small_blocks_x = value < 1 ? 1 : value;
    else if (k == "min_tiles_per_split") t.min_tiles_per_split = value;
    else if (k == "patch_chunk_bytes") t.patch_chunk_bytes = value;
    else if (k == "syrk_force_bm") t.syrk_force_bm = value;
    else if (k == "use_wave_kernel") t.use_wave_kernel = value;
#ifdef KFAC_MEASUREMENT_KNOBS
    // skips MFMAs or loads inside the wave kernels (wrong results): only in builds made for measuring
    else if (k == "wave_debug") t.wave_debug = value;
#endif
    else if (k == "fuse_conv3") t.fuse_conv3 = value;
    else if (k == "fuse_conv3_max_c") t.fuse_conv3_max_c = value;
    else if (k == "split_gemm_min_k") t.split_gemm_min_k = value;
    else if (k == "gemm_kslice_stages") t.gemm_kslice_stages = value;
    else if (k == "invert_border_refine") t.invert_border_refine = value;
    else if (k == "update_bm") t.update_bm = value;
    else if (k == "use_small_kernel") t.use_small_kernel = value;
    else if (k == "invert_fused_max_n") t.invert_fused_max_n = value;
    else if (k == "use_corr3") t.use_corr3 = value;
    else if (k == "corr3_lds_kb") t.corr3_lds_kb = value;
    else if (k == "invert_border") t.invert_border = value;
    else if (k == "invert_two_streams") t.invert_two_streams = value;
    else if (k == "invert_outer_block") t.invert_outer_block = value;
    else if (k == "invert_refine") t.invert_refine = value;
    else if (k == "bf16_rows_copy") t.bf16_rows_copy = value;
    else if (k == "invert_panel_split") t.invert_panel_split = value;
    else if (k == "invert_refine_cond") t.invert_refine_cond = value < 0 ? 0 : value;
    else if (k == "invert_fused_refine_cond") t.invert_fused_refine_cond = value < 0 ? 0 : value;
    else if (k == "eigen_max_sweeps") t.eigen_max_sweeps = value;
    else if (k == "eigen_inner_sweeps") t.eigen_inner_sweeps = value;
    else if (k == "im2col_piece_elems") t.im2col_piece_elems = value;
    else if (k == "im2col_block_bytes") t.im2col_block_bytes = value;
    else if (k == "im2col_lds_bytes") t.im2col_lds_bytes = value;
    else if (k == "im2col_min_blocks") t.im2col_min_blocks = value;
    else if (k == "use_bf16_mfma") t.use_bf16_mfma = value;
    else if (k == "use_wave_gemm") t.use_wave_gemm = value;
    else if (k == "use_split_gemm") t.use_split_gemm = value;
    else if (k == "use_split_syrk") t.use_split_syrk = value;
    else if (k == "split_syrk_fill_rows") t.split_syrk_fill_rows = value;
    else if (k == "split_syrk_min_d") t.split_syrk_min_d = value < 64 ? 64 : value;
    else if (k == "split_syrk_max_stages") t.split_syrk_max_stages = value < 1 ? 1 : value;
    else if (k == "split_syrk_fill_nchw") t.split_syrk_fill_nchw = value;
    else if (k == "split_gemm_min_m") t.split_gemm_min_m = value;
    else if (k == "split_gemm_min_fill") t.split_gemm_min_fill = value;
    else if (k == "gemm_xcd_remap_min") t.gemm_xcd_remap_min = value;
    else if (k == "gemm_bm") t.gemm_bm = value;
    else return 1;
    return 0;
}

}  // extern "C"

// Joint layout / kernel-variant tuning (Section 5.2 of the paper, cut down to
// what a finite set of compiled kernels needs): for each layout candidate the
// best latency over kernel variants is that layout's reward; the search is
// staged as in the paper — a joint stage that spends part of the measurement
// budget across all layouts (variants tried best-estimate first), then a
// loop-only stage on the winning layout.  Every trial is an on-device
// measurement; the budget counts measurements (Section 6).  Also the tune
// cache and the chain planner.
#include <algorithm>
#include <chrono>
#include <cmath>
#include <fstream>
#include <sstream>

#include "ops.h"

namespace alt {

std::string conv_key(alt_handle_t h, const alt_conv_desc_t *d)
{
    std::ostringstream o;
    o << "conv|" << h->arch << "|" << d->N << "," << d->C << "," << d->H << "," << d->W << "," << d->K << ","
      << d->R << "," << d->S << "|" << d->stride_h << "," << d->stride_w << "," << d->pad_h << "," << d->pad_w
      << "," << d->dil_h << "," << d->dil_w << "," << (d->groups > 1 ? d->groups : 1) << "|" << d->in_dtype << ","
      << d->out_dtype << "," << d->epilogue
      << "|" << layout_text(&d->x_layout) << "|" << layout_text(&d->w_layout) << "|" << layout_text(&d->y_layout);
    return o.str();
}

std::string gemm_key(alt_handle_t h, const alt_gemm_desc_t *d)
{
    std::ostringstream o;
    o << "gemm|" << h->arch << "|" << d->batch << "," << d->M << "," << d->N << "," << d->K << "|" << d->in_dtype
      << "," << d->out_dtype << "|" << layout_text(&d->a_layout) << "|" << layout_text(&d->b_layout) << "|"
      << layout_text(&d->c_layout);
    return o.str();
}

namespace {

__global__ void fill_kernel(uint32_t *dst, size_t nwords, uint32_t seed, int bf16)
{
    for (size_t i = blockIdx.x * (size_t)256 + threadIdx.x; i < nwords; i += (size_t)gridDim.x * 256) {
        uint32_t z = (uint32_t)i * 0x9E3779B9u + seed;
        z ^= z >> 16; z *= 0x85EBCA6Bu; z ^= z >> 13; z *= 0xC2B2AE35u; z ^= z >> 16;
        if (bf16) {
            // two bf16 values in [-1, 1): sign, exponent 0x7e/0x7d.., 7 random mantissa bits
            uint32_t lo = ((z & 0x8000u) | 0x3f00u | (z & 0x7fu));
            uint32_t hi = (((z >> 16) & 0x8000u) | 0x3e80u | ((z >> 16) & 0x7fu));
            dst[i] = lo | (hi << 16);
        } else {
            dst[i] = (z & 0x80000000u) | 0x3f000000u | (z & 0x007fffffu);   // +-[0.5, 1)
        }
    }
}

alt_status_t fill_random(alt_handle_t h, void *dst, size_t bytes, uint32_t seed, int dtype, hipStream_t st)
{
    size_t nwords = bytes / 4;
    if (nwords == 0) return ALT_OK;
    unsigned blocks = (unsigned)std::min<size_t>((nwords + 255) / 256, 4096);
    hipLaunchKernelGGL(fill_kernel, dim3(blocks), dim3(256), 0, st, (uint32_t *)dst, nwords, seed, dtype == ALT_BF16);
    ALT_CHECK_HIP(h, hipGetLastError());
    return ALT_OK;
}

struct Arena {
    char *base;
    size_t size, used;
    void *take(size_t bytes)
    {
        size_t a = (used + 255) & ~(size_t)255;
        if (a + bytes > size) return nullptr;
        used = a + bytes;
        return base + a;
    }
};

struct Timer {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    bool ok = false;
    Timer() { ok = hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess; }
    ~Timer()
    {
        if (e0) (void)hipEventDestroy(e0);
        if (e1) (void)hipEventDestroy(e1);
    }
};

// Average latency in microseconds of `launch` over `reps` back-to-back launches.
template <typename F>
alt_status_t measure(alt_handle_t h, Timer &tm, hipStream_t st, int warmup, int reps, F launch, float *us)
{
    for (int i = 0; i < warmup; ++i) {
        alt_status_t s = launch();
        if (s != ALT_OK) return s;
    }
    ALT_CHECK_HIP(h, hipEventRecord(tm.e0, st));
    for (int i = 0; i < reps; ++i) {
        alt_status_t s = launch();
        if (s != ALT_OK) return s;
    }
    ALT_CHECK_HIP(h, hipEventRecord(tm.e1, st));
    ALT_CHECK_HIP(h, hipEventSynchronize(tm.e1));
    float ms = 0.f;
    ALT_CHECK_HIP(h, hipEventElapsedTime(&ms, tm.e0, tm.e1));
    *us = ms * 1000.f / reps;
    return ALT_OK;
}

// ALT_VERBOSE=1 in the environment prints every trial to stderr.
bool verbose()
{
    static const bool v = std::getenv("ALT_VERBOSE") != nullptr;
    return v;
}

struct Trial {
    int variant;
    double est;
};

std::vector<Trial> ordered_variants(const Problem &pb, size_t ws_limit)
{
    std::vector<Trial> v;
    const auto &tab = igemm_table();
    const int ns = igemm_num_splits();
    for (int ki = 0; ki < (int)tab.size(); ++ki)
        for (int si = 0; si < ns; ++si) {
            IgemmParams p;
            if (!igemm_applicable(pb, tab[ki], kSplitFactors[si], &p, nullptr)) continue;
            if (igemm_workspace(pb, kSplitFactors[si]) > ws_limit) continue;
            v.push_back({ki * ns + si, igemm_estimate(pb, tab[ki], p)});
        }
    std::sort(v.begin(), v.end(), [](const Trial &a, const Trial &b) { return a.est < b.est; });
    return v;
}

struct ConvCand {
    const char *name, *x, *w, *y;
    int block;           // channel block that must divide C (x side) and K (y side); 0 = none
};

const ConvCand kConvCands[] = {
    {"NCHW/OIHW", "NCHW->NCHW", "OIHW->OIHW", "NCHW->NCHW", 0},
    {"NHWC/OHWI", "NCHW->NHWC", "OIHW->OHWI", "NCHW->NHWC", 0},
    {"NCHW8c/OIHW8o8i", "NCHW->NCHW8c", "OIHW->OIHW8o8i", "NCHW->NCHW8c", 8},
    {"NCHW16c/OIHW16o16i", "NCHW->NCHW16c", "OIHW->OIHW16o16i", "NCHW->NCHW16c", 16},
    {"NCHW32c/OIHW32o32i", "NCHW->NCHW32c", "OIHW->OIHW32o32i", "NCHW->NCHW32c", 32},
    {"NCHW64c/OIHW64o64i", "NCHW->NCHW64c", "OIHW->OIHW64o64i", "NCHW->NCHW64c", 64},
    {"NHWC/OIHW16o16i", "NCHW->NHWC", "OIHW->OIHW16o16i", "NCHW->NHWC", 16},
    {"NCHW32c/OHWI", "NCHW->NCHW32c", "OIHW->OHWI", "NCHW->NCHW32c", 32},
};
constexpr int kNumConvCands = sizeof(kConvCands) / sizeof(kConvCands[0]);

struct GemmCand {
    const char *name, *a, *b, *c;
    int bm, bk, bn;      // blocks that must divide M, K, N; 0 = none
};

// Row-major everything is the default; "NK" is the transposed weight; the
// blocked forms are the (M/m_t)(K/k_t) m_t k_t / (K/k_t)(N/n_t) ... template
// of Section 5.1 with the reduction index innermost, which is what the matrix
// cores consume.
const GemmCand kGemmCands[] = {
    {"MK,KN,MN", "MK->MK", "KN->KN", "MN->MN", 0, 0, 0},
    {"MK,NK,MN", "MK->MK", "KN->NK", "MN->MN", 0, 0, 0},
    {"MK,NK64n32k,MN", "MK->MK", "KN->NK64n32k", "MN->MN", 0, 32, 64},
    {"MK,NK128n64k,MN", "MK->MK", "KN->NK128n64k", "MN->MN", 0, 64, 128},
    {"MK128m32k,NK128n32k,MN", "MK->MK128m32k", "KN->NK128n32k", "MN->MN", 128, 32, 128},
    {"MK128m64k,NK128n64k,MN", "MK->MK128m64k", "KN->NK128n64k", "MN->MN", 128, 64, 128},
    {"MK,KN64k32n,MN", "MK->MK", "KN->KN64k32n", "MN->MN", 0, 64, 32},
};
constexpr int kNumGemmCands = sizeof(kGemmCands) / sizeof(kGemmCands[0]);

int opt_warmup(const alt_tune_opts_t *o) { return o->warmup > 0 ? o->warmup : 3; }
int opt_reps(const alt_tune_opts_t *o) { return o->reps > 0 ? o->reps : 20; }

size_t conv_bytes_x(const alt_conv_desc_t *d) { return (size_t)d->N * d->C * d->H * d->W * dtype_size(d->in_dtype); }
size_t conv_bytes_w(const alt_conv_desc_t *d)
{
    return (size_t)d->K * (d->C / (d->groups > 1 ? d->groups : 1)) * d->R * d->S * dtype_size(d->in_dtype);
}
size_t conv_bytes_y(const alt_conv_desc_t *d)
{
    int64_t o[4];
    if (alt_conv2d_output_shape(d, o) != ALT_OK) return 0;
    return (size_t)(o[0] * o[1] * o[2] * o[3]) * dtype_size(d->out_dtype);
}
size_t conv_ws_budget(const alt_conv_desc_t *d)
{
    int64_t o[4];
    if (alt_conv2d_output_shape(d, o) != ALT_OK) return 0;
    size_t one = (size_t)(o[0] * o[1] * o[2] * o[3]) * 4;
    return std::min<size_t>(one * 36, (size_t)256 << 20);
}

// Searches kernel variants for one fully specified conv; buffers are given.
alt_status_t tune_variants_conv(alt_handle_t h, const alt_conv_desc_t *d, const void *x, const void *w,
                                const float *bias, void *y, void *ws, size_t ws_bytes, hipStream_t st, Timer &tm,
                                int warmup, int reps, int max_trials, int *trials, float *best_us, int *best_variant)
{
    Problem pb;
    alt_status_t s = conv_problem(h, d, x, w, bias, y, &pb);
    if (s != ALT_OK) return s;
    std::vector<Trial> order = ordered_variants(pb, ws_bytes);
    *best_us = INFINITY;
    *best_variant = -1;
    int done = 0;
    for (const Trial &t : order) {
        if (max_trials > 0 && done >= max_trials) break;
        float us = 0.f;
        s = measure(h, tm, st, warmup, reps, [&] { return igemm_run(h, pb, t.variant, ws, ws_bytes, st); }, &us);
        if (s != ALT_OK) return s;
        ++done;
        if (verbose()) std::fprintf(stderr, "[alt tune] %-28s %9.2f us\n", igemm_variant_name(t.variant).c_str(), us);
        if (us < *best_us) { *best_us = us; *best_variant = t.variant; }
    }
    *trials += done;
    return ALT_OK;
}

}  // namespace
}  // namespace alt

using namespace alt;

extern "C" {

alt_status_t alt_tune_conv2d_arena_size(alt_handle_t h, const alt_conv_desc_t *d, size_t *bytes)
{
    if (!h) return ALT_INVALID_ARG;
    if (!d || !bytes) return fail(h, ALT_INVALID_ARG, "null argument");
    size_t y = conv_bytes_y(d);
    if (y == 0) return fail(h, ALT_INVALID_ARG, "bad conv shape");
    *bytes = 2 * conv_bytes_x(d) + 2 * conv_bytes_w(d) + y + (size_t)d->K * 4 + conv_ws_budget(d) + 8 * 256;
    return ALT_OK;
}

alt_status_t alt_tune_gemm_arena_size(alt_handle_t h, const alt_gemm_desc_t *d, size_t *bytes)
{
    if (!h) return ALT_INVALID_ARG;
    if (!d || !bytes) return fail(h, ALT_INVALID_ARG, "null argument");
    size_t es = dtype_size(d->in_dtype);
    size_t a = (size_t)d->batch * d->M * d->K * es, b = (size_t)d->batch * d->K * d->N * es;
    size_t c = (size_t)d->batch * d->M * d->N * 4;
    *bytes = 2 * a + 2 * b + c + std::min<size_t>(c * 36, (size_t)256 << 20) + 8 * 256;
    return ALT_OK;
}

alt_status_t alt_tune_conv2d_variants(alt_handle_t h, alt_conv_desc_t *d, const alt_tune_opts_t *opts, float *best_us,
                                      int *trials)
{
    if (!h) return ALT_INVALID_ARG;
    if (!d || !opts || !best_us || !trials) return fail(h, ALT_INVALID_ARG, "null argument");
    if (!h->has_gpu) return fail(h, ALT_HIP_ERROR, "no GPU device available");
    if (!opts->arena) return fail(h, ALT_INVALID_ARG, "tuning needs an arena");
    hipStream_t st = (hipStream_t)opts->stream;
    Arena ar{(char *)opts->arena, opts->arena_bytes, 0};
    void *x = ar.take(conv_bytes_x(d)), *w = ar.take(conv_bytes_w(d)), *y = ar.take(conv_bytes_y(d));
    float *bias = (float *)ar.take((size_t)d->K * 4);
    if (!x || !w || !y || !bias) return fail(h, ALT_WORKSPACE_TOO_SMALL, "arena too small for the tuner's tensors");
    size_t ws_bytes = std::min(conv_ws_budget(d), ar.size - ((ar.used + 255) & ~(size_t)255));
    void *ws = ar.take(ws_bytes);
    alt_status_t s;
    if ((s = fill_random(h, x, conv_bytes_x(d), 1, d->in_dtype, st)) != ALT_OK) return s;
    if ((s = fill_random(h, w, conv_bytes_w(d), 2, d->in_dtype, st)) != ALT_OK) return s;
    if ((s = fill_random(h, bias, (size_t)d->K * 4, 3, ALT_F32, st)) != ALT_OK) return s;
    Timer tm;
    if (!tm.ok) return fail(h, ALT_HIP_ERROR, "cannot create events");
    int best_v = -1;
    *trials = 0;
    s = tune_variants_conv(h, d, x, w, bias, y, ws, ws ? ws_bytes : 0, st, tm, opt_warmup(opts), opt_reps(opts),
                           opts->max_trials, trials, best_us, &best_v);
    if (s != ALT_OK) return s;
    if (best_v < 0) return fail(h, ALT_UNSUPPORTED, "no kernel variant applies");
    d->variant = -1;
    h->cache[conv_key(h, d)] = TuneEntry{best_v, *best_us};
    ++h->cache_gen;
    d->variant = best_v;
    return ALT_OK;
}

alt_status_t alt_tune_conv2d(alt_handle_t h, const alt_conv_desc_t *shape, const alt_tune_opts_t *opts,
                             alt_conv_desc_t *best_out, alt_tune_report_t *report)
{
    if (!h) return ALT_INVALID_ARG;
    if (!shape || !opts || !best_out) return fail(h, ALT_INVALID_ARG, "null argument");
    if (!h->has_gpu) return fail(h, ALT_HIP_ERROR, "no GPU device available");
    if (!opts->arena) return fail(h, ALT_INVALID_ARG, "tuning needs an arena");
    if (conv_bytes_y(shape) == 0) return fail(h, ALT_INVALID_ARG, "bad conv shape");
    hipStream_t st = (hipStream_t)opts->stream;
    alt_tune_report_t rep;
    std::memset(&rep, 0, sizeof rep);
    rep.best_us = INFINITY;
    rep.default_us = INFINITY;

    Arena ar{(char *)opts->arena, opts->arena_bytes, 0};
    const size_t xb = conv_bytes_x(shape), wbytes = conv_bytes_w(shape), yb = conv_bytes_y(shape);
    void *x0 = ar.take(xb), *x1 = ar.take(xb), *w0 = ar.take(wbytes), *w1 = ar.take(wbytes), *y = ar.take(yb);
    float *bias = (float *)ar.take((size_t)shape->K * 4);
    if (!x0 || !x1 || !w0 || !w1 || !y || !bias)
        return fail(h, ALT_WORKSPACE_TOO_SMALL, "arena too small for the tuner's tensors");
    size_t ws_bytes = std::min(conv_ws_budget(shape), ar.size - ((ar.used + 255) & ~(size_t)255));
    void *ws = ar.take(ws_bytes);
    if (!ws) ws_bytes = 0;
    alt_status_t s;
    if ((s = fill_random(h, x0, xb, 1, shape->in_dtype, st)) != ALT_OK) return s;
    if ((s = fill_random(h, w0, wbytes, 2, shape->in_dtype, st)) != ALT_OK) return s;
    if ((s = fill_random(h, bias, (size_t)shape->K * 4, 3, ALT_F32, st)) != ALT_OK) return s;
    Timer tm;
    if (!tm.ok) return fail(h, ALT_HIP_ERROR, "cannot create events");

    // candidate layouts valid for this shape
    std::vector<int> cands;
    for (int c = 0; c < kNumConvCands; ++c) {
        if (opts->layout_mask && !(opts->layout_mask & (1 << c))) continue;
        int b = kConvCands[c].block;
        // channel blocks must divide the channels, of one group for group-wise problems
        const int64_t G = shape->groups > 1 ? shape->groups : 1;
        if (b && ((shape->C / G) % b || (shape->K / G) % b)) continue;
        cands.push_back(c);
    }
    if (cands.empty()) return fail(h, ALT_INVALID_ARG, "layout_mask leaves no candidate");
    const int budget = opts->max_trials;
    const int joint_budget = budget > 0 ? std::max<int>((int)cands.size(), budget * 3 / 10) : 0;
    const int per_layout = budget > 0 ? std::max(1, joint_budget / (int)cands.size()) : 0;

    const int64_t xs[4] = {shape->N, shape->C, shape->H, shape->W};
    alt_layout_t plain_x;
    alt_layout_parse("NCHW->NCHW", &plain_x);
    std::vector<alt_conv_desc_t> descs(cands.size());
    int best_c = -1;
    for (size_t ci = 0; ci < cands.size(); ++ci) {
        const ConvCand &cc = kConvCands[cands[ci]];
        alt_conv_desc_t d = *shape;
        d.variant = -1;
        alt_layout_parse(cc.x, &d.x_layout);
        alt_layout_parse(cc.w, &d.w_layout);
        alt_layout_parse(cc.y, &d.y_layout);
        // inputs under this layout (conversion and weight packing are not timed)
        BoundLayout bs, bd;
        std::string err;
        if ((s = bind_layout(&plain_x, 4, xs, &bs, &err)) != ALT_OK) return fail(h, s, "%s", err.c_str());
        if ((s = bind_layout(&d.x_layout, 4, xs, &bd, &err)) != ALT_OK) return fail(h, s, "%s", err.c_str());
        if ((s = transform_bound(h, (int)dtype_size(d.in_dtype), bs, x0, bd, x1, st)) != ALT_OK) return s;
        if ((s = alt_pack_weights(h, &d, w0, w1, st)) != ALT_OK) return s;
        float us = INFINITY;
        int v = -1;
        if (verbose()) std::fprintf(stderr, "[alt tune] layout %s\n", cc.name);
        s = tune_variants_conv(h, &d, x1, w1, bias, y, ws, ws_bytes, st, tm, opt_warmup(opts), opt_reps(opts),
                               per_layout, &rep.trials, &us, &v);
        if (s != ALT_OK) return s;
        d.variant = v;
        descs[ci] = d;
        int slot = rep.n_layouts++;
        rep.layout_best_us[slot] = us;
        rep.layout_best_variant[slot] = v;
        std::snprintf(rep.layout_name[slot], sizeof rep.layout_name[slot], "%s", cc.name);
        if (cands[ci] == 0) rep.default_us = us;
        if (v >= 0 && us < rep.best_us) { rep.best_us = us; best_c = (int)ci; }
    }
    if (best_c < 0) return fail(h, ALT_UNSUPPORTED, "no kernel variant applies under any layout");
    // loop-only stage on the winner with whatever budget is left
    if (budget > 0 && rep.trials < budget) {
        const ConvCand &cc = kConvCands[cands[best_c]];
        alt_conv_desc_t d = descs[best_c];
        BoundLayout bs, bd;
        std::string err;
        bind_layout(&plain_x, 4, xs, &bs, &err);
        bind_layout(&d.x_layout, 4, xs, &bd, &err);
        if ((s = transform_bound(h, (int)dtype_size(d.in_dtype), bs, x0, bd, x1, st)) != ALT_OK) return s;
        if ((s = alt_pack_weights(h, &d, w0, w1, st)) != ALT_OK) return s;
        float us = INFINITY;
        int v = -1, extra = 0;
        s = tune_variants_conv(h, &d, x1, w1, bias, y, ws, ws_bytes, st, tm, opt_warmup(opts), opt_reps(opts),
                               budget - rep.trials + per_layout, &extra, &us, &v);
        if (s != ALT_OK) return s;
        rep.trials += std::max(0, extra - per_layout);     // the first per_layout trials repeat the joint stage
        if (v >= 0 && us < rep.best_us) {
            rep.best_us = us;
            descs[best_c].variant = v;
            for (int sl = 0; sl < rep.n_layouts; ++sl)
                if (!std::strcmp(rep.layout_name[sl], cc.name)) { rep.layout_best_us[sl] = us; rep.layout_best_variant[sl] = v; }
        }
    }
    for (size_t ci = 0; ci < cands.size(); ++ci) {
        if (descs[ci].variant < 0) continue;
        alt_conv_desc_t k = descs[ci];
        k.variant = -1;
        h->cache[conv_key(h, &k)] = TuneEntry{descs[ci].variant, rep.layout_best_us[ci]};
    }
    ++h->cache_gen;
    *best_out = descs[best_c];
    if (report) *report = rep;
    return ALT_OK;
}

alt_status_t alt_tune_gemm(alt_handle_t h, const alt_gemm_desc_t *shape, const alt_tune_opts_t *opts,
                           alt_gemm_desc_t *best_out, alt_tune_report_t *report)
{
    if (!h) return ALT_INVALID_ARG;
    if (!shape || !opts || !best_out) return fail(h, ALT_INVALID_ARG, "null argument");
    if (!h->has_gpu) return fail(h, ALT_HIP_ERROR, "no GPU device available");
    if (!opts->arena) return fail(h, ALT_INVALID_ARG, "tuning needs an arena");
    if (shape->batch < 1 || shape->M < 1 || shape->N < 1 || shape->K < 1) return fail(h, ALT_INVALID_ARG, "bad gemm shape");
    hipStream_t st = (hipStream_t)opts->stream;
    alt_tune_report_t rep;
    std::memset(&rep, 0, sizeof rep);
    rep.best_us = INFINITY;
    rep.default_us = INFINITY;
    const size_t es = dtype_size(shape->in_dtype);
    const size_t ab = (size_t)shape->batch * shape->M * shape->K * es, bb = (size_t)shape->batch * shape->K * shape->N * es;
    const size_t cb = (size_t)shape->batch * shape->M * shape->N * dtype_size(shape->out_dtype);
    Arena ar{(char *)opts->arena, opts->arena_bytes, 0};
    void *a0 = ar.take(ab), *a1 = ar.take(ab), *b0 = ar.take(bb), *b1 = ar.take(bb), *c = ar.take(cb);
    if (!a0 || !a1 || !b0 || !b1 || !c) return fail(h, ALT_WORKSPACE_TOO_SMALL, "arena too small for the tuner's tensors");
    size_t ws_bytes = std::min(std::min<size_t>((size_t)shape->batch * shape->M * shape->N * 4 * 36, (size_t)256 << 20),
                               ar.size - ((ar.used + 255) & ~(size_t)255));
    void *ws = ar.take(ws_bytes);
    if (!ws) ws_bytes = 0;
    alt_status_t s;
    if ((s = fill_random(h, a0, ab, 1, shape->in_dtype, st)) != ALT_OK) return s;
    if ((s = fill_random(h, b0, bb, 2, shape->in_dtype, st)) != ALT_OK) return s;
    Timer tm;
    if (!tm.ok) return fail(h, ALT_HIP_ERROR, "cannot create events");
    std::vector<int> cands;
    for (int ci = 0; ci < kNumGemmCands; ++ci) {
        if (opts->layout_mask && !(opts->layout_mask & (1 << ci))) continue;
        const GemmCand &g = kGemmCands[ci];
        if ((g.bm && shape->M % g.bm) || (g.bk && shape->K % g.bk) || (g.bn && shape->N % g.bn)) continue;
        cands.push_back(ci);
    }
    if (cands.empty()) return fail(h, ALT_INVALID_ARG, "layout_mask leaves no candidate");
    const int budget = opts->max_trials;
    const int per_layout = budget > 0 ? std::max(1, budget / (int)cands.size()) : 0;
    alt_layout_t la, lb;
    alt_layout_parse("MK->MK", &la);
    alt_layout_parse("KN->KN", &lb);
    const int64_t as[2] = {shape->M, shape->K}, bs2[2] = {shape->K, shape->N};
    int best_c = -1;
    std::vector<alt_gemm_desc_t> descs(cands.size());
    for (size_t ci = 0; ci < cands.size(); ++ci) {
        const GemmCand &g = kGemmCands[cands[ci]];
        alt_gemm_desc_t d = *shape;
        d.variant = -1;
        alt_layout_parse(g.a, &d.a_layout);
        alt_layout_parse(g.b, &d.b_layout);
        alt_layout_parse(g.c, &d.c_layout);
        BoundLayout s0, s1;
        std::string err;
        // operands under this layout, one batch entry at a time (untimed)
        for (int64_t bz = 0; bz < shape->batch; ++bz) {
            if ((s = bind_layout(&la, 2, as, &s0, &err)) != ALT_OK) return fail(h, s, "%s", err.c_str());
            if ((s = bind_layout(&d.a_layout, 2, as, &s1, &err)) != ALT_OK) return fail(h, s, "%s", err.c_str());
            size_t off = (size_t)bz * shape->M * shape->K * es;
            if ((s = transform_bound(h, (int)es, s0, (char *)a0 + off, s1, (char *)a1 + off, st)) != ALT_OK) return s;
            if ((s = bind_layout(&lb, 2, bs2, &s0, &err)) != ALT_OK) return fail(h, s, "%s", err.c_str());
            if ((s = bind_layout(&d.b_layout, 2, bs2, &s1, &err)) != ALT_OK) return fail(h, s, "%s", err.c_str());
            off = (size_t)bz * shape->K * shape->N * es;
            if ((s = transform_bound(h, (int)es, s0, (char *)b0 + off, s1, (char *)b1 + off, st)) != ALT_OK) return s;
        }
        Problem pb;
        if ((s = gemm_problem(h, &d, a1, b1, c, &pb)) != ALT_OK) return s;
        std::vector<Trial> order = ordered_variants(pb, ws_bytes);
        float best = INFINITY;
        int bv = -1, done = 0;
        for (const Trial &t : order) {
            if (per_layout > 0 && done >= per_layout) break;
            float us = 0.f;
            s = measure(h, tm, st, opt_warmup(opts), opt_reps(opts),
                        [&] { return igemm_run(h, pb, t.variant, ws, ws_bytes, st); }, &us);
            if (s != ALT_OK) return s;
            ++done;
            if (us < best) { best = us; bv = t.variant; }
        }
        rep.trials += done;
        d.variant = bv;
        descs[ci] = d;
        int slot = rep.n_layouts++;
        rep.layout_best_us[slot] = best;
        rep.layout_best_variant[slot] = bv;
        std::snprintf(rep.layout_name[slot], sizeof rep.layout_name[slot], "%s", g.name);
        if (cands[ci] == 0) rep.default_us = best;
        if (bv >= 0 && best < rep.best_us) { rep.best_us = best; best_c = (int)ci; }
        if (bv >= 0) {
            alt_gemm_desc_t k = d;
            k.variant = -1;
            h->cache[gemm_key(h, &k)] = TuneEntry{bv, best};
            ++h->cache_gen;
        }
    }
    if (best_c < 0) return fail(h, ALT_UNSUPPORTED, "no kernel variant applies under any layout");
    *best_out = descs[best_c];
    if (report) *report = rep;
    return ALT_OK;
}

alt_status_t alt_plan_chain(int nops, int nl, const float *op_cost, const float *conv_cost, int in_layout,
                            int *out_in_idx, int *out_out_idx, float *out_total)
{
    if (!op_cost || !conv_cost || !out_in_idx || !out_out_idx || !out_total) return ALT_INVALID_ARG;
    if (nops < 1 || nops > ALT_MAX_CHAIN || nl < 1 || nl > ALT_MAX_CANDIDATES || in_layout < 0 || in_layout >= nl)
        return ALT_INVALID_ARG;
    // best[i][b]: cheapest way to have operator i's output in layout b
    std::vector<std::vector<double>> best(nops, std::vector<double>(nl, INFINITY));
    std::vector<std::vector<int>> arg_a(nops, std::vector<int>(nl, -1)), arg_prev(nops, std::vector<int>(nl, -1));
    auto OC = [&](int i, int a, int b) { return (double)op_cost[((size_t)i * nl + a) * nl + b]; };
    auto CC = [&](int i, int a, int b) { return a == b ? 0.0 : (double)conv_cost[((size_t)i * nl + a) * nl + b]; };
    for (int i = 0; i < nops; ++i)
        for (int b = 0; b < nl; ++b)
            for (int a = 0; a < nl; ++a) {
                if (!(OC(i, a, b) < INFINITY)) continue;
                if (i == 0) {
                    double c = CC(0, in_layout, a) + OC(0, a, b);
                    if (c < best[0][b]) { best[0][b] = c; arg_a[0][b] = a; arg_prev[0][b] = in_layout; }
                } else {
                    for (int pb = 0; pb < nl; ++pb) {
                        if (!(best[i - 1][pb] < INFINITY)) continue;
                        double c = best[i - 1][pb] + CC(i, pb, a) + OC(i, a, b);
                        if (c < best[i][b]) { best[i][b] = c; arg_a[i][b] = a; arg_prev[i][b] = pb; }
                    }
                }
            }
    int b = -1;
    for (int j = 0; j < nl; ++j)
        if (best[nops - 1][j] < INFINITY && (b < 0 || best[nops - 1][j] < best[nops - 1][b])) b = j;
    if (b < 0) return ALT_UNSUPPORTED;
    *out_total = (float)best[nops - 1][b];
    for (int i = nops - 1; i >= 0; --i) {
        out_out_idx[i] = b;
        out_in_idx[i] = arg_a[i][b];
        b = arg_prev[i][b];
    }
    return ALT_OK;
}

// Layout families the chain planner considers on every edge.
static const char *const kEdgeLayouts[] = {"NCHW->NCHW", "NCHW->NHWC", "NCHW->NCHW16c", "NCHW->NCHW32c"};
static const int kEdgeBlock[] = {0, 0, 16, 32};
static const char *const kEdgeWeights[] = {"OIHW->OIHW", "OIHW->OHWI", "OIHW->OHWI", "OIHW->OHWI"};
constexpr int kNumEdgeLayouts = 4;

alt_status_t alt_tune_chain(alt_handle_t h, const alt_conv_desc_t *ops, int nops, const alt_layout_t *in_layout,
                            const alt_tune_opts_t *opts, alt_chain_plan_t *plan)
{
    if (!h) return ALT_INVALID_ARG;
    if (!ops || !in_layout || !opts || !plan) return fail(h, ALT_INVALID_ARG, "null argument");
    if (nops < 1 || nops > ALT_MAX_CHAIN) return fail(h, ALT_INVALID_ARG, "chain length out of range");
    if (!h->has_gpu) return fail(h, ALT_HIP_ERROR, "no GPU device available");
    if (!opts->arena) return fail(h, ALT_INVALID_ARG, "tuning needs an arena");
    hipStream_t st = (hipStream_t)opts->stream;
    const int nl = kNumEdgeLayouts;
    std::memset(plan, 0, sizeof *plan);
    // shapes must chain
    for (int i = 0; i < nops; ++i) {
        int64_t o[4];
        if (alt_conv2d_output_shape(&ops[i], o) != ALT_OK) return fail(h, ALT_INVALID_ARG, "operator %d: bad shape", i);
        if (i + 1 < nops && (ops[i + 1].N != o[0] || ops[i + 1].C != o[1] || ops[i + 1].H != o[2] || ops[i + 1].W != o[3]))
            return fail(h, ALT_SHAPE_MISMATCH, "operator %d does not consume operator %d's output", i + 1, i);
        if (i + 1 < nops && ops[i].out_dtype != ops[i + 1].in_dtype)
            return fail(h, ALT_SHAPE_MISMATCH, "operator %d's output type is not operator %d's input type", i, i + 1);
    }
    alt_layout_t L[kNumEdgeLayouts];
    for (int j = 0; j < nl; ++j) alt_layout_parse(kEdgeLayouts[j], &L[j]);
    int in_idx = -1;
    for (int j = 0; j < nl; ++j)
        if (layout_text(&L[j]) == layout_text(in_layout)) in_idx = j;
    if (in_idx < 0) return fail(h, ALT_UNSUPPORTED, "chain input layout is not one of the planner's edge layouts");

    size_t max_x = 0, max_w = 0, max_y = 0, max_ws = 0;
    int64_t max_k = 0;
    for (int i = 0; i < nops; ++i) {
        max_x = std::max(max_x, conv_bytes_x(&ops[i]));
        max_w = std::max(max_w, conv_bytes_w(&ops[i]));
        max_y = std::max(max_y, conv_bytes_y(&ops[i]));
        max_ws = std::max(max_ws, std::min<size_t>(conv_ws_budget(&ops[i]), (size_t)64 << 20));
        max_k = std::max(max_k, ops[i].K);
    }
    Arena ar{(char *)opts->arena, opts->arena_bytes, 0};
    void *x0 = ar.take(max_x), *x1 = ar.take(max_x), *w0 = ar.take(max_w), *w1 = ar.take(max_w), *y = ar.take(max_y);
    float *bias = (float *)ar.take((size_t)max_k * 4);
    if (!x0 || !x1 || !w0 || !w1 || !y || !bias) return fail(h, ALT_WORKSPACE_TOO_SMALL, "arena too small for the chain");
    size_t ws_bytes = std::min(max_ws, ar.size - ((ar.used + 255) & ~(size_t)255));
    void *ws = ar.take(ws_bytes);
    if (!ws) ws_bytes = 0;
    Timer tm;
    if (!tm.ok) return fail(h, ALT_HIP_ERROR, "cannot create events");
    alt_status_t s;
    if ((s = fill_random(h, x0, max_x, 1, ops[0].in_dtype, st)) != ALT_OK) return s;
    if ((s = fill_random(h, w0, max_w, 2, ops[0].in_dtype, st)) != ALT_OK) return s;
    if ((s = fill_random(h, bias, (size_t)max_k * 4, 3, ALT_F32, st)) != ALT_OK) return s;

    std::vector<float> op_cost((size_t)nops * nl * nl, INFINITY), conv_cost((size_t)nops * nl * nl, 0.f);
    std::vector<int> op_var((size_t)nops * nl * nl, -1);
    const int per_pair = opts->max_trials > 0 ? std::max(1, opts->max_trials / (nops * nl * nl)) : 8;
    alt_layout_t plain_x;
    alt_layout_parse("NCHW->NCHW", &plain_x);
    for (int i = 0; i < nops; ++i) {
        const int64_t xs[4] = {ops[i].N, ops[i].C, ops[i].H, ops[i].W};
        for (int a = 0; a < nl; ++a) {
            if (kEdgeBlock[a] && ops[i].C % kEdgeBlock[a]) continue;
            BoundLayout bs, bd;
            std::string err;
            if ((s = bind_layout(&plain_x, 4, xs, &bs, &err)) != ALT_OK) return fail(h, s, "%s", err.c_str());
            if ((s = bind_layout(&L[a], 4, xs, &bd, &err)) != ALT_OK) return fail(h, s, "%s", err.c_str());
            if ((s = transform_bound(h, (int)dtype_size(ops[i].in_dtype), bs, x0, bd, x1, st)) != ALT_OK) return s;
            // conversions of this edge, a -> b
            for (int b = 0; b < nl; ++b) {
                if (a == b || (kEdgeBlock[b] && ops[i].C % kEdgeBlock[b])) continue;
                BoundLayout bb;
                if ((s = bind_layout(&L[b], 4, xs, &bb, &err)) != ALT_OK) return fail(h, s, "%s", err.c_str());
                float us = 0.f;
                s = measure(h, tm, st, opt_warmup(opts), opt_reps(opts), [&] {
                    return transform_bound(h, (int)dtype_size(ops[i].in_dtype), bd, x1, bb, y, st);
                }, &us);
                if (s != ALT_OK) return s;
                ++plan->trials;
                conv_cost[((size_t)i * nl + a) * nl + b] = us;
            }
            for (int b = 0; b < nl; ++b) {
                if (kEdgeBlock[b] && ops[i].K % kEdgeBlock[b]) continue;
                alt_conv_desc_t d = ops[i];
                d.variant = -1;
                d.x_layout = L[a];
                d.y_layout = L[b];
                alt_layout_parse(kEdgeWeights[a], &d.w_layout);
                if ((s = alt_pack_weights(h, &d, w0, w1, st)) != ALT_OK) return s;
                float us = INFINITY;
                int v = -1;
                s = tune_variants_conv(h, &d, x1, w1, bias, y, ws, ws_bytes, st, tm, opt_warmup(opts), opt_reps(opts),
                                       per_pair, &plan->trials, &us, &v);
                if (s != ALT_OK) return s;
                if (v < 0) continue;
                op_cost[((size_t)i * nl + a) * nl + b] = us;
                op_var[((size_t)i * nl + a) * nl + b] = v;
                h->cache[conv_key(h, &d)] = TuneEntry{v, us};
                ++h->cache_gen;
            }
        }
    }
    int ins[ALT_MAX_CHAIN], outs[ALT_MAX_CHAIN];
    float total = 0.f;
    s = alt_plan_chain(nops, nl, op_cost.data(), conv_cost.data(), in_idx, ins, outs, &total);
    if (s != ALT_OK) return fail(h, s, "no feasible plan");
    plan->nops = nops;
    plan->total_us = total;
    plan->edge_layout[0] = L[in_idx];
    int prev = in_idx;
    for (int i = 0; i < nops; ++i) {
        alt_conv_desc_t d = ops[i];
        d.x_layout = L[ins[i]];
        d.y_layout = L[outs[i]];
        alt_layout_parse(kEdgeWeights[ins[i]], &d.w_layout);
        d.variant = op_var[((size_t)i * nl + ins[i]) * nl + outs[i]];
        plan->op[i] = d;
        plan->transform_before[i] = prev != ins[i];
        plan->transform_us[i] = prev != ins[i] ? conv_cost[((size_t)i * nl + prev) * nl + ins[i]] : 0.f;
        plan->op_us[i] = op_cost[((size_t)i * nl + ins[i]) * nl + outs[i]];
        plan->edge_layout[i + 1] = L[outs[i]];
        prev = outs[i];
    }
    plan->default_total_us = 0.f;
    for (int i = 0; i < nops; ++i) plan->default_total_us += op_cost[((size_t)i * nl + 0) * nl + 0];
    if (in_idx != 0) plan->default_total_us += conv_cost[((size_t)0 * nl + in_idx) * nl + 0];
    return ALT_OK;
}

// ---- graphs: layout propagation through element-wise operators (Section 4.2) -------------

alt_status_t alt_plan_graph(int nnodes, const int32_t *kind, const int32_t *in0, const int32_t *in1, int nl,
                            const float *op_cost, const float *conv_cost, const float *add_cost, int in_layout,
                            int32_t *tensor_layout, int32_t *read_layout, float *total)
{
    if (!kind || !in0 || !in1 || !op_cost || !conv_cost || !add_cost || !tensor_layout || !read_layout || !total)
        return ALT_INVALID_ARG;
    if (nnodes < 1 || nnodes > ALT_MAX_GRAPH || nl < 1 || nl > ALT_MAX_CANDIDATES || in_layout < 0 || in_layout >= nl)
        return ALT_INVALID_ARG;
    for (int i = 0; i < nnodes; ++i) {
        if (kind[i] != ALT_NODE_CONV && kind[i] != ALT_NODE_ADD) return ALT_INVALID_ARG;
        if (in0[i] < 0 || in0[i] > i) return ALT_INVALID_ARG;
        if (kind[i] == ALT_NODE_ADD && (in1[i] < 0 || in1[i] > i)) return ALT_INVALID_ARG;
    }
    auto OC = [&](int i, int a, int b) { return (double)op_cost[((size_t)i * nl + a) * nl + b]; };
    auto CC = [&](int t, int a, int b) { return a == b ? 0.0 : (double)conv_cost[((size_t)t * nl + a) * nl + b]; };
    // Every assignment of a stored layout to the node outputs (tensor 0 is given) and of a layout
    // each convolution reads; a sum reads both inputs in the layout it writes.  A tensor converted
    // to one layout is paid for once, however many consumers read that copy.  Beyond 2^24
    // assignments the convolutions' read layouts are no longer enumerated but picked greedily in
    // node order (cheapest conversion + kernel given the copies already made).
    std::vector<int> s(nnodes + 1, 0), rd(nnodes * 2, -1), best_s, best_rd, conv_nodes;
    for (int i = 0; i < nnodes; ++i)
        if (kind[i] == ALT_NODE_CONV) conv_nodes.push_back(i);
    s[0] = in_layout;
    double best = INFINITY;
    double space = 1.0;
    for (int i = 0; i < nnodes + (int)conv_nodes.size(); ++i) space *= nl;
    const bool exact = space <= (double)(1 << 24);
    const int nvar = nnodes + (exact ? (int)conv_nodes.size() : 0);
    long long combos = 1;
    for (int i = 0; i < nvar; ++i) combos *= nl;
    std::vector<int> want(nnodes, -1);
    for (long long c = 0; c < combos; ++c) {
        long long r = c;
        for (int i = 0; i < nnodes; ++i) { s[i + 1] = (int)(r % nl); r /= nl; }
        if (exact)
            for (int i : conv_nodes) { want[i] = (int)(r % nl); r /= nl; }
        double tot = 0.0;
        unsigned paid[ALT_MAX_GRAPH + 1] = {0};
        auto convert = [&](int t, int to) {
            if (s[t] == to || (paid[t] >> to & 1u)) return 0.0;
            return CC(t, s[t], to);
        };
        for (int i = 0; i < nnodes && tot < best; ++i) {
            const int out = s[i + 1];
            if (kind[i] == ALT_NODE_CONV) {
                double m = INFINITY;
                int arg = -1;
                for (int a = 0; a < nl; ++a) {
                    if (exact && a != want[i]) continue;
                    const double v = convert(in0[i], a) + OC(i, a, out);
                    if (v < m) { m = v; arg = a; }
                }
                if (arg >= 0) paid[in0[i]] |= 1u << arg;
                rd[i * 2] = arg; rd[i * 2 + 1] = -1;
                tot += m;
            } else {
                rd[i * 2] = out; rd[i * 2 + 1] = out;
                tot += (double)add_cost[i] + convert(in0[i], out);
                paid[in0[i]] |= 1u << out;
                tot += convert(in1[i], out);
                paid[in1[i]] |= 1u << out;
            }
        }
        if (tot < best) { best = tot; best_s = s; best_rd = rd; }
    }
    if (!(best < INFINITY)) return ALT_UNSUPPORTED;
    for (int t = 0; t <= nnodes; ++t) tensor_layout[t] = best_s[t];
    for (int i = 0; i < nnodes * 2; ++i) read_layout[i] = best_rd[i];
    *total = (float)best;
    return ALT_OK;
}

alt_status_t alt_tune_graph(alt_handle_t h, const alt_graph_node_t *nodes, int nnodes, const alt_layout_t *in_layout,
                            const alt_tune_opts_t *opts, alt_graph_plan_t *plan)
{
    if (!h) return ALT_INVALID_ARG;
    if (!nodes || !in_layout || !opts || !plan) return fail(h, ALT_INVALID_ARG, "null argument");
    if (nnodes < 1 || nnodes > ALT_MAX_GRAPH) return fail(h, ALT_INVALID_ARG, "graph size out of range");
    if (!h->has_gpu) return fail(h, ALT_HIP_ERROR, "no GPU device available");
    if (!opts->arena) return fail(h, ALT_INVALID_ARG, "tuning needs an arena");
    hipStream_t st = (hipStream_t)opts->stream;
    const int nl = kNumEdgeLayouts;
    std::memset(plan, 0, sizeof *plan);

    // shape and element type of every tensor
    struct Tensor { int64_t shape[4]; int dtype; bool known, consumed; };
    std::vector<Tensor> T(nnodes + 1);
    for (auto &t : T) { t.known = false; t.consumed = false; }
    auto same = [](const Tensor &a, const int64_t *sh, int dt) {
        return a.shape[0] == sh[0] && a.shape[1] == sh[1] && a.shape[2] == sh[2] && a.shape[3] == sh[3] && a.dtype == dt;
    };
    for (int i = 0; i < nnodes; ++i) {
        const alt_graph_node_t &nd = nodes[i];
        if (nd.kind != ALT_NODE_CONV && nd.kind != ALT_NODE_ADD) return fail(h, ALT_INVALID_ARG, "node %d: bad kind", i);
        if (nd.in0 < 0 || nd.in0 > i || (nd.kind == ALT_NODE_ADD && (nd.in1 < 0 || nd.in1 > i)))
            return fail(h, ALT_INVALID_ARG, "node %d reads a tensor that is not produced before it", i);
        if (nd.kind == ALT_NODE_CONV) {
            const int64_t xs[4] = {nd.conv.N, nd.conv.C, nd.conv.H, nd.conv.W};
            int64_t o[4];
            if (alt_conv2d_output_shape(&nd.conv, o) != ALT_OK) return fail(h, ALT_INVALID_ARG, "node %d: bad shape", i);
            Tensor &in = T[nd.in0];
            if (!in.known) { std::memcpy(in.shape, xs, sizeof xs); in.dtype = nd.conv.in_dtype; in.known = true; }
            else if (!same(in, xs, nd.conv.in_dtype)) return fail(h, ALT_SHAPE_MISMATCH, "node %d does not fit the tensor it reads", i);
            in.consumed = true;
            std::memcpy(T[i + 1].shape, o, sizeof o);
            T[i + 1].dtype = nd.conv.out_dtype;
            T[i + 1].known = true;
        } else {
            Tensor &a = T[nd.in0], &b = T[nd.in1];
            if (!a.known && b.known) a = b;
            if (!b.known && a.known) { const bool c = b.consumed; b = a; b.consumed = c; }
            if (!a.known || !same(a, b.shape, b.dtype)) return fail(h, ALT_SHAPE_MISMATCH, "node %d adds tensors of different shape or type", i);
            a.consumed = b.consumed = true;
            T[i + 1] = a;
            T[i + 1].consumed = false;
        }
    }
    alt_layout_t L[kNumEdgeLayouts];
    for (int j = 0; j < nl; ++j) alt_layout_parse(kEdgeLayouts[j], &L[j]);
    int in_idx = -1;
    for (int j = 0; j < nl; ++j)
        if (layout_text(&L[j]) == layout_text(in_layout)) in_idx = j;
    if (in_idx < 0) return fail(h, ALT_UNSUPPORTED, "graph input layout is not one of the planner's layouts");

    size_t max_t = 0, max_w = 16, max_ws = 0;
    int64_t max_k = 1;
    for (auto &t : T) max_t = std::max<size_t>(max_t, (size_t)(t.shape[0] * t.shape[1] * t.shape[2] * t.shape[3]) * dtype_size((alt_dtype_t)t.dtype));
    for (int i = 0; i < nnodes; ++i)
        if (nodes[i].kind == ALT_NODE_CONV) {
            max_w = std::max(max_w, conv_bytes_w(&nodes[i].conv));
            max_ws = std::max(max_ws, std::min<size_t>(conv_ws_budget(&nodes[i].conv), (size_t)64 << 20));
            max_k = std::max(max_k, nodes[i].conv.K);
        }
    Arena ar{(char *)opts->arena, opts->arena_bytes, 0};
    void *x0 = ar.take(max_t), *x1 = ar.take(max_t), *w0 = ar.take(max_w), *w1 = ar.take(max_w), *y = ar.take(max_t);
    float *bias = (float *)ar.take((size_t)max_k * 4);
    if (!x0 || !x1 || !w0 || !w1 || !y || !bias) return fail(h, ALT_WORKSPACE_TOO_SMALL, "arena too small for the graph");
    size_t ws_bytes = std::min(max_ws, ar.size - ((ar.used + 255) & ~(size_t)255));
    void *ws = ar.take(ws_bytes);
    if (!ws) ws_bytes = 0;
    Timer tm;
    if (!tm.ok) return fail(h, ALT_HIP_ERROR, "cannot create events");
    alt_status_t s;
    if ((s = fill_random(h, x0, max_t, 1, T[0].dtype, st)) != ALT_OK) return s;
    if ((s = fill_random(h, x1, max_t, 4, T[0].dtype, st)) != ALT_OK) return s;
    if ((s = fill_random(h, w0, max_w, 2, T[0].dtype, st)) != ALT_OK) return s;
    if ((s = fill_random(h, bias, (size_t)max_k * 4, 3, ALT_F32, st)) != ALT_OK) return s;

    std::vector<float> op_cost((size_t)nnodes * nl * nl, INFINITY), conv_cost((size_t)(nnodes + 1) * nl * nl, INFINITY);
    std::vector<float> add_cost(nnodes, 0.f);
    std::vector<int> op_var((size_t)nnodes * nl * nl, -1);
    int nconv = 0;
    for (int i = 0; i < nnodes; ++i) nconv += nodes[i].kind == ALT_NODE_CONV;
    const int per_pair = opts->max_trials > 0 ? std::max(1, opts->max_trials / (std::max(nconv, 1) * nl * nl)) : 8;
    alt_layout_t plain_x;
    alt_layout_parse("NCHW->NCHW", &plain_x);
    std::string err;
    // conversions of every consumed tensor
    for (int t = 0; t <= nnodes; ++t) {
        if (!T[t].consumed) continue;
        const int esz = (int)dtype_size((alt_dtype_t)T[t].dtype);
        for (int a = 0; a < nl; ++a) {
            if (kEdgeBlock[a] && T[t].shape[1] % kEdgeBlock[a]) continue;
            conv_cost[((size_t)t * nl + a) * nl + a] = 0.f;
            BoundLayout ba;
            if ((s = bind_layout(&L[a], 4, T[t].shape, &ba, &err)) != ALT_OK) return fail(h, s, "%s", err.c_str());
            for (int b = 0; b < nl; ++b) {
                if (a == b || (kEdgeBlock[b] && T[t].shape[1] % kEdgeBlock[b])) continue;
                BoundLayout bb;
                if ((s = bind_layout(&L[b], 4, T[t].shape, &bb, &err)) != ALT_OK) return fail(h, s, "%s", err.c_str());
                float us = 0.f;
                s = measure(h, tm, st, opt_warmup(opts), opt_reps(opts), [&] { return transform_bound(h, esz, ba, x0, bb, y, st); }, &us);
                if (s != ALT_OK) return s;
                ++plan->trials;
                conv_cost[((size_t)t * nl + a) * nl + b] = us;
            }
        }
    }
    for (int i = 0; i < nnodes; ++i) {
        if (nodes[i].kind == ALT_NODE_ADD) {
            const Tensor &t = T[i + 1];
            const int64_t numel = t.shape[0] * t.shape[1] * t.shape[2] * t.shape[3];
            float us = 0.f;
            s = measure(h, tm, st, opt_warmup(opts), opt_reps(opts), [&] { return eltwise_add(h, t.dtype, numel, x0, x1, y, nodes[i].relu, st); }, &us);
            if (s != ALT_OK) return s;
            ++plan->trials;
            add_cost[i] = us;
            continue;
        }
        const alt_conv_desc_t &op = nodes[i].conv;
        const int64_t xs[4] = {op.N, op.C, op.H, op.W};
        for (int a = 0; a < nl; ++a) {
            if (kEdgeBlock[a] && op.C % kEdgeBlock[a]) continue;
            BoundLayout bs, bd;
            if ((s = bind_layout(&plain_x, 4, xs, &bs, &err)) != ALT_OK) return fail(h, s, "%s", err.c_str());
            if ((s = bind_layout(&L[a], 4, xs, &bd, &err)) != ALT_OK) return fail(h, s, "%s", err.c_str());
            if ((s = transform_bound(h, (int)dtype_size(op.in_dtype), bs, x0, bd, x1, st)) != ALT_OK) return s;
            for (int b = 0; b < nl; ++b) {
                if (kEdgeBlock[b] && op.K % kEdgeBlock[b]) continue;
                alt_conv_desc_t d = op;
                d.variant = -1;
                d.x_layout = L[a];
                d.y_layout = L[b];
                alt_layout_parse(kEdgeWeights[a], &d.w_layout);
                if ((s = alt_pack_weights(h, &d, w0, w1, st)) != ALT_OK) return s;
                float us = INFINITY;
                int v = -1;
                s = tune_variants_conv(h, &d, x1, w1, bias, y, ws, ws_bytes, st, tm, opt_warmup(opts), opt_reps(opts),
                                       per_pair, &plan->trials, &us, &v);
                if (s != ALT_OK) return s;
                if (v < 0) continue;
                op_cost[((size_t)i * nl + a) * nl + b] = us;
                op_var[((size_t)i * nl + a) * nl + b] = v;
                h->cache[conv_key(h, &d)] = TuneEntry{v, us};
                ++h->cache_gen;
            }
        }
    }
    std::vector<int32_t> kind(nnodes), i0(nnodes), i1(nnodes), tl(nnodes + 1), rl(nnodes * 2);
    for (int i = 0; i < nnodes; ++i) { kind[i] = nodes[i].kind; i0[i] = nodes[i].in0; i1[i] = nodes[i].kind == ALT_NODE_ADD ? nodes[i].in1 : 0; }
    float total = 0.f;
    s = alt_plan_graph(nnodes, kind.data(), i0.data(), i1.data(), nl, op_cost.data(), conv_cost.data(), add_cost.data(), in_idx,
                       tl.data(), rl.data(), &total);
    if (s != ALT_OK) return fail(h, s, "no feasible plan");
    plan->nnodes = nnodes;
    plan->total_us = total;
    for (int t = 0; t <= nnodes; ++t) plan->tensor_layout[t] = L[tl[t]];
    auto CC = [&](int t, int a, int b) { return a == b ? 0.f : conv_cost[((size_t)t * nl + a) * nl + b]; };
    double dflt = 0.0;
    for (int i = 0; i < nnodes; ++i) {
        const int nin = nodes[i].kind == ALT_NODE_ADD ? 2 : 1;
        for (int j = 0; j < nin; ++j) {
            const int t = j == 0 ? i0[i] : i1[i];
            const int r = rl[i * 2 + j];
            plan->read_layout[i][j] = L[r];
            plan->convert[i][j] = r != tl[t];
            bool shared = false;                 // an earlier consumer already has this copy made
            for (int i2 = 0; i2 <= i && !shared; ++i2)
                for (int j2 = 0; j2 < 2 && !shared; ++j2) {
                    if (i2 == i && j2 >= j) break;
                    const bool reads = j2 == 0 ? i0[i2] == t : (nodes[i2].kind == ALT_NODE_ADD && i1[i2] == t);
                    shared = reads && rl[i2 * 2 + j2] == r;
                }
            plan->convert_us[i][j] = shared ? 0.f : CC(t, tl[t], r);
        }
        if (nodes[i].kind == ALT_NODE_CONV) {
            const int a = rl[i * 2], b = tl[i + 1];
            alt_conv_desc_t d = nodes[i].conv;
            d.x_layout = L[a];
            d.y_layout = L[b];
            alt_layout_parse(kEdgeWeights[a], &d.w_layout);
            d.variant = op_var[((size_t)i * nl + a) * nl + b];
            plan->conv[i] = d;
            plan->node_us[i] = op_cost[((size_t)i * nl + a) * nl + b];
            dflt += op_cost[((size_t)i * nl + 0) * nl + 0];
        } else {
            plan->node_us[i] = add_cost[i];
            dflt += add_cost[i];
        }
    }
    if (in_idx != 0) dflt += CC(0, in_idx, 0);     // the all-NCHW graph converts its input once
    plan->default_total_us = (float)dflt;

    // sums that a convolution's epilogue can compute (Fig. 6's fused nest)
    for (int i = 0; i < nnodes; ++i) plan->fused_into[i] = -1;
    for (int i = 0; i < nnodes; ++i) {
        if (nodes[i].kind != ALT_NODE_ADD) continue;
        for (int j = 0; j < 2 && plan->fused_into[i] < 0; ++j) {
            if (plan->convert[i][j]) continue;                           // the sum reads the convolution's output as stored
                                                                         // (the other operand may be a converted copy)
            const int t = j == 0 ? i0[i] : i1[i], other = j == 0 ? i1[i] : i0[i];
            const int c = t - 1;                                         // the node that produces tensor t
            if (c < 0 || nodes[c].kind != ALT_NODE_CONV || (nodes[c].conv.epilogue & ALT_EPI_RELU) || other >= t) continue;   // (the other operand exists before the convolution runs)
            if (T[other].dtype != T[t].dtype) continue;
            int readers = 0;
            for (int i2 = 0; i2 < nnodes; ++i2)
                readers += (i0[i2] == t) + (nodes[i2].kind == ALT_NODE_ADD && i1[i2] == t);
            bool already = false;                                        // one sum per epilogue
            for (int i2 = 0; i2 < nnodes; ++i2) already = already || plan->fused_into[i2] == c;
            if (readers != 1 || already) continue;
            alt_conv_desc_t d = plan->conv[c];
            if (nodes[i].relu) d.epilogue |= ALT_EPI_RELU;
            const alt_conv_desc_t &op = nodes[c].conv;
            const int64_t xs[4] = {op.N, op.C, op.H, op.W};
            BoundLayout bs, bd;
            if ((s = bind_layout(&plain_x, 4, xs, &bs, &err)) != ALT_OK) return fail(h, s, "%s", err.c_str());
            if ((s = bind_layout(&d.x_layout, 4, xs, &bd, &err)) != ALT_OK) return fail(h, s, "%s", err.c_str());
            if ((s = transform_bound(h, (int)dtype_size(op.in_dtype), bs, x0, bd, x1, st)) != ALT_OK) return s;
            if ((s = alt_pack_weights(h, &d, w0, w1, st)) != ALT_OK) return s;
            float us = INFINITY;
            // (x0 serves as the addend: any buffer of the output's size does for timing)
            s = measure(h, tm, st, opt_warmup(opts), opt_reps(opts),
                        [&] { return alt_conv2d_add(h, &d, x1, w1, bias, x0, y, ws, ws_bytes, st); }, &us);
            ++plan->trials;
            if (s == ALT_UNSUPPORTED) continue;                          // not a tile-kernel problem
            if (s != ALT_OK) return s;
            if (us < plan->node_us[c] + plan->node_us[i]) {
                plan->total_us -= plan->node_us[c] + plan->node_us[i] - us;
                plan->node_us[c] = us;
                plan->node_us[i] = 0.f;
                plan->conv[c] = d;
                plan->fused_into[i] = c;
            }
        }
    }
    return ALT_OK;
}

alt_status_t alt_tune_conv2d_multi(alt_handle_t h, const alt_conv_call_t *calls, int32_t n, const alt_tune_opts_t *opts,
                                   int32_t *variants, int32_t *order, float *step_us, int32_t *measurements)
{
    if (!h) return ALT_INVALID_ARG;
    if (!calls || !opts || !variants || !order || n < 1 || n > ALT_MAX_MULTI)
        return fail(h, ALT_INVALID_ARG, "alt_tune_conv2d_multi: bad arguments");
    if (!h->has_gpu) return fail(h, ALT_HIP_ERROR, "no GPU device available");
    Timer tm;
    if (!tm.ok) return fail(h, ALT_HIP_ERROR, "hipEventCreate failed");
    const int warmup = opt_warmup(opts), reps = opt_reps(opts);

    struct Cand { int variant; float us; };
    std::vector<Problem> pb(n);
    std::vector<std::vector<Cand>> cands(n);
    std::vector<int> choice(n);
    for (int i = 0; i < n; ++i) {
        const alt_conv_call_t &c = calls[i];
        if (!c.d || !c.x || !c.w || !c.y) return fail(h, ALT_INVALID_ARG, "alt_tune_conv2d_multi: null argument in call %d", i);
        alt_status_t s = conv_problem(h, c.d, c.x, c.w, c.bias, c.y, &pb[i]);
        if (s != ALT_OK) return s;
        if (pb[i].depthwise) return fail(h, ALT_UNSUPPORTED, "alt_tune_conv2d_multi: call %d is depth-wise (no variants)", i);
        const size_t ws_limit = c.workspace ? c.ws_bytes : 0;
        int done = 0;
        for (const Trial &t : ordered_variants(pb[i], ws_limit)) {
            if (opts->max_trials > 0 && done >= opts->max_trials) break;
            float us = 0.f;
            s = measure(h, tm, (hipStream_t)c.stream, warmup, reps,
                        [&] { return igemm_run(h, pb[i], t.variant, c.workspace, ws_limit, (hipStream_t)c.stream); }, &us);
            if (s != ALT_OK) return s;
            ++done;
            cands[i].push_back({t.variant, us});
        }
        if (cands[i].empty()) return fail(h, ALT_UNSUPPORTED, "alt_tune_conv2d_multi: no kernel variant applies to call %d", i);
        std::sort(cands[i].begin(), cands[i].end(), [](const Cand &a, const Cand &b) { return a.us < b.us; });
        size_t keep = 0;
        while (keep < cands[i].size() && keep < 40 && cands[i][keep].us <= 2.f * cands[i][0].us) ++keep;
        cands[i].resize(keep);
        choice[i] = cands[i][0].variant;
        // a variant the caller asked for starts the search if it is among the candidates
        for (const Cand &k : cands[i])
            if (k.variant == c.d->variant) choice[i] = k.variant;
    }

    std::vector<int> ord(n);
    for (int i = 0; i < n; ++i) ord[i] = i;
    auto sync_all = [&]() -> alt_status_t {
        for (int i = 0; i < n; ++i) ALT_CHECK_HIP(h, hipStreamSynchronize((hipStream_t)calls[i].stream));
        return ALT_OK;
    };
    // microseconds per step of the launch under `var` issued in order `o`: median of three runs of `steps`
    auto step_time = [&](const std::vector<int> &var, const std::vector<int> &o, int steps, float *us) -> alt_status_t {
        auto one = [&]() -> alt_status_t {
            for (int k = 0; k < n; ++k) {
                const alt_conv_call_t &c = calls[o[k]];
                alt_status_t s = igemm_run(h, pb[o[k]], var[o[k]], c.workspace, c.workspace ? c.ws_bytes : 0, (hipStream_t)c.stream);
                if (s != ALT_OK) return s;
            }
            return ALT_OK;
        };
        alt_status_t s;
        for (int w = 0; w < 10; ++w)
            if ((s = one()) != ALT_OK) return s;
        if ((s = sync_all()) != ALT_OK) return s;
        float t[3];
        for (int r = 0; r < 3; ++r) {
            const auto t0 = std::chrono::steady_clock::now();
            for (int k = 0; k < steps; ++k)
                if ((s = one()) != ALT_OK) return s;
            if ((s = sync_all()) != ALT_OK) return s;
            t[r] = std::chrono::duration<float, std::micro>(std::chrono::steady_clock::now() - t0).count() / steps;
        }
        std::sort(t, t + 3);
        *us = t[1];
        return ALT_OK;
    };

    int nmeas = 0;
    float best = 0.f;
    alt_status_t s = step_time(choice, ord, 300, &best);
    if (s != ALT_OK) return s;
    ++nmeas;
    for (int round = 0; round < 3; ++round) {
        bool improved = false;
        for (int i = 0; i < n; ++i)
            for (const Cand &k : cands[i]) {
                if (k.variant == choice[i]) continue;
                std::vector<int> trial = choice;
                trial[i] = k.variant;
                float us = 0.f;
                if ((s = step_time(trial, ord, 150, &us)) != ALT_OK) return s;
                ++nmeas;
                if (us >= best * 0.985f) continue;
                if ((s = step_time(trial, ord, 300, &us)) != ALT_OK) return s;   // confirm before taking it
                ++nmeas;
                if (us < best * 0.99f) { best = us; choice = trial; improved = true; }
            }
        if (!improved) break;
    }
    if (n <= 5) {
        std::vector<int> perm = ord, best_ord = ord;
        while (std::next_permutation(perm.begin(), perm.end())) {
            float us = 0.f;
            if ((s = step_time(choice, perm, 100, &us)) != ALT_OK) return s;
            ++nmeas;
            if (us >= best * 0.985f) continue;
            if ((s = step_time(choice, perm, 300, &us)) != ALT_OK) return s;
            ++nmeas;
            if (us < best * 0.99f) { best = us; best_ord = perm; }
        }
        ord = best_ord;
    }
    for (int i = 0; i < n; ++i) { variants[i] = choice[i]; order[i] = ord[i]; }
    if (step_us) *step_us = best;
    if (measurements) *measurements = nmeas;
    return ALT_OK;
}

alt_status_t alt_cache_save(alt_handle_t h, const char *path)
{
    if (!h) return ALT_INVALID_ARG;
    if (!path) return fail(h, ALT_INVALID_ARG, "null path");
    std::ofstream f(path);
    if (!f) return fail(h, ALT_INVALID_ARG, "cannot open %s for writing", path);
    f << "# alt tune cache v1: key <tab> variant-name <tab> microseconds\n";
    for (auto &kv : h->cache) f << kv.first << "\t" << igemm_variant_name(kv.second.variant) << "\t" << kv.second.us << "\n";
    return f.good() ? ALT_OK : fail(h, ALT_INVALID_ARG, "write to %s failed", path);
}

alt_status_t alt_cache_load(alt_handle_t h, const char *path)
{
    if (!h) return ALT_INVALID_ARG;
    if (!path) return fail(h, ALT_INVALID_ARG, "null path");
    std::ifstream f(path);
    if (!f) return fail(h, ALT_INVALID_ARG, "cannot open %s", path);
    std::map<std::string, int> by_name;
    for (int v = 0; v < igemm_variant_count(); ++v) by_name[igemm_variant_name(v)] = v;
    std::string line;
    while (std::getline(f, line)) {
        if (line.empty() || line[0] == '#') continue;
        size_t t1 = line.find('\t'), t2 = line.find('\t', t1 == std::string::npos ? 0 : t1 + 1);
        if (t1 == std::string::npos || t2 == std::string::npos) return fail(h, ALT_INVALID_ARG, "malformed cache line");
        auto it = by_name.find(line.substr(t1 + 1, t2 - t1 - 1));
        if (it == by_name.end()) continue;             // a variant this build does not have
        h->cache[line.substr(0, t1)] = TuneEntry{it->second, (float)std::atof(line.c_str() + t2 + 1)};
    }
    ++h->cache_gen;
    return ALT_OK;
}

alt_status_t alt_cache_clear(alt_handle_t h)
{
    if (!h) return ALT_INVALID_ARG;
    h->cache.clear();
    ++h->cache_gen;
    return ALT_OK;
}

}  // extern "C"

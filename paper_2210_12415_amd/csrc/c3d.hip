// 3-D convolution (C3D in the operator list of Section 6.1 of the paper) on the 2-D kernels.
// Unfolding the depth into tiles of T slices every stride_d (the unfold primitive of Section
// 4.1.2, Eq. 1, with zero slices for the depth padding) and placing the tile index beside the
// channels turns the T depth taps into T*C input channels of a 2-D convolution whose batch is
// (n, od):
//   y[(n,od),k,oh,ow] = sum_{(t,c),r,s} x'[(n,od),(t,c),ih,iw] * w'[k,(t,c),r,s],
//   x'[(n,od),(t,c),h,w] = x[(n, od*stride_d - pad_d + t*dil_d), c, h, w]  (zero outside the depth),
//   w'[k,(t,c),r,s]      = w[k,c,t,r,s].
// One kernel writes x' under the activation layout into the workspace per call, one writes
// w' once, offline (a weight tensor is a constant, Section 4.2); alt_conv2d does the work.
//
// The transposed 3-D convolution (T3D of the same list) is the forward one at stride 1 over x
// with stride-1 zeros between its elements in all three directions, with the filter mirrored,
// its channel dimensions exchanged and padding dil*(T-1)-pad: the same two kernels, the
// first reading x[.., d/stride_d, h/stride_h, w/stride_w] where all three divide and zero
// elsewhere, the second reading the filter back to front.  Where the output extents are multiples
// of the strides and the taps of the stride_d*stride_h*stride_w output phases fit one symmetric
// window per direction (4x4x4 at stride 2 with padding 1, 2x2x2 at stride 2, ...) it takes the
// sub-pixel form instead: the phases are stride-1 convolutions of x itself, merged into one
// forward 3-D convolution with that many times K output channels over the common window, whose
// result a last kernel moves into place; no inserted zeros are multiplied.
#include <hip/hip_runtime.h>

#include <string>

#include "common.h"
#include "fast_layout.h"
#include "layout_eval.h"
#include "ops.h"
#include "subpixel.h"

namespace alt {
namespace {

constexpr int kC3dThreads = 256;

template <int BYTES> struct Word;
template <> struct Word<2> { using type = uint16_t; };
template <> struct Word<4> { using type = uint32_t; };
template <> struct Word<16> { using type = uint4; };

struct GatherParams {
    const void *src;
    void *dst;
    BoundLayout ls, ld;           // x over (N*D, C, H, W); x' over (N*OD, T*C, He, We)
    int64_t D, OD, C;
    int32_t sd, pd, dd;           // depth stride, padding, dilation of the forward problem
    int32_t zd, zh, zw;           // x sits at every zd-th slice, zh-th row, zw-th column of the tensor convolved (1: x itself)
};

// One thread per element of x', any pair of layouts.
template <int ELSZ>
__global__ __launch_bounds__(kC3dThreads) void c3d_gather_kernel(GatherParams p)
{
    using E = typename Word<ELSZ>::type;
    const int64_t n = p.ld.numel;
    for (int64_t e = blockIdx.x * (int64_t)kC3dThreads + threadIdx.x; e < n; e += (int64_t)gridDim.x * kC3dThreads) {
        int64_t idx[ALT_MAX_RANK];
        int64_t r = e;
        for (int d = 3; d >= 0; --d) { idx[d] = r % p.ld.shape[d]; r /= p.ld.shape[d]; }
        const int64_t out = eval_offset(p.ld, idx);
        const int64_t img = idx[0] / p.OD, od = idx[0] - img * p.OD;
        const int64_t t = idx[1] / p.C, c = idx[1] - t * p.C;
        const int64_t de = od * p.sd - p.pd + t * p.dd;
        E v = 0;
        if (de >= 0 && de % p.zd == 0 && de / p.zd < p.D && idx[2] % p.zh == 0 && idx[3] % p.zw == 0) {
            idx[0] = img * p.D + de / p.zd;
            idx[1] = c;
            idx[2] /= p.zh;
            idx[3] /= p.zw;
            v = ((const E *)p.src)[eval_offset(p.ls, idx)];
        }
        ((E *)p.dst)[out] = v;
    }
}

struct GatherFastParams {
    const void *src;
    void *dst;
    FastLayout ls, ld;
    FastDiv by_od, by_c, by_zd, by_zh, by_zw;
    uint32_t D, nvec;
    int32_t sd, pd, dd, pad_;
};

// The same for separable layouts with fewer than 2^31 elements, walked in the order of the
// memory of x': a thread owns VEC consecutive elements there (16 bytes of a run along the
// channels or along a row when both layouts end in such a run), recovers their logical
// index from the offset digit by digit and copies them from x.  32-bit arithmetic,
// divisions by multiplication.
template <int ELSZ, int VEC>
__global__ __launch_bounds__(kC3dThreads) void c3d_gather_fast_kernel(GatherFastParams p)
{
    using V = typename Word<ELSZ * VEC>::type;
    for (uint32_t v = blockIdx.x * kC3dThreads + threadIdx.x; v < p.nvec; v += gridDim.x * kC3dThreads) {
        const uint32_t o = v * VEC;
        uint32_t idx[4] = {0, 0, 0, 0};
        for (int j = 0; j < p.ld.n; ++j) {
            const FastAtom &a = p.ld.a[j];
            idx[a.dim] += fast_mod(fast_div(o, a.by_stride), a.by_ext) * a.div;
        }
        const uint32_t img = fast_div(idx[0], p.by_od), od = idx[0] - img * p.by_od.d;
        const uint32_t t = fast_div(idx[1], p.by_c), c = idx[1] - t * p.by_c.d;
        const int32_t de = (int32_t)od * p.sd - p.pd + (int32_t)t * p.dd;
        const uint32_t d = fast_div((uint32_t)de, p.by_zd), qh = fast_div(idx[2], p.by_zh), qw = fast_div(idx[3], p.by_zw);
        V w;
        __builtin_memset(&w, 0, sizeof w);
        if (de >= 0 && d * p.by_zd.d == (uint32_t)de && d < p.D && qh * p.by_zh.d == idx[2] && qw * p.by_zw.d == idx[3]) {
            idx[0] = img * p.D + d;
            idx[1] = c;
            idx[2] = qh;
            idx[3] = qw;
            uint32_t so = 0;
            for (int j = 0; j < p.ls.n; ++j) {
                const FastAtom &a = p.ls.a[j];
                so += fast_mod(fast_div(idx[a.dim], a.by_div), a.by_ext) * a.stride;
            }
            w = *(const V *)((const char *)p.src + (size_t)so * ELSZ);
        }
        *(V *)((char *)p.dst + (size_t)o * ELSZ) = w;
    }
}

// Elements per thread: 16 bytes' worth when both layouts end in a contiguous run of the same
// logical dimension (channels or width), whole in that dimension's innermost piece, with
// extents (and, for channels, C itself: a run may not cross from one depth tap to the next)
// that are multiples of it; else one.
int gather_vec(const BoundLayout &ls, const BoundLayout &ld, int elsz, int64_t C, int zw, const void *src, const void *dst)
{
    const int want = 16 / elsz;
    const Atom *is = unit_stride_atom(ls), *id = unit_stride_atom(ld);
    if (!is || !id || is->dim != id->dim || (is->dim != 1 && is->dim != 3) || is->div != 1 || id->div != 1) return 1;
    if (is->dim == 3 && zw != 1) return 1;                 // zeros between the elements of a row: no common run
    if (is->ext % want || id->ext % want || (is->dim == 1 && C % want)) return 1;
    if ((uintptr_t)src % 16 || (uintptr_t)dst % 16) return 1;
    return want;
}

struct PackParams {
    const void *src;              // dense (K, C, T, R, S); (C, K, T, R, S) for the transposed operator
    void *dst;
    BoundLayout ld;               // w' over (K, T*C, R, S) under w_layout
    int64_t C, T;
    int32_t mirrored, pad_;
};

// w'[k, t*C + c, r, s] = w[k, c, t, r, s], or w[c, k, T-1-t, R-1-r, S-1-s] for the transposed operator;
// one thread per element.
template <int ELSZ>
__global__ __launch_bounds__(kC3dThreads) void c3d_pack_kernel(PackParams p)
{
    using E = typename Word<ELSZ>::type;
    const int64_t n = p.ld.numel;
    const int64_t R = p.ld.shape[2], S = p.ld.shape[3];
    for (int64_t e = blockIdx.x * (int64_t)kC3dThreads + threadIdx.x; e < n; e += (int64_t)gridDim.x * kC3dThreads) {
        int64_t idx[ALT_MAX_RANK];
        int64_t r = e;
        for (int d = 3; d >= 0; --d) { idx[d] = r % p.ld.shape[d]; r /= p.ld.shape[d]; }
        const int64_t t = idx[1] / p.C, c = idx[1] - t * p.C;
        const int64_t K = p.ld.shape[0];
        const int64_t src = p.mirrored ? ((((c * K + idx[0]) * p.T + (p.T - 1 - t)) * R + (R - 1 - idx[2])) * S + (S - 1 - idx[3]))
                                       : ((((idx[0] * p.C + c) * p.T + t) * R + idx[2]) * S + idx[3]);
        ((E *)p.dst)[eval_offset(p.ld, idx)] = ((const E *)p.src)[src];
    }
}

struct Merge3dParams {
    const void *src;              // dense (C, K, T, R, S)
    void *dst;
    BoundLayout ld;               // the merged filter over (K', Tm*C, Rm, Sm) under w_layout
    int64_t C, K, T, R, S;
    int32_t sd, sh, sw, pad_d, pad_h, pad_w, dil_d, dil_h, dil_w, pm_d, pm_h, pm_w;
};

// w_m[((pd*sh + ph)*sw + pw)*K + k, a_d*C + c, a, b] = w[c, k, t, r, s] for the tap with
// t*dil_d = pd + pad_d - sd*(a_d - pm_d), r*dil_h = ph + pad_h - sh*(a - pm_h), s*dil_w = pw + pad_w - sw*(b - pm_w);
// zero if there is none.  One thread per element.
template <int ELSZ>
__global__ __launch_bounds__(kC3dThreads) void c3d_merge_kernel(Merge3dParams p)
{
    using E = typename Word<ELSZ>::type;
    const int64_t n = p.ld.numel;
    for (int64_t e = blockIdx.x * (int64_t)kC3dThreads + threadIdx.x; e < n; e += (int64_t)gridDim.x * kC3dThreads) {
        int64_t idx[ALT_MAX_RANK];
        int64_t rem = e;
        for (int d = 3; d >= 0; --d) { idx[d] = rem % p.ld.shape[d]; rem /= p.ld.shape[d]; }
        const int64_t phase = idx[0] / p.K, k = idx[0] - phase * p.K;
        const int64_t pd = phase / (p.sh * p.sw), phw = phase - pd * (p.sh * p.sw), ph = phw / p.sw, pw = phw - ph * p.sw;
        const int64_t ad = idx[1] / p.C, c = idx[1] - ad * p.C;
        const int64_t nt = pd + p.pad_d - p.sd * (ad - p.pm_d), nr = ph + p.pad_h - p.sh * (idx[2] - p.pm_h),
                      ns = pw + p.pad_w - p.sw * (idx[3] - p.pm_w);
        E v = 0;
        if (nt >= 0 && nr >= 0 && ns >= 0 && nt % p.dil_d == 0 && nr % p.dil_h == 0 && ns % p.dil_w == 0 && nt / p.dil_d < p.T &&
            nr / p.dil_h < p.R && ns / p.dil_w < p.S)
            v = ((const E *)p.src)[(((c * p.K + k) * p.T + nt / p.dil_d) * p.R + nr / p.dil_h) * p.S + ns / p.dil_w];
        ((E *)p.dst)[eval_offset(p.ld, idx)] = v;
    }
}

unsigned blocks_for(int64_t n)
{
    const int64_t b = (n + kC3dThreads - 1) / kC3dThreads;
    return (unsigned)(b < 1 ? 1 : b > 256 * 64 ? 256 * 64 : b);
}

size_t round256(size_t n) { return (n + 255) / 256 * 256; }

int64_t out_depth(const alt_conv3d_desc_t *d)
{
    const int64_t span = d->D + 2 * (int64_t)d->pad_d - (int64_t)d->dil_d * (d->T - 1) - 1;
    return span < 0 ? 0 : span / d->stride_d + 1;
}

// What the two kernels and alt_conv2d need to know of a 3-D problem.
struct Problem3d {
    alt_conv_desc_t f;            // the 2-D problem: batch N*OD, T*C channels
    int64_t xs[4];                // x as a stack of slices: (N*D, C, H, W)
    int64_t D, OD, C;
    int32_t sd, pd, dd;           // depth stride, padding, dilation of the forward problem
    int32_t zd, zh, zw;           // zero-insertion strides (1 for the forward operator)
    bool gather;                  // false: the 2-D problem reads x itself
};

// The forward operator.
alt_status_t forward_problem(alt_handle_t h, const alt_conv3d_desc_t *d, Problem3d *out, const char *who = "alt_conv3d")
{
    const alt_conv_desc_t &q = d->plane;
    if (q.N < 1 || q.C < 1 || q.H < 1 || q.W < 1 || d->D < 1 || d->T < 1) return fail(h, ALT_INVALID_ARG, "%s: extents must be positive", who);
    if (d->stride_d < 1 || d->dil_d < 1 || d->pad_d < 0) return fail(h, ALT_INVALID_ARG, "%s: bad depth stride, padding or dilation", who);
    if (q.groups > 1) return fail(h, ALT_UNSUPPORTED, "%s: groups are not supported", who);
    const int64_t OD = out_depth(d);
    if (OD < 1) return fail(h, ALT_INVALID_ARG, "%s: the filter is deeper than the padded input", who);
    Problem3d &p = *out;
    p.f = q;
    p.f.N = q.N * OD;
    p.f.C = q.C * d->T;
    p.xs[0] = q.N * d->D; p.xs[1] = q.C; p.xs[2] = q.H; p.xs[3] = q.W;
    p.D = d->D; p.OD = OD; p.C = q.C;
    p.sd = d->stride_d; p.pd = d->pad_d; p.dd = d->dil_d;
    p.zd = p.zh = p.zw = 1;
    p.gather = !(d->T == 1 && d->stride_d == 1 && d->pad_d == 0);
    return ALT_OK;
}

int64_t transposed_extent(int64_t in, int stride, int pad, int dil, int64_t taps)
{
    return (in - 1) * stride - 2 * (int64_t)pad + (int64_t)dil * (taps - 1) + 1;
}

// The transposed operator as the forward one over the zero-inserted input.
alt_status_t transposed_problem(alt_handle_t h, const alt_conv3d_desc_t *d, Problem3d *out)
{
    const alt_conv_desc_t &q = d->plane;
    if (q.N < 1 || q.C < 1 || q.H < 1 || q.W < 1 || q.K < 1 || q.R < 1 || q.S < 1 || d->D < 1 || d->T < 1)
        return fail(h, ALT_INVALID_ARG, "alt_conv3d_transpose: extents must be positive");
    if (d->stride_d < 1 || q.stride_h < 1 || q.stride_w < 1 || d->dil_d < 1 || q.dil_h < 1 || q.dil_w < 1 || d->pad_d < 0 ||
        q.pad_h < 0 || q.pad_w < 0)
        return fail(h, ALT_INVALID_ARG, "alt_conv3d_transpose: bad stride, padding or dilation");
    if (q.groups > 1) return fail(h, ALT_UNSUPPORTED, "alt_conv3d_transpose: groups are not supported");
    if (d->pad_d > d->dil_d * (d->T - 1) || q.pad_h > q.dil_h * (q.R - 1) || q.pad_w > q.dil_w * (q.S - 1))
        return fail(h, ALT_UNSUPPORTED, "alt_conv3d_transpose: padding beyond dil*(taps-1) is not supported");
    Problem3d &p = *out;
    p.OD = transposed_extent(d->D, d->stride_d, d->pad_d, d->dil_d, d->T);
    if (p.OD < 1) return fail(h, ALT_INVALID_ARG, "alt_conv3d_transpose: empty output");
    p.f = q;
    p.f.N = q.N * p.OD;
    p.f.C = q.C * d->T;
    p.f.H = (q.H - 1) * q.stride_h + 1;
    p.f.W = (q.W - 1) * q.stride_w + 1;
    p.f.stride_h = p.f.stride_w = 1;
    p.f.pad_h = q.dil_h * (int32_t)(q.R - 1) - q.pad_h;
    p.f.pad_w = q.dil_w * (int32_t)(q.S - 1) - q.pad_w;
    p.xs[0] = q.N * d->D; p.xs[1] = q.C; p.xs[2] = q.H; p.xs[3] = q.W;
    p.D = d->D; p.C = q.C;
    p.sd = 1; p.pd = d->dil_d * (int32_t)(d->T - 1) - d->pad_d; p.dd = d->dil_d;
    p.zd = d->stride_d; p.zh = q.stride_h; p.zw = q.stride_w;
    p.gather = !(d->T == 1 && d->stride_d == 1 && d->pad_d == 0 && q.stride_h == 1 && q.stride_w == 1);
    return ALT_OK;
}

// The sub-pixel form of the transposed operator: the merged forward 3-D problem on x itself.
struct SubPixel3d {
    alt_conv3d_desc_t m;          // forward descriptor: K' output channels, merged filter extents, stride 1
    Problem3d pr;                 // its 2-D problem
    PhaseAxis ad, ah, aw;
};

// Whether the descriptor takes the sub-pixel form (decided from the descriptor alone, so the weight pack,
// the workspace size and the call agree).
bool subpixel3d_plan(alt_handle_t h, const alt_conv3d_desc_t *d, SubPixel3d *out)
{
    const alt_conv_desc_t &q = d->plane;
    if (d->stride_d == 1 && q.stride_h == 1 && q.stride_w == 1) return false;
    if (d->stride_d > 8 || q.stride_h > 8 || q.stride_w > 8) return false;
    SubPixel3d &s = *out;
    s.ad = phase_axis(d->D, d->T, d->stride_d, d->pad_d, d->dil_d);
    s.ah = phase_axis(q.H, q.R, q.stride_h, q.pad_h, q.dil_h);
    s.aw = phase_axis(q.W, q.S, q.stride_w, q.pad_w, q.dil_w);
    if (!s.ad.ok || !s.ah.ok || !s.aw.ok) return false;
    s.m = *d;
    s.m.plane.K = q.K * d->stride_d * q.stride_h * q.stride_w;
    s.m.plane.R = s.ah.taps;
    s.m.plane.S = s.aw.taps;
    s.m.plane.stride_h = s.m.plane.stride_w = 1;
    s.m.plane.dil_h = s.m.plane.dil_w = 1;
    s.m.plane.pad_h = s.ah.pad;
    s.m.plane.pad_w = s.aw.pad;
    s.m.T = s.ad.taps;
    s.m.stride_d = 1;
    s.m.dil_d = 1;
    s.m.pad_d = s.ad.pad;
    // the filter and output layouts must take the merged extents
    BoundLayout b;
    std::string err;
    const int64_t ws[4] = {s.m.plane.K, q.C * s.m.T, s.m.plane.R, s.m.plane.S};
    const int64_t ys[4] = {q.N * s.ad.outq, s.m.plane.K, s.ah.outq, s.aw.outq};
    if (bind_layout(&q.w_layout, 4, ws, &b, &err) != ALT_OK) return false;
    if (bind_layout(&q.y_layout, 4, ys, &b, &err) != ALT_OK) return false;
    return forward_problem(h, &s.m, &s.pr, "alt_conv3d_transpose") == ALT_OK && s.pr.OD == s.ad.outq;
}

size_t gathered_bytes(const Problem3d &p)
{
    return round256((size_t)(p.f.N * p.f.C * p.f.H * p.f.W) * dtype_size(p.f.in_dtype));
}

alt_status_t workspace_size(alt_handle_t h, const Problem3d &p, size_t *bytes)
{
    size_t conv_ws = 0;
    const alt_status_t s = alt_conv2d_workspace_size(h, &p.f, &conv_ws);
    if (s != ALT_OK) return s;
    *bytes = (p.gather ? gathered_bytes(p) : 0) + conv_ws;
    return ALT_OK;
}

alt_status_t pack3d(alt_handle_t h, const alt_conv3d_desc_t *d, const void *w, void *w_packed, void *stream, bool mirrored,
                    const char *who)
{
    if (!d || !w || !w_packed) return fail(h, ALT_INVALID_ARG, "%s: null argument", who);
    const alt_conv_desc_t &q = d->plane;
    if (q.in_dtype != ALT_F32 && q.in_dtype != ALT_BF16) return fail(h, ALT_INVALID_ARG, "%s: bad dtype", who);
    if (q.K < 1 || q.C < 1 || q.R < 1 || q.S < 1 || d->T < 1) return fail(h, ALT_INVALID_ARG, "%s: extents must be positive", who);
    if (!h->has_gpu) return fail(h, ALT_HIP_ERROR, "no GPU device available");
    const int64_t wsh[4] = {q.K, q.C * d->T, q.R, q.S};
    PackParams p;
    std::string err;
    const alt_status_t s = bind_layout(&q.w_layout, 4, wsh, &p.ld, &err);
    if (s != ALT_OK) return fail(h, s, "w_layout: %s", err.c_str());
    p.src = w;
    p.dst = w_packed;
    p.C = q.C;
    p.T = d->T;
    p.mirrored = mirrored ? 1 : 0;
    p.pad_ = 0;
    hipStream_t st = (hipStream_t)stream;
    if (dtype_size(q.in_dtype) == 2) hipLaunchKernelGGL(c3d_pack_kernel<2>, dim3(blocks_for(p.ld.numel)), dim3(kC3dThreads), 0, st, p);
    else hipLaunchKernelGGL(c3d_pack_kernel<4>, dim3(blocks_for(p.ld.numel)), dim3(kC3dThreads), 0, st, p);
    ALT_CHECK_HIP(h, hipGetLastError());
    return ALT_OK;
}

alt_status_t run3d(alt_handle_t h, const Problem3d &pr, const void *x, const void *w_packed, const float *bias, void *y,
                   void *workspace, size_t ws_bytes, void *stream, const char *who)
{
    if (!pr.gather) return alt_conv2d(h, &pr.f, x, w_packed, bias, y, workspace, ws_bytes, stream);

    if (!h->has_gpu) return fail(h, ALT_HIP_ERROR, "no GPU device available");
    const alt_conv_desc_t &f = pr.f;
    const int elsz = (int)dtype_size(f.in_dtype);
    const size_t xu_bytes = gathered_bytes(pr);
    if (!workspace || ws_bytes < xu_bytes)
        return fail(h, ALT_WORKSPACE_TOO_SMALL, "%s: the workspace must hold the depth-unfolded input (%zu bytes)", who, xu_bytes);
    if ((uintptr_t)workspace % 16) return fail(h, ALT_INVALID_ARG, "%s: workspace must be 16-byte aligned", who);
    GatherParams p;
    const int64_t us[4] = {f.N, f.C, f.H, f.W};
    std::string err;
    alt_status_t s;
    if ((s = bind_layout(&f.x_layout, 4, pr.xs, &p.ls, &err)) != ALT_OK) return fail(h, s, "x_layout: %s", err.c_str());
    if ((s = bind_layout(&f.x_layout, 4, us, &p.ld, &err)) != ALT_OK) return fail(h, s, "x_layout (depth-unfolded input): %s", err.c_str());
    p.src = x;
    p.dst = workspace;
    p.D = pr.D; p.OD = pr.OD; p.C = pr.C;
    p.sd = pr.sd; p.pd = pr.pd; p.dd = pr.dd;
    p.zd = pr.zd; p.zh = pr.zh; p.zw = pr.zw;
    hipStream_t st = (hipStream_t)stream;
    GatherFastParams g;
    const int64_t T = f.C / pr.C;
    const bool small = pr.D < ((int64_t)1 << 20) && pr.OD < ((int64_t)1 << 20) && T < ((int64_t)1 << 10) &&
                       (int64_t)pr.sd * pr.OD + (int64_t)pr.dd * T + pr.pd < ((int64_t)1 << 30);
    if (small && fast_layout(p.ls, &g.ls) && fast_layout(p.ld, &g.ld)) {
        const int vec = gather_vec(p.ls, p.ld, elsz, pr.C, pr.zw, x, workspace);
        g.src = x;
        g.dst = workspace;
        g.by_od = make_fastdiv((uint32_t)pr.OD);
        g.by_c = make_fastdiv((uint32_t)pr.C);
        g.by_zd = make_fastdiv((uint32_t)pr.zd);
        g.by_zh = make_fastdiv((uint32_t)pr.zh);
        g.by_zw = make_fastdiv((uint32_t)pr.zw);
        g.D = (uint32_t)pr.D;
        g.nvec = (uint32_t)(p.ld.numel / vec);
        g.sd = pr.sd;
        g.pd = pr.pd;
        g.dd = pr.dd;
        g.pad_ = 0;
        const dim3 grid(blocks_for(g.nvec)), block(kC3dThreads);
        if (elsz == 2 && vec == 8) hipLaunchKernelGGL((c3d_gather_fast_kernel<2, 8>), grid, block, 0, st, g);
        else if (elsz == 2) hipLaunchKernelGGL((c3d_gather_fast_kernel<2, 1>), grid, block, 0, st, g);
        else if (vec == 4) hipLaunchKernelGGL((c3d_gather_fast_kernel<4, 4>), grid, block, 0, st, g);
        else hipLaunchKernelGGL((c3d_gather_fast_kernel<4, 1>), grid, block, 0, st, g);
    } else if (elsz == 2) {
        hipLaunchKernelGGL(c3d_gather_kernel<2>, dim3(blocks_for(p.ld.numel)), dim3(kC3dThreads), 0, st, p);
    } else {
        hipLaunchKernelGGL(c3d_gather_kernel<4>, dim3(blocks_for(p.ld.numel)), dim3(kC3dThreads), 0, st, p);
    }
    ALT_CHECK_HIP(h, hipGetLastError());
    return alt_conv2d(h, &f, workspace, w_packed, bias, y, (char *)workspace + xu_bytes, ws_bytes - xu_bytes, stream);
}

size_t subpixel3d_y_bytes(const SubPixel3d &s)
{
    return round256((size_t)(s.pr.f.N * s.pr.f.K * s.ah.outq * s.aw.outq) * dtype_size(s.pr.f.out_dtype));
}
size_t subpixel3d_bias_bytes(const SubPixel3d &s) { return round256((size_t)s.pr.f.K * sizeof(float)); }

// Workspace: the phase-major output y', the replicated bias, then what the forward 3-D problem wants.
alt_status_t run_subpixel3d(alt_handle_t h, const alt_conv3d_desc_t *d, const SubPixel3d &s, const void *x, const void *w_packed,
                            const float *bias, void *y, void *workspace, size_t ws_bytes, void *stream)
{
    if (!h->has_gpu) return fail(h, ALT_HIP_ERROR, "no GPU device available");
    const alt_conv_desc_t &q = d->plane;
    const size_t yb = subpixel3d_y_bytes(s), bb = subpixel3d_bias_bytes(s);
    if (!workspace || ws_bytes < yb + bb)
        return fail(h, ALT_WORKSPACE_TOO_SMALL, "alt_conv3d_transpose: the workspace must hold the phase-major output (%zu bytes)", yb + bb);
    if ((uintptr_t)workspace % 16 || (uintptr_t)y % 16) return fail(h, ALT_INVALID_ARG, "alt_conv3d_transpose: workspace and y must be 16-byte aligned");
    if ((q.epilogue & ALT_EPI_BIAS) && !bias) return fail(h, ALT_INVALID_ARG, "alt_conv3d_transpose: ALT_EPI_BIAS without a bias");
    hipStream_t st = (hipStream_t)stream;
    float *bias_m = (float *)((char *)workspace + yb);
    alt_status_t st_;
    if (q.epilogue & ALT_EPI_BIAS)
        if ((st_ = phase_bias(h, bias, bias_m, q.K, s.pr.f.K, st)) != ALT_OK) return st_;
    st_ = run3d(h, s.pr, x, w_packed, (q.epilogue & ALT_EPI_BIAS) ? bias_m : nullptr, workspace, (char *)workspace + yb + bb,
                ws_bytes - yb - bb, stream, "alt_conv3d_transpose");
    if (st_ != ALT_OK) return st_;
    return phase_shuffle(h, &q.y_layout, q.N, q.K, s.ad.outq, s.ah.outq, s.aw.outq, d->stride_d, q.stride_h, q.stride_w,
                         (int)dtype_size(q.out_dtype), workspace, y, st);
}

}  // namespace
}  // namespace alt

using namespace alt;

extern "C" alt_status_t alt_conv3d_output_shape(const alt_conv3d_desc_t *d, int64_t *out)
{
    if (!d || !out) return ALT_INVALID_ARG;
    if (d->D < 1 || d->T < 1 || d->stride_d < 1 || d->dil_d < 1 || d->pad_d < 0) return ALT_INVALID_ARG;
    int64_t o4[4];
    const alt_status_t s = alt_conv2d_output_shape(&d->plane, o4);
    if (s != ALT_OK) return s;
    const int64_t OD = out_depth(d);
    if (OD < 1) return ALT_INVALID_ARG;
    out[0] = o4[0];
    out[1] = o4[1];
    out[2] = OD;
    out[3] = o4[2];
    out[4] = o4[3];
    return ALT_OK;
}

extern "C" alt_status_t alt_conv3d_problem(alt_handle_t h, const alt_conv3d_desc_t *d, alt_conv_desc_t *out)
{
    if (!h) return ALT_INVALID_ARG;
    if (!d || !out) return fail(h, ALT_INVALID_ARG, "null argument");
    Problem3d p;
    const alt_status_t s = forward_problem(h, d, &p);
    if (s == ALT_OK) *out = p.f;
    return s;
}

extern "C" alt_status_t alt_conv3d_transpose_problem(alt_handle_t h, const alt_conv3d_desc_t *d, alt_conv_desc_t *out)
{
    if (!h) return ALT_INVALID_ARG;
    if (!d || !out) return fail(h, ALT_INVALID_ARG, "null argument");
    Problem3d p;
    const alt_status_t s = transposed_problem(h, d, &p);
    if (s != ALT_OK) return s;
    SubPixel3d sp;
    *out = subpixel3d_plan(h, d, &sp) ? sp.pr.f : p.f;
    return ALT_OK;
}

extern "C" alt_status_t alt_conv3d_workspace_size(alt_handle_t h, const alt_conv3d_desc_t *d, size_t *bytes)
{
    if (!h) return ALT_INVALID_ARG;
    if (!d || !bytes) return fail(h, ALT_INVALID_ARG, "null argument");
    Problem3d p;
    const alt_status_t s = forward_problem(h, d, &p);
    return s != ALT_OK ? s : workspace_size(h, p, bytes);
}

extern "C" alt_status_t alt_pack_weights3d(alt_handle_t h, const alt_conv3d_desc_t *d, const void *w_kctrs,
                                           void *w_packed, void *stream)
{
    if (!h) return ALT_INVALID_ARG;
    return pack3d(h, d, w_kctrs, w_packed, stream, false, "alt_pack_weights3d");
}

extern "C" alt_status_t alt_conv3d(alt_handle_t h, const alt_conv3d_desc_t *d, const void *x, const void *w_packed,
                                   const float *bias, void *y, void *workspace, size_t ws_bytes, void *stream)
{
    if (!h) return ALT_INVALID_ARG;
    if (!d || !x || !w_packed || !y) return fail(h, ALT_INVALID_ARG, "alt_conv3d: null argument");
    if (d->plane.in_dtype != ALT_F32 && d->plane.in_dtype != ALT_BF16) return fail(h, ALT_INVALID_ARG, "alt_conv3d: bad dtype");
    Problem3d p;
    const alt_status_t s = forward_problem(h, d, &p);
    return s != ALT_OK ? s : run3d(h, p, x, w_packed, bias, y, workspace, ws_bytes, stream, "alt_conv3d");
}

extern "C" alt_status_t alt_conv3d_transpose_output_shape(const alt_conv3d_desc_t *d, int64_t *out)
{
    if (!d || !out) return ALT_INVALID_ARG;
    const alt_conv_desc_t &q = d->plane;
    if (d->stride_d < 1 || q.stride_h < 1 || q.stride_w < 1 || d->dil_d < 1 || q.dil_h < 1 || q.dil_w < 1) return ALT_INVALID_ARG;
    out[0] = q.N;
    out[1] = q.K;
    out[2] = transposed_extent(d->D, d->stride_d, d->pad_d, d->dil_d, d->T);
    out[3] = transposed_extent(q.H, q.stride_h, q.pad_h, q.dil_h, q.R);
    out[4] = transposed_extent(q.W, q.stride_w, q.pad_w, q.dil_w, q.S);
    return (out[2] < 1 || out[3] < 1 || out[4] < 1) ? ALT_INVALID_ARG : ALT_OK;
}

extern "C" alt_status_t alt_conv3d_transpose_workspace_size(alt_handle_t h, const alt_conv3d_desc_t *d, size_t *bytes)
{
    if (!h) return ALT_INVALID_ARG;
    if (!d || !bytes) return fail(h, ALT_INVALID_ARG, "null argument");
    Problem3d p;
    const alt_status_t s = transposed_problem(h, d, &p);
    if (s != ALT_OK) return s;
    SubPixel3d sp;
    if (subpixel3d_plan(h, d, &sp)) {
        size_t inner = 0;
        const alt_status_t s2 = workspace_size(h, sp.pr, &inner);
        if (s2 != ALT_OK) return s2;
        *bytes = subpixel3d_y_bytes(sp) + subpixel3d_bias_bytes(sp) + inner;
        return ALT_OK;
    }
    return workspace_size(h, p, bytes);
}

extern "C" alt_status_t alt_pack_weights3d_transpose(alt_handle_t h, const alt_conv3d_desc_t *d, const void *w_cktrs,
                                                     void *w_packed, void *stream)
{
    if (!h) return ALT_INVALID_ARG;
    if (!d || !w_cktrs || !w_packed) return fail(h, ALT_INVALID_ARG, "alt_pack_weights3d_transpose: null argument");
    if (d->plane.in_dtype != ALT_F32 && d->plane.in_dtype != ALT_BF16) return fail(h, ALT_INVALID_ARG, "alt_pack_weights3d_transpose: bad dtype");
    if (!h->has_gpu) return fail(h, ALT_HIP_ERROR, "no GPU device available");
    Problem3d chk;
    const alt_status_t cs = transposed_problem(h, d, &chk);
    if (cs != ALT_OK) return cs;
    SubPixel3d sp;
    if (!subpixel3d_plan(h, d, &sp)) return pack3d(h, d, w_cktrs, w_packed, stream, true, "alt_pack_weights3d_transpose");
    const alt_conv_desc_t &q = d->plane;
    Merge3dParams m;
    const int64_t msh[4] = {sp.m.plane.K, q.C * sp.m.T, sp.m.plane.R, sp.m.plane.S};
    std::string err;
    const alt_status_t ms = bind_layout(&q.w_layout, 4, msh, &m.ld, &err);
    if (ms != ALT_OK) return fail(h, ms, "w_layout: %s", err.c_str());
    m.src = w_cktrs;
    m.dst = w_packed;
    m.C = q.C; m.K = q.K; m.T = d->T; m.R = q.R; m.S = q.S;
    m.sd = d->stride_d; m.sh = q.stride_h; m.sw = q.stride_w;
    m.pad_d = d->pad_d; m.pad_h = q.pad_h; m.pad_w = q.pad_w;
    m.dil_d = d->dil_d; m.dil_h = q.dil_h; m.dil_w = q.dil_w;
    m.pm_d = sp.ad.pad; m.pm_h = sp.ah.pad; m.pm_w = sp.aw.pad;
    hipStream_t st = (hipStream_t)stream;
    if (dtype_size(q.in_dtype) == 2) hipLaunchKernelGGL(c3d_merge_kernel<2>, dim3(blocks_for(m.ld.numel)), dim3(kC3dThreads), 0, st, m);
    else hipLaunchKernelGGL(c3d_merge_kernel<4>, dim3(blocks_for(m.ld.numel)), dim3(kC3dThreads), 0, st, m);
    ALT_CHECK_HIP(h, hipGetLastError());
    return ALT_OK;
}

extern "C" alt_status_t alt_conv3d_transpose_weight_shape(alt_handle_t h, const alt_conv3d_desc_t *d, int64_t *out)
{
    if (!h) return ALT_INVALID_ARG;
    if (!d || !out) return fail(h, ALT_INVALID_ARG, "null argument");
    Problem3d p;
    const alt_status_t s = transposed_problem(h, d, &p);
    if (s != ALT_OK) return s;
    SubPixel3d sp;
    if (subpixel3d_plan(h, d, &sp)) {
        out[0] = sp.m.plane.K; out[1] = d->plane.C * sp.m.T; out[2] = sp.m.plane.R; out[3] = sp.m.plane.S;
    } else {
        out[0] = d->plane.K; out[1] = d->plane.C * d->T; out[2] = d->plane.R; out[3] = d->plane.S;
    }
    return ALT_OK;
}

extern "C" alt_status_t alt_conv3d_transpose(alt_handle_t h, const alt_conv3d_desc_t *d, const void *x, const void *w_packed,
                                             const float *bias, void *y, void *workspace, size_t ws_bytes, void *stream)
{
    if (!h) return ALT_INVALID_ARG;
    if (!d || !x || !w_packed || !y) return fail(h, ALT_INVALID_ARG, "alt_conv3d_transpose: null argument");
    if (d->plane.in_dtype != ALT_F32 && d->plane.in_dtype != ALT_BF16) return fail(h, ALT_INVALID_ARG, "alt_conv3d_transpose: bad dtype");
    Problem3d p;
    const alt_status_t s = transposed_problem(h, d, &p);
    if (s != ALT_OK) return s;
    SubPixel3d sp;
    if (subpixel3d_plan(h, d, &sp)) return run_subpixel3d(h, d, sp, x, w_packed, bias, y, workspace, ws_bytes, stream);
    return run3d(h, p, x, w_packed, bias, y, workspace, ws_bytes, stream, "alt_conv3d_transpose");
}

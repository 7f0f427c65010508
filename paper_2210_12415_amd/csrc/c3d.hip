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
#include <hip/hip_runtime.h>

#include <string>

#include "common.h"
#include "fast_layout.h"
#include "layout_eval.h"
#include "ops.h"

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
    BoundLayout ls, ld;           // x over (N*D, C, H, W); x' over (N*OD, T*C, H, W)
    int64_t D, OD, C;
    int32_t sd, pd, dd, pad_;
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
        const int64_t d = od * p.sd - p.pd + t * p.dd;
        E v = 0;
        if (d >= 0 && d < p.D) {
            idx[0] = img * p.D + d;
            idx[1] = c;
            v = ((const E *)p.src)[eval_offset(p.ls, idx)];
        }
        ((E *)p.dst)[out] = v;
    }
}

struct GatherFastParams {
    const void *src;
    void *dst;
    FastLayout ls, ld;
    FastDiv by_od, by_c;
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
        const int32_t d = (int32_t)od * p.sd - p.pd + (int32_t)t * p.dd;
        V w;
        __builtin_memset(&w, 0, sizeof w);
        if ((uint32_t)d < p.D) {
            idx[0] = img * p.D + (uint32_t)d;
            idx[1] = c;
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
int gather_vec(const BoundLayout &ls, const BoundLayout &ld, int elsz, int64_t C, const void *src, const void *dst)
{
    const int want = 16 / elsz;
    const Atom *is = unit_stride_atom(ls), *id = unit_stride_atom(ld);
    if (!is || !id || is->dim != id->dim || (is->dim != 1 && is->dim != 3) || is->div != 1 || id->div != 1) return 1;
    if (is->ext % want || id->ext % want || (is->dim == 1 && C % want)) return 1;
    if ((uintptr_t)src % 16 || (uintptr_t)dst % 16) return 1;
    return want;
}

struct PackParams {
    const void *src;              // dense (K, C, T, R, S)
    void *dst;
    BoundLayout ld;               // w' over (K, T*C, R, S) under w_layout
    int64_t C, T;
};

// w'[k, t*C + c, r, s] = w[k, c, t, r, s], one thread per element.
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
        const int64_t src = (((idx[0] * p.C + c) * p.T + t) * R + idx[2]) * S + idx[3];
        ((E *)p.dst)[eval_offset(p.ld, idx)] = ((const E *)p.src)[src];
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

// The equivalent 2-D problem of a 3-D descriptor; *gather says whether x' differs from x.
alt_status_t plane_desc(alt_handle_t h, const alt_conv3d_desc_t *d, alt_conv_desc_t *f, bool *gather)
{
    const alt_conv_desc_t &q = d->plane;
    if (q.N < 1 || q.C < 1 || d->D < 1 || d->T < 1) return fail(h, ALT_INVALID_ARG, "alt_conv3d: extents must be positive");
    if (d->stride_d < 1 || d->dil_d < 1 || d->pad_d < 0) return fail(h, ALT_INVALID_ARG, "alt_conv3d: bad depth stride, padding or dilation");
    if (q.groups > 1) return fail(h, ALT_UNSUPPORTED, "alt_conv3d: groups are not supported");
    const int64_t OD = out_depth(d);
    if (OD < 1) return fail(h, ALT_INVALID_ARG, "alt_conv3d: the filter is deeper than the padded input");
    *f = q;
    f->N = q.N * OD;
    f->C = q.C * d->T;
    *gather = !(d->T == 1 && d->stride_d == 1 && d->pad_d == 0);
    return ALT_OK;
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

extern "C" alt_status_t alt_conv3d_workspace_size(alt_handle_t h, const alt_conv3d_desc_t *d, size_t *bytes)
{
    if (!h) return ALT_INVALID_ARG;
    if (!d || !bytes) return fail(h, ALT_INVALID_ARG, "null argument");
    alt_conv_desc_t f;
    bool gather;
    alt_status_t s = plane_desc(h, d, &f, &gather);
    if (s != ALT_OK) return s;
    size_t conv_ws = 0;
    if ((s = alt_conv2d_workspace_size(h, &f, &conv_ws)) != ALT_OK) return s;
    *bytes = (gather ? round256((size_t)(f.N * f.C * f.H * f.W) * dtype_size(f.in_dtype)) : 0) + conv_ws;
    return ALT_OK;
}

extern "C" alt_status_t alt_pack_weights3d(alt_handle_t h, const alt_conv3d_desc_t *d, const void *w_kctrs,
                                           void *w_packed, void *stream)
{
    if (!h) return ALT_INVALID_ARG;
    if (!d || !w_kctrs || !w_packed) return fail(h, ALT_INVALID_ARG, "alt_pack_weights3d: null argument");
    const alt_conv_desc_t &q = d->plane;
    if (q.in_dtype != ALT_F32 && q.in_dtype != ALT_BF16) return fail(h, ALT_INVALID_ARG, "alt_pack_weights3d: bad dtype");
    if (q.K < 1 || q.C < 1 || q.R < 1 || q.S < 1 || d->T < 1) return fail(h, ALT_INVALID_ARG, "alt_pack_weights3d: extents must be positive");
    if (!h->has_gpu) return fail(h, ALT_HIP_ERROR, "no GPU device available");
    const int64_t wsh[4] = {q.K, q.C * d->T, q.R, q.S};
    PackParams p;
    std::string err;
    alt_status_t s = bind_layout(&q.w_layout, 4, wsh, &p.ld, &err);
    if (s != ALT_OK) return fail(h, s, "w_layout: %s", err.c_str());
    p.src = w_kctrs;
    p.dst = w_packed;
    p.C = q.C;
    p.T = d->T;
    hipStream_t st = (hipStream_t)stream;
    if (dtype_size(q.in_dtype) == 2) hipLaunchKernelGGL(c3d_pack_kernel<2>, dim3(blocks_for(p.ld.numel)), dim3(kC3dThreads), 0, st, p);
    else hipLaunchKernelGGL(c3d_pack_kernel<4>, dim3(blocks_for(p.ld.numel)), dim3(kC3dThreads), 0, st, p);
    ALT_CHECK_HIP(h, hipGetLastError());
    return ALT_OK;
}

extern "C" alt_status_t alt_conv3d(alt_handle_t h, const alt_conv3d_desc_t *d, const void *x, const void *w_packed,
                                   const float *bias, void *y, void *workspace, size_t ws_bytes, void *stream)
{
    if (!h) return ALT_INVALID_ARG;
    if (!d || !x || !w_packed || !y) return fail(h, ALT_INVALID_ARG, "alt_conv3d: null argument");
    const alt_conv_desc_t &q = d->plane;
    if (q.in_dtype != ALT_F32 && q.in_dtype != ALT_BF16) return fail(h, ALT_INVALID_ARG, "alt_conv3d: bad dtype");
    alt_conv_desc_t f;
    bool gather;
    alt_status_t s = plane_desc(h, d, &f, &gather);
    if (s != ALT_OK) return s;
    if (!gather) return alt_conv2d(h, &f, x, w_packed, bias, y, workspace, ws_bytes, stream);

    if (!h->has_gpu) return fail(h, ALT_HIP_ERROR, "no GPU device available");
    if (q.H < 1 || q.W < 1) return fail(h, ALT_INVALID_ARG, "alt_conv3d: extents must be positive");
    const int elsz = (int)dtype_size(q.in_dtype);
    const size_t xu_bytes = round256((size_t)(f.N * f.C * f.H * f.W) * elsz);
    if (!workspace || ws_bytes < xu_bytes)
        return fail(h, ALT_WORKSPACE_TOO_SMALL, "alt_conv3d: the workspace must hold the depth-unfolded input (%zu bytes)", xu_bytes);
    if ((uintptr_t)workspace % 16) return fail(h, ALT_INVALID_ARG, "alt_conv3d: workspace must be 16-byte aligned");
    GatherParams p;
    const int64_t OD = out_depth(d);
    const int64_t xs[4] = {q.N * d->D, q.C, q.H, q.W}, us[4] = {f.N, f.C, f.H, f.W};
    std::string err;
    if ((s = bind_layout(&q.x_layout, 4, xs, &p.ls, &err)) != ALT_OK) return fail(h, s, "x_layout: %s", err.c_str());
    if ((s = bind_layout(&q.x_layout, 4, us, &p.ld, &err)) != ALT_OK) return fail(h, s, "x_layout (depth-unfolded input): %s", err.c_str());
    p.src = x;
    p.dst = workspace;
    p.D = d->D;
    p.OD = OD;
    p.C = q.C;
    p.sd = d->stride_d;
    p.pd = d->pad_d;
    p.dd = d->dil_d;
    p.pad_ = 0;
    hipStream_t st = (hipStream_t)stream;
    GatherFastParams g;
    const bool small = d->D < ((int64_t)1 << 20) && OD < ((int64_t)1 << 20) && d->T < ((int64_t)1 << 10) &&
                       (int64_t)d->stride_d * OD + (int64_t)d->dil_d * d->T + d->pad_d < ((int64_t)1 << 30);
    if (small && fast_layout(p.ls, &g.ls) && fast_layout(p.ld, &g.ld)) {
        const int vec = gather_vec(p.ls, p.ld, elsz, q.C, x, workspace);
        g.src = x;
        g.dst = workspace;
        g.by_od = make_fastdiv((uint32_t)OD);
        g.by_c = make_fastdiv((uint32_t)q.C);
        g.D = (uint32_t)d->D;
        g.nvec = (uint32_t)(p.ld.numel / vec);
        g.sd = d->stride_d;
        g.pd = d->pad_d;
        g.dd = d->dil_d;
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

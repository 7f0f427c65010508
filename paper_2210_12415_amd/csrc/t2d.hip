// Transposed 2-D convolution (T2D in the operator list of Section 6.1 of the paper) on the
// forward convolution kernels.  The scatter
//   y[n,k,ih*stride-pad+r*dil, iw*stride-pad+s*dil] += x[n,c,ih,iw] * w[c,k,r,s]
// is the gather of a stride-1 convolution over x with stride-1 zeros between its pixels,
// with the filter mirrored in both directions, its channel dimensions exchanged, and
// padding dil*(R-1)-pad.  Two small kernels prepare the operands under their layouts (the
// filter once, offline: it is a constant like any other weight tensor, Section 4.2; the
// expanded input per call, into the workspace), then alt_conv2d does the work.
#include <hip/hip_runtime.h>

#include <string>

#include "common.h"
#include "fast_layout.h"
#include "layout_eval.h"
#include "ops.h"
#include "subpixel.h"

namespace alt {
namespace {

constexpr int kT2dThreads = 256;

template <int ELSZ> struct Elem;
template <> struct Elem<2> { using type = uint16_t; };
template <> struct Elem<4> { using type = uint32_t; };
template <int BYTES> struct Word;
template <> struct Word<2> { using type = uint16_t; };
template <> struct Word<4> { using type = uint32_t; };
template <> struct Word<16> { using type = uint4; };

struct SpreadParams {
    const void *src;
    void *dst;
    BoundLayout ls, ld;           // x over (N,C,H,W); the expanded tensor over (N,C,(H-1)*sh+1,(W-1)*sw+1)
    int32_t sh, sw;
};

// One thread per element of the expanded tensor: x's element where both spatial indices are
// multiples of the stride, zero elsewhere.
template <int ELSZ>
__global__ __launch_bounds__(kT2dThreads) void t2d_spread_kernel(SpreadParams p)
{
    using E = typename Elem<ELSZ>::type;
    const int64_t n = p.ld.numel;
    for (int64_t e = blockIdx.x * (int64_t)kT2dThreads + threadIdx.x; e < n; e += (int64_t)gridDim.x * kT2dThreads) {
        int64_t idx[ALT_MAX_RANK];
        int64_t r = e;
        for (int d = 3; d >= 0; --d) { idx[d] = r % p.ld.shape[d]; r /= p.ld.shape[d]; }
        const int64_t out = eval_offset(p.ld, idx);
        E v = 0;
        if (idx[2] % p.sh == 0 && idx[3] % p.sw == 0) {
            idx[2] /= p.sh;
            idx[3] /= p.sw;
            v = ((const E *)p.src)[eval_offset(p.ls, idx)];
        }
        ((E *)p.dst)[out] = v;
    }
}

// The same for separable layouts with fewer than 2^31 elements, walked in the order of the
// expanded tensor's memory: a thread owns VEC consecutive elements there (one element, or
// 16 bytes of a channel run when both layouts end in the same contiguous channel block),
// recovers their logical index from the offset digit by digit and gathers from x.  All
// index arithmetic is 32-bit with divisions by multiplication.
struct SpreadFastParams {
    const void *src;
    void *dst;
    FastLayout ls, ld;
    FastDiv by_sh, by_sw;
    uint32_t nvec, pad_;
};

template <int ELSZ, int VEC>
__global__ __launch_bounds__(kT2dThreads) void t2d_spread_fast_kernel(SpreadFastParams p)
{
    using V = typename Word<ELSZ * VEC>::type;
    for (uint32_t v = blockIdx.x * kT2dThreads + threadIdx.x; v < p.nvec; v += gridDim.x * kT2dThreads) {
        const uint32_t o = v * VEC;
        uint32_t idx[4] = {0, 0, 0, 0};
        for (int j = 0; j < p.ld.n; ++j) {
            const FastAtom &a = p.ld.a[j];
            idx[a.dim] += fast_mod(fast_div(o, a.by_stride), a.by_ext) * a.div;
        }
        const uint32_t qh = fast_div(idx[2], p.by_sh), qw = fast_div(idx[3], p.by_sw);
        V w;
        __builtin_memset(&w, 0, sizeof w);
        if (qh * p.by_sh.d == idx[2] && qw * p.by_sw.d == idx[3]) {
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

// Elements per thread: eight (16 bytes of bf16) or four (of fp32) when both layouts end in
// the same contiguous channel piece whose extent is a multiple of that, else one.
int spread_vec(const BoundLayout &ls, const BoundLayout &ld, int elsz, const void *src, const void *dst)
{
    const int want = 16 / elsz;
    const Atom *is = nullptr, *id = nullptr;
    for (int j = 0; j < ls.nsub; ++j) if (ls.atom[j].stride == 1) is = &ls.atom[j];
    for (int j = 0; j < ld.nsub; ++j) if (ld.atom[j].stride == 1) id = &ld.atom[j];
    if (!is || !id || is->dim != 1 || id->dim != 1 || is->div != 1 || id->div != 1 || is->ext != id->ext) return 1;
    if (is->ext % want || (uintptr_t)src % 16 || (uintptr_t)dst % 16) return 1;
    return want;
}

struct FlipParams {
    const void *src;              // dense (C,K,R,S)
    void *dst;
    BoundLayout ld;               // the forward filter (K,C,R,S) under w_layout
};

// w'[k,c,r,s] = w[c,k,R-1-r,S-1-s], one thread per element.
template <int ELSZ>
__global__ __launch_bounds__(kT2dThreads) void t2d_flip_kernel(FlipParams p)
{
    using E = typename Elem<ELSZ>::type;
    const int64_t n = p.ld.numel;
    const int64_t K = p.ld.shape[0], R = p.ld.shape[2], S = p.ld.shape[3];
    for (int64_t e = blockIdx.x * (int64_t)kT2dThreads + threadIdx.x; e < n; e += (int64_t)gridDim.x * kT2dThreads) {
        int64_t idx[ALT_MAX_RANK];
        int64_t r = e;
        for (int d = 3; d >= 0; --d) { idx[d] = r % p.ld.shape[d]; r /= p.ld.shape[d]; }
        const int64_t src = ((idx[1] * K + idx[0]) * R + (R - 1 - idx[2])) * S + (S - 1 - idx[3]);
        ((E *)p.dst)[eval_offset(p.ld, idx)] = ((const E *)p.src)[src];
    }
}

unsigned blocks_for(int64_t n)
{
    const int64_t b = (n + kT2dThreads - 1) / kT2dThreads;
    return (unsigned)(b < 1 ? 1 : b > 256 * 64 ? 256 * 64 : b);
}

size_t round256(size_t n) { return (n + 255) / 256 * 256; }

// The equivalent forward problem of a transposed-convolution descriptor.
alt_status_t forward_desc(alt_handle_t h, const alt_conv_desc_t *d, alt_conv_desc_t *f)
{
    if (d->N < 1 || d->C < 1 || d->H < 1 || d->W < 1 || d->K < 1 || d->R < 1 || d->S < 1)
        return fail(h, ALT_INVALID_ARG, "alt_conv2d_transpose: extents must be positive");
    if (d->stride_h < 1 || d->stride_w < 1 || d->dil_h < 1 || d->dil_w < 1 || d->pad_h < 0 || d->pad_w < 0)
        return fail(h, ALT_INVALID_ARG, "alt_conv2d_transpose: bad stride, padding or dilation");
    if (d->groups > 1) return fail(h, ALT_UNSUPPORTED, "alt_conv2d_transpose: groups are not supported");
    if (d->pad_h > d->dil_h * (d->R - 1) || d->pad_w > d->dil_w * (d->S - 1))
        return fail(h, ALT_UNSUPPORTED, "alt_conv2d_transpose: padding beyond dil*(R-1) is not supported");
    *f = *d;
    f->H = (d->H - 1) * d->stride_h + 1;
    f->W = (d->W - 1) * d->stride_w + 1;
    f->stride_h = f->stride_w = 1;
    f->pad_h = d->dil_h * (int32_t)(d->R - 1) - d->pad_h;
    f->pad_w = d->dil_w * (int32_t)(d->S - 1) - d->pad_w;
    return ALT_OK;
}

// ---- the sub-pixel form ---------------------------------------------------------------------
// Output pixel oh = q*stride + ph takes input rows ih with oh = ih*stride - pad + r*dil, that is
// ih = q + delta with delta = (ph + pad - r*dil) / stride for the taps r where that divides.
// The stride*stride phases (ph, pw) are therefore stride-1 convolutions of x itself, each with
// its own taps at offsets delta; written over the common range of offsets (filter extent
// delta_max - delta_min + 1, padding -delta_min, zeros where a phase has no tap) they are ONE
// convolution with stride_h*stride_w*K output channels, channel (ph*stride_w + pw)*K + k, whose
// result y'[n, (ph,pw,k), q, p] = y[n, k, q*stride_h + ph, p*stride_w + pw] a second kernel
// moves into place.  No inserted zeros are multiplied, x is read where it lies.  It applies
// when the output extents are multiples of the strides and the symmetric padding -delta_min
// yields exactly OH/stride_h by OW/stride_w outputs (4x4 at stride 2 with padding 1, 2x2 at
// stride 2, 6x6 at stride 2 with padding 2, 8x8 at stride 4 with padding 2, ...).
struct SubPixelPlan {
    alt_conv_desc_t f;            // the merged stride-1 problem on x: K' = stride_h*stride_w*K channels out
    PhaseAxis ah, aw;
};

// Whether the descriptor runs in the sub-pixel form (decided from the descriptor alone, so the
// weight pack, the workspace size and the call agree), and the merged problem if so.
bool subpixel_plan(const alt_conv_desc_t *d, SubPixelPlan *out)
{
    if (d->stride_h == 1 && d->stride_w == 1) return false;
    if (d->stride_h > 8 || d->stride_w > 8) return false;
    SubPixelPlan &s = *out;
    s.ah = phase_axis(d->H, d->R, d->stride_h, d->pad_h, d->dil_h);
    s.aw = phase_axis(d->W, d->S, d->stride_w, d->pad_w, d->dil_w);
    if (!s.ah.ok || !s.aw.ok) return false;
    s.f = *d;
    s.f.K = d->K * d->stride_h * d->stride_w;
    s.f.R = s.ah.taps;
    s.f.S = s.aw.taps;
    s.f.stride_h = s.f.stride_w = 1;
    s.f.dil_h = s.f.dil_w = 1;
    s.f.pad_h = s.ah.pad;
    s.f.pad_w = s.aw.pad;
    // the three layouts must take the merged extents (block factors dividing K')
    BoundLayout b;
    std::string err;
    const int64_t ws[4] = {s.f.K, s.f.C, s.f.R, s.f.S}, ys[4] = {s.f.N, s.f.K, s.ah.outq, s.aw.outq};
    if (bind_layout(&d->w_layout, 4, ws, &b, &err) != ALT_OK) return false;
    if (bind_layout(&d->y_layout, 4, ys, &b, &err) != ALT_OK) return false;
    return true;
}

struct MergeParams {
    const void *src;              // dense (C,K,R,S)
    void *dst;
    BoundLayout ld;               // the merged filter (K', C, Rm, Sm) under w_layout
    int64_t K, R, S;
    int32_t sh, sw, pad_h, pad_w, dil_h, dil_w, pm_h, pm_w;
};

// w_m[(ph*sw + pw)*K + k, c, a, b] = w[c, k, r, s] for the tap (r, s) with
// r*dil_h = ph + pad_h - sh*(a - pm_h), s*dil_w = pw + pad_w - sw*(b - pm_w); zero if there is none.
template <int ELSZ>
__global__ __launch_bounds__(kT2dThreads) void t2d_merge_kernel(MergeParams p)
{
    using E = typename Elem<ELSZ>::type;
    const int64_t n = p.ld.numel;
    for (int64_t e = blockIdx.x * (int64_t)kT2dThreads + threadIdx.x; e < n; e += (int64_t)gridDim.x * kT2dThreads) {
        int64_t idx[ALT_MAX_RANK];
        int64_t rem = e;
        for (int d = 3; d >= 0; --d) { idx[d] = rem % p.ld.shape[d]; rem /= p.ld.shape[d]; }
        const int64_t phase = idx[0] / p.K, k = idx[0] - phase * p.K;
        const int64_t ph = phase / p.sw, pw = phase - ph * p.sw;
        const int64_t nr = ph + p.pad_h - p.sh * (idx[2] - p.pm_h), ns = pw + p.pad_w - p.sw * (idx[3] - p.pm_w);
        E v = 0;
        if (nr >= 0 && ns >= 0 && nr % p.dil_h == 0 && ns % p.dil_w == 0 && nr / p.dil_h < p.R && ns / p.dil_w < p.S)
            v = ((const E *)p.src)[((idx[1] * p.K + k) * p.R + nr / p.dil_h) * p.S + ns / p.dil_w];
        ((E *)p.dst)[eval_offset(p.ld, idx)] = v;
    }
}

// bias'[(ph*sw + pw)*K + k] = bias[k]
__global__ __launch_bounds__(kT2dThreads) void t2d_bias_kernel(const float *bias, float *out, int K, int n)
{
    const int i = blockIdx.x * kT2dThreads + threadIdx.x;
    if (i < n) out[i] = bias[i % K];
}

struct ShuffleParams {
    const void *src;              // y' over (N*OD/sd, K', OH/sh, OW/sw) under y_layout
    void *dst;                    // y over (N*OD, K, OH, OW) under y_layout (OD = sd = 1 for the 2-D operator)
    BoundLayout ls, ld;
    int32_t sd, sh, sw, pad_;
    int64_t K, OD;
};

// One thread per element of y, any layout.
template <int ELSZ>
__global__ __launch_bounds__(kT2dThreads) void t2d_shuffle_kernel(ShuffleParams p)
{
    using E = typename Elem<ELSZ>::type;
    const int64_t n = p.ld.numel;
    for (int64_t e = blockIdx.x * (int64_t)kT2dThreads + threadIdx.x; e < n; e += (int64_t)gridDim.x * kT2dThreads) {
        int64_t idx[ALT_MAX_RANK];
        int64_t r = e;
        for (int d = 3; d >= 0; --d) { idx[d] = r % p.ld.shape[d]; r /= p.ld.shape[d]; }
        const int64_t out = eval_offset(p.ld, idx);
        const int64_t q = idx[2] / p.sh, ph = idx[2] - q * p.sh, c = idx[3] / p.sw, pw = idx[3] - c * p.sw;
        const int64_t img = idx[0] / p.OD, od = idx[0] - img * p.OD, qd = od / p.sd, pd = od - qd * p.sd;
        idx[0] = img * (p.OD / p.sd) + qd;
        idx[1] += ((pd * p.sh + ph) * p.sw + pw) * p.K;
        idx[2] = q;
        idx[3] = c;
        ((E *)p.dst)[out] = ((const E *)p.src)[eval_offset(p.ls, idx)];
    }
}

struct ShuffleFastParams {
    const void *src;
    void *dst;
    FastLayout ls, ld;
    FastDiv by_sh, by_sw, by_sd, by_od;
    uint32_t K, nvec, ODq, pad_;
};

// The same for separable layouts with fewer than 2^31 elements, walked in the order of y's
// memory, VEC consecutive channels per thread where both layouts end in a channel run.
template <int ELSZ, int VEC>
__global__ __launch_bounds__(kT2dThreads) void t2d_shuffle_fast_kernel(ShuffleFastParams p)
{
    using V = typename Word<ELSZ * VEC>::type;
    for (uint32_t v = blockIdx.x * kT2dThreads + threadIdx.x; v < p.nvec; v += gridDim.x * kT2dThreads) {
        const uint32_t o = v * VEC;
        uint32_t idx[4] = {0, 0, 0, 0};
        for (int j = 0; j < p.ld.n; ++j) {
            const FastAtom &a = p.ld.a[j];
            idx[a.dim] += fast_mod(fast_div(o, a.by_stride), a.by_ext) * a.div;
        }
        const uint32_t q = fast_div(idx[2], p.by_sh), ph = idx[2] - q * p.by_sh.d;
        const uint32_t c = fast_div(idx[3], p.by_sw), pw = idx[3] - c * p.by_sw.d;
        const uint32_t img = fast_div(idx[0], p.by_od), od = idx[0] - img * p.by_od.d;
        const uint32_t qd = fast_div(od, p.by_sd), pd = od - qd * p.by_sd.d;
        idx[0] = img * p.ODq + qd;
        idx[1] += ((pd * p.by_sh.d + ph) * p.by_sw.d + pw) * p.K;
        idx[2] = q;
        idx[3] = c;
        uint32_t so = 0;
        for (int j = 0; j < p.ls.n; ++j) {
            const FastAtom &a = p.ls.a[j];
            so += fast_mod(fast_div(idx[a.dim], a.by_div), a.by_ext) * a.stride;
        }
        *(V *)((char *)p.dst + (size_t)o * ELSZ) = *(const V *)((const char *)p.src + (size_t)so * ELSZ);
    }
}

// Elements per thread of the shuffle: 16 bytes' worth when both layouts end in a contiguous
// channel run (the innermost piece of the channels) whose extents, and K itself, are multiples of it.
int shuffle_vec(const BoundLayout &ls, const BoundLayout &ld, int elsz, int64_t K, const void *src, const void *dst)
{
    const int want = 16 / elsz;
    const Atom *is = unit_stride_atom(ls), *id = unit_stride_atom(ld);
    if (!is || !id || is->dim != 1 || id->dim != 1 || is->div != 1 || id->div != 1) return 1;
    if (is->ext % want || id->ext % want || K % want || (uintptr_t)src % 16 || (uintptr_t)dst % 16) return 1;
    return want;
}

// Workspace of the sub-pixel form: y', then bias', then what alt_conv2d wants.
size_t subpixel_y_bytes(const SubPixelPlan &s)
{
    return round256((size_t)(s.f.N * s.f.K * s.ah.outq * s.aw.outq) * dtype_size(s.f.out_dtype));
}
size_t subpixel_bias_bytes(const SubPixelPlan &s) { return round256((size_t)s.f.K * sizeof(float)); }

}  // namespace

// y[(n, qd*sd + pd), k, q*sh + ph, p*sw + pw] = y'[(n, qd), ((pd*sh + ph)*sw + pw)*K + k, q, p], both under `layout`
// (y' over (N*ODq, sd*sh*sw*K, OHq, OWq); ODq = sd = 1 for the 2-D operator).
alt_status_t phase_shuffle(alt_handle_t h, const alt_layout_t *layout, int64_t N, int64_t K, int64_t ODq, int64_t OHq, int64_t OWq,
                           int sd, int sh, int sw, int elsz, const void *src, void *dst, hipStream_t st)
{
    ShuffleParams p;
    const int64_t qs[4] = {N * ODq, K * sd * sh * sw, OHq, OWq};
    const int64_t os[4] = {N * ODq * sd, K, OHq * sh, OWq * sw};
    std::string err;
    alt_status_t st_;
    if ((st_ = bind_layout(layout, 4, qs, &p.ls, &err)) != ALT_OK) return fail(h, st_, "y_layout (phase-major output): %s", err.c_str());
    if ((st_ = bind_layout(layout, 4, os, &p.ld, &err)) != ALT_OK) return fail(h, st_, "y_layout: %s", err.c_str());
    p.src = src;
    p.dst = dst;
    p.sd = sd; p.sh = sh; p.sw = sw; p.pad_ = 0;
    p.K = K;
    p.OD = ODq * sd;
    ShuffleFastParams q;
    if (fast_layout(p.ls, &q.ls) && fast_layout(p.ld, &q.ld)) {
        const int vec = shuffle_vec(p.ls, p.ld, elsz, K, src, dst);
        q.src = src;
        q.dst = dst;
        q.by_sh = make_fastdiv((uint32_t)sh);
        q.by_sw = make_fastdiv((uint32_t)sw);
        q.by_sd = make_fastdiv((uint32_t)sd);
        q.by_od = make_fastdiv((uint32_t)p.OD);
        q.K = (uint32_t)K;
        q.ODq = (uint32_t)ODq;
        q.pad_ = 0;
        q.nvec = (uint32_t)(p.ld.numel / vec);
        const dim3 grid(blocks_for(q.nvec)), block(kT2dThreads);
        if (elsz == 2 && vec == 8) hipLaunchKernelGGL((t2d_shuffle_fast_kernel<2, 8>), grid, block, 0, st, q);
        else if (elsz == 2) hipLaunchKernelGGL((t2d_shuffle_fast_kernel<2, 1>), grid, block, 0, st, q);
        else if (vec == 4) hipLaunchKernelGGL((t2d_shuffle_fast_kernel<4, 4>), grid, block, 0, st, q);
        else hipLaunchKernelGGL((t2d_shuffle_fast_kernel<4, 1>), grid, block, 0, st, q);
    } else if (elsz == 2) {
        hipLaunchKernelGGL(t2d_shuffle_kernel<2>, dim3(blocks_for(p.ld.numel)), dim3(kT2dThreads), 0, st, p);
    } else {
        hipLaunchKernelGGL(t2d_shuffle_kernel<4>, dim3(blocks_for(p.ld.numel)), dim3(kT2dThreads), 0, st, p);
    }
    ALT_CHECK_HIP(h, hipGetLastError());
    return ALT_OK;
}

// bias'[j*K + k] = bias[k] for the n = phases*K entries of `out`
alt_status_t phase_bias(alt_handle_t h, const float *bias, float *out, int64_t K, int64_t n, hipStream_t st)
{
    hipLaunchKernelGGL(t2d_bias_kernel, dim3((unsigned)((n + kT2dThreads - 1) / kT2dThreads)), dim3(kT2dThreads), 0, st, bias, out,
                       (int)K, (int)n);
    ALT_CHECK_HIP(h, hipGetLastError());
    return ALT_OK;
}

namespace {

alt_status_t run_subpixel(alt_handle_t h, const alt_conv_desc_t *d, const SubPixelPlan &s, const void *x, const void *w_packed,
                          const float *bias, void *y, void *workspace, size_t ws_bytes, void *stream)
{
    if (!h->has_gpu) return fail(h, ALT_HIP_ERROR, "no GPU device available");
    const size_t yb = subpixel_y_bytes(s), bb = subpixel_bias_bytes(s);
    if (!workspace || ws_bytes < yb + bb)
        return fail(h, ALT_WORKSPACE_TOO_SMALL, "alt_conv2d_transpose: the workspace must hold the phase-major output (%zu bytes)", yb + bb);
    if ((uintptr_t)workspace % 16 || (uintptr_t)y % 16) return fail(h, ALT_INVALID_ARG, "alt_conv2d_transpose: workspace and y must be 16-byte aligned");
    if ((d->epilogue & ALT_EPI_BIAS) && !bias) return fail(h, ALT_INVALID_ARG, "alt_conv2d_transpose: ALT_EPI_BIAS without a bias");
    hipStream_t st = (hipStream_t)stream;
    float *bias_m = (float *)((char *)workspace + yb);
    alt_status_t st_;
    if (d->epilogue & ALT_EPI_BIAS)
        if ((st_ = phase_bias(h, bias, bias_m, d->K, s.f.K, st)) != ALT_OK) return st_;
    st_ = alt_conv2d(h, &s.f, x, w_packed, (d->epilogue & ALT_EPI_BIAS) ? bias_m : nullptr, workspace,
                     (char *)workspace + yb + bb, ws_bytes - yb - bb, stream);
    if (st_ != ALT_OK) return st_;
    return phase_shuffle(h, &d->y_layout, d->N, d->K, 1, s.ah.outq, s.aw.outq, 1, d->stride_h, d->stride_w,
                         (int)dtype_size(d->out_dtype), workspace, y, st);
}

}  // namespace
}  // namespace alt

using namespace alt;

extern "C" alt_status_t alt_conv2d_transpose_output_shape(const alt_conv_desc_t *d, int64_t *out)
{
    if (!d || !out) return ALT_INVALID_ARG;
    if (d->stride_h < 1 || d->stride_w < 1 || d->dil_h < 1 || d->dil_w < 1) return ALT_INVALID_ARG;
    out[0] = d->N;
    out[1] = d->K;
    out[2] = (d->H - 1) * d->stride_h - 2 * d->pad_h + d->dil_h * (d->R - 1) + 1;
    out[3] = (d->W - 1) * d->stride_w - 2 * d->pad_w + d->dil_w * (d->S - 1) + 1;
    return (out[2] < 1 || out[3] < 1) ? ALT_INVALID_ARG : ALT_OK;
}

extern "C" alt_status_t alt_conv2d_transpose_weight_shape(const alt_conv_desc_t *d, int64_t *out)
{
    if (!d || !out) return ALT_INVALID_ARG;
    if (d->K < 1 || d->C < 1 || d->R < 1 || d->S < 1 || d->H < 1 || d->W < 1 || d->stride_h < 1 || d->stride_w < 1 || d->dil_h < 1 ||
        d->dil_w < 1 || d->pad_h < 0 || d->pad_w < 0)
        return ALT_INVALID_ARG;
    SubPixelPlan sp;
    if (subpixel_plan(d, &sp)) {
        out[0] = sp.f.K; out[1] = sp.f.C; out[2] = sp.f.R; out[3] = sp.f.S;
    } else {
        out[0] = d->K; out[1] = d->C; out[2] = d->R; out[3] = d->S;
    }
    return ALT_OK;
}

extern "C" alt_status_t alt_conv2d_transpose_problem(alt_handle_t h, const alt_conv_desc_t *d, alt_conv_desc_t *out)
{
    if (!h) return ALT_INVALID_ARG;
    if (!d || !out) return fail(h, ALT_INVALID_ARG, "null argument");
    alt_conv_desc_t f;
    const alt_status_t s = forward_desc(h, d, &f);
    if (s != ALT_OK) return s;
    SubPixelPlan sp;
    *out = subpixel_plan(d, &sp) ? sp.f : f;
    return ALT_OK;
}

extern "C" alt_status_t alt_conv2d_transpose_workspace_size(alt_handle_t h, const alt_conv_desc_t *d, size_t *bytes)
{
    if (!h) return ALT_INVALID_ARG;
    if (!d || !bytes) return fail(h, ALT_INVALID_ARG, "null argument");
    alt_conv_desc_t f;
    alt_status_t s = forward_desc(h, d, &f);
    if (s != ALT_OK) return s;
    size_t conv_ws = 0;
    SubPixelPlan sp;
    if (subpixel_plan(d, &sp)) {
        if ((s = alt_conv2d_workspace_size(h, &sp.f, &conv_ws)) != ALT_OK) return s;
        *bytes = subpixel_y_bytes(sp) + subpixel_bias_bytes(sp) + conv_ws;
        return ALT_OK;
    }
    if ((s = alt_conv2d_workspace_size(h, &f, &conv_ws)) != ALT_OK) return s;
    const bool spread = d->stride_h > 1 || d->stride_w > 1;
    *bytes = (spread ? round256((size_t)(f.N * f.C * f.H * f.W) * dtype_size(d->in_dtype)) : 0) + conv_ws;
    return ALT_OK;
}

extern "C" alt_status_t alt_pack_weights_transpose(alt_handle_t h, const alt_conv_desc_t *d, const void *w_ckrs,
                                                   void *w_packed, void *stream)
{
    if (!h) return ALT_INVALID_ARG;
    if (!d || !w_ckrs || !w_packed) return fail(h, ALT_INVALID_ARG, "alt_pack_weights_transpose: null argument");
    if (d->in_dtype != ALT_F32 && d->in_dtype != ALT_BF16) return fail(h, ALT_INVALID_ARG, "alt_pack_weights_transpose: bad dtype");
    if (!h->has_gpu) return fail(h, ALT_HIP_ERROR, "no GPU device available");
    {
        alt_conv_desc_t f;
        const alt_status_t fs = forward_desc(h, d, &f);
        if (fs != ALT_OK) return fs;
    }
    SubPixelPlan sp;
    if (subpixel_plan(d, &sp)) {
        MergeParams m;
        const int64_t msh[4] = {sp.f.K, sp.f.C, sp.f.R, sp.f.S};
        std::string merr;
        const alt_status_t ms = bind_layout(&d->w_layout, 4, msh, &m.ld, &merr);
        if (ms != ALT_OK) return fail(h, ms, "w_layout: %s", merr.c_str());
        m.src = w_ckrs;
        m.dst = w_packed;
        m.K = d->K; m.R = d->R; m.S = d->S;
        m.sh = d->stride_h; m.sw = d->stride_w; m.pad_h = d->pad_h; m.pad_w = d->pad_w; m.dil_h = d->dil_h; m.dil_w = d->dil_w;
        m.pm_h = sp.ah.pad; m.pm_w = sp.aw.pad;
        hipStream_t mst = (hipStream_t)stream;
        if (dtype_size(d->in_dtype) == 2) hipLaunchKernelGGL(t2d_merge_kernel<2>, dim3(blocks_for(m.ld.numel)), dim3(kT2dThreads), 0, mst, m);
        else hipLaunchKernelGGL(t2d_merge_kernel<4>, dim3(blocks_for(m.ld.numel)), dim3(kT2dThreads), 0, mst, m);
        ALT_CHECK_HIP(h, hipGetLastError());
        return ALT_OK;
    }
    const int64_t wsh[4] = {d->K, d->C, d->R, d->S};
    FlipParams p;
    std::string err;
    alt_status_t s = bind_layout(&d->w_layout, 4, wsh, &p.ld, &err);
    if (s != ALT_OK) return fail(h, s, "w_layout: %s", err.c_str());
    p.src = w_ckrs;
    p.dst = w_packed;
    hipStream_t st = (hipStream_t)stream;
    if (dtype_size(d->in_dtype) == 2) hipLaunchKernelGGL(t2d_flip_kernel<2>, dim3(blocks_for(p.ld.numel)), dim3(kT2dThreads), 0, st, p);
    else hipLaunchKernelGGL(t2d_flip_kernel<4>, dim3(blocks_for(p.ld.numel)), dim3(kT2dThreads), 0, st, p);
    ALT_CHECK_HIP(h, hipGetLastError());
    return ALT_OK;
}

extern "C" alt_status_t alt_conv2d_transpose(alt_handle_t h, const alt_conv_desc_t *d, const void *x, const void *w_packed,
                                             const float *bias, void *y, void *workspace, size_t ws_bytes, void *stream)
{
    if (!h) return ALT_INVALID_ARG;
    if (!d || !x || !w_packed || !y) return fail(h, ALT_INVALID_ARG, "alt_conv2d_transpose: null argument");
    if (d->in_dtype != ALT_F32 && d->in_dtype != ALT_BF16) return fail(h, ALT_INVALID_ARG, "alt_conv2d_transpose: bad dtype");
    alt_conv_desc_t f;
    alt_status_t s = forward_desc(h, d, &f);
    if (s != ALT_OK) return s;
    if (d->stride_h == 1 && d->stride_w == 1)
        return alt_conv2d(h, &f, x, w_packed, bias, y, workspace, ws_bytes, stream);
    SubPixelPlan sp;
    if (subpixel_plan(d, &sp)) return run_subpixel(h, d, sp, x, w_packed, bias, y, workspace, ws_bytes, stream);

    if (!h->has_gpu) return fail(h, ALT_HIP_ERROR, "no GPU device available");
    const size_t xe_bytes = round256((size_t)(f.N * f.C * f.H * f.W) * dtype_size(d->in_dtype));
    if (!workspace || ws_bytes < xe_bytes)
        return fail(h, ALT_WORKSPACE_TOO_SMALL, "alt_conv2d_transpose: the workspace must hold the expanded input (%zu bytes)", xe_bytes);
    if ((uintptr_t)workspace % 16) return fail(h, ALT_INVALID_ARG, "alt_conv2d_transpose: workspace must be 16-byte aligned");
    SpreadParams p;
    const int64_t xs[4] = {d->N, d->C, d->H, d->W}, es[4] = {f.N, f.C, f.H, f.W};
    std::string err;
    if ((s = bind_layout(&d->x_layout, 4, xs, &p.ls, &err)) != ALT_OK) return fail(h, s, "x_layout: %s", err.c_str());
    if ((s = bind_layout(&d->x_layout, 4, es, &p.ld, &err)) != ALT_OK) return fail(h, s, "x_layout (expanded input): %s", err.c_str());
    p.src = x;
    p.dst = workspace;
    p.sh = d->stride_h;
    p.sw = d->stride_w;
    hipStream_t st = (hipStream_t)stream;
    const int elsz = (int)dtype_size(d->in_dtype);
    SpreadFastParams q;
    if (fast_layout(p.ls, &q.ls) && fast_layout(p.ld, &q.ld)) {
        const int vec = spread_vec(p.ls, p.ld, elsz, x, workspace);
        q.src = x;
        q.dst = workspace;
        q.by_sh = make_fastdiv((uint32_t)d->stride_h);
        q.by_sw = make_fastdiv((uint32_t)d->stride_w);
        q.nvec = (uint32_t)(p.ld.numel / vec);
        q.pad_ = 0;
        const dim3 grid(blocks_for(q.nvec)), block(kT2dThreads);
        if (elsz == 2 && vec == 8) hipLaunchKernelGGL((t2d_spread_fast_kernel<2, 8>), grid, block, 0, st, q);
        else if (elsz == 2) hipLaunchKernelGGL((t2d_spread_fast_kernel<2, 1>), grid, block, 0, st, q);
        else if (vec == 4) hipLaunchKernelGGL((t2d_spread_fast_kernel<4, 4>), grid, block, 0, st, q);
        else hipLaunchKernelGGL((t2d_spread_fast_kernel<4, 1>), grid, block, 0, st, q);
    } else if (elsz == 2) {
        hipLaunchKernelGGL(t2d_spread_kernel<2>, dim3(blocks_for(p.ld.numel)), dim3(kT2dThreads), 0, st, p);
    } else {
        hipLaunchKernelGGL(t2d_spread_kernel<4>, dim3(blocks_for(p.ld.numel)), dim3(kT2dThreads), 0, st, p);
    }
    ALT_CHECK_HIP(h, hipGetLastError());
    return alt_conv2d(h, &f, workspace, w_packed, bias, y, (char *)workspace + xe_bytes, ws_bytes - xe_bytes, stream);
}

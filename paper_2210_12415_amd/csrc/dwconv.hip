// Depth-wise 2-D convolution (one filter per channel: groups = C = K), the
// memory-bound member of the C2D family of Section 6.1 of the paper:
//   y[n,c,oh,ow] = sum_{r,s} x[n,c,oh*stride-pad+r*dil, ow*stride-pad+s*dil] * w[c,0,r,s]
// fp32 accumulation over the taps in (r, s) order, then bias, ReLU and the
// output rounding.  There is no reduction over channels, so nothing for the
// matrix cores to do: the kernels are a gather over the filter window, and
// the data layout decides how wide the accesses are.
//
//  * vector kernel: bf16 tensors whose channel is contiguous in runs of at
//    least eight on activations, weights and output (NHWC or NCHW[x]c with
//    channel-last weights): a thread owns eight channels of one output pixel,
//    every access is 16 bytes;
//    (3x3 filters without dilation get a register-tiled version of it);
//  * row kernel: bf16 tensors whose width is contiguous on activations and
//    output (NCHW), 3x3 filters with padding 1 along the width: a thread owns
//    four or eight consecutive outputs of one row of one channel plane,
//    reads the input columns under them as 8- or 16-byte vectors (plus the
//    column before them) and stores one such vector;
//  * element kernel: any separable layout; a thread owns one output element,
//    threads run along the output's contiguous dimension.
#include <hip/hip_runtime.h>

#include "igemm.h"
#include "ops.h"

namespace alt {
namespace {

constexpr int kDwThreads = 256;

struct DwParams {
    const void *x, *w;
    const float *bias;
    void *y;
    int32_t N, C, H, W, R, S, OH, OW;
    int32_t stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
    int32_t epilogue, in_bf16, out_bf16, chan_fast;
    Dim2 xn, xc, xh, xw, wo, wr, ws, yn, yk, yh, yw;
};

__device__ __forceinline__ float load_elem(const void *p, int64_t off, int bf16)
{
    if (bf16) return __builtin_bit_cast(float, (uint32_t)((const uint16_t *)p)[off] << 16);
    return ((const float *)p)[off];
}

__global__ __launch_bounds__(kDwThreads) void dwconv_elem_kernel(const DwParams p)
{
    const int64_t total = (int64_t)p.N * p.C * p.OH * p.OW;
    for (int64_t e = blockIdx.x * (int64_t)kDwThreads + threadIdx.x; e < total; e += (int64_t)gridDim.x * kDwThreads) {
        int n, c, oh, ow;
        if (total <= 0x7fffffff) {                  // 32-bit divisions cost a fraction of 64-bit ones
            uint32_t r = (uint32_t)e;
            if (p.chan_fast) {
                c = (int)(r % (uint32_t)p.C); r /= (uint32_t)p.C;
                ow = (int)(r % (uint32_t)p.OW); r /= (uint32_t)p.OW;
                oh = (int)(r % (uint32_t)p.OH); n = (int)(r / (uint32_t)p.OH);
            } else {
                ow = (int)(r % (uint32_t)p.OW); r /= (uint32_t)p.OW;
                oh = (int)(r % (uint32_t)p.OH); r /= (uint32_t)p.OH;
                c = (int)(r % (uint32_t)p.C); n = (int)(r / (uint32_t)p.C);
            }
        } else {
            int64_t r = e;
            if (p.chan_fast) {
                c = (int)(r % p.C); r /= p.C;
                ow = (int)(r % p.OW); r /= p.OW;
                oh = (int)(r % p.OH); n = (int)(r / p.OH);
            } else {
                ow = (int)(r % p.OW); r /= p.OW;
                oh = (int)(r % p.OH); r /= p.OH;
                c = (int)(r % p.C); n = (int)(r / p.C);
            }
        }
        const int64_t xb = dim2_off(p.xn, n) + dim2_off(p.xc, c), wb = dim2_off(p.wo, c);
        float acc = 0.f;
        // (H, W, R and S are rarely blocked: then an offset is a multiply, not a division)
        const bool lin = p.xh.f >= p.H && p.xw.f >= p.W && p.wr.f >= p.R && p.ws.f >= p.S;
        for (int fr = 0; fr < p.R; ++fr) {
            const int ih = oh * p.stride_h - p.pad_h + fr * p.dil_h;
            if ((unsigned)ih >= (unsigned)p.H) continue;
            const int64_t xr = xb + (lin ? ih * p.xh.si : dim2_off(p.xh, ih));
            const int64_t wr = wb + (lin ? fr * p.wr.si : dim2_off(p.wr, fr));
            for (int fs = 0; fs < p.S; ++fs) {
                const int iw = ow * p.stride_w - p.pad_w + fs * p.dil_w;
                if ((unsigned)iw >= (unsigned)p.W) continue;
                acc += load_elem(p.x, xr + (lin ? iw * p.xw.si : dim2_off(p.xw, iw)), p.in_bf16) *
                       load_elem(p.w, wr + (lin ? fs * p.ws.si : dim2_off(p.ws, fs)), p.in_bf16);
            }
        }
        if (p.epilogue & ALT_EPI_BIAS) acc += p.bias[c];
        if (p.epilogue & ALT_EPI_RELU) acc = fmaxf(acc, 0.f);
        const int64_t yo = dim2_off(p.yn, n) + dim2_off(p.yk, c) + dim2_off(p.yh, oh) + dim2_off(p.yw, ow);
        if (p.out_bf16) ((uint16_t *)p.y)[yo] = f32_to_bf16_rne(acc);
        else ((float *)p.y)[yo] = acc;
    }
}

// bf16 in and out, eight consecutive channels per thread (one 16-byte access per tensor and tap).
__global__ __launch_bounds__(kDwThreads) void dwconv_vec8_kernel(const DwParams p)
{
    typedef uint32_t w4_t __attribute__((ext_vector_type(4)));
    typedef float f4_t __attribute__((ext_vector_type(4)));
    const int C8 = p.C >> 3;
    const int64_t total = (int64_t)p.N * p.OH * p.OW * C8;
    for (int64_t e = blockIdx.x * (int64_t)kDwThreads + threadIdx.x; e < total; e += (int64_t)gridDim.x * kDwThreads) {
        int64_t r = e;
        const int c = (int)(r % C8) * 8; r /= C8;
        const int ow = (int)(r % p.OW); r /= p.OW;
        const int oh = (int)(r % p.OH);
        const int n = (int)(r / p.OH);
        const int64_t xb = dim2_off(p.xn, n) + dim2_off(p.xc, c), wb = dim2_off(p.wo, c);
        // even channels of each pair in lo, odd ones in hi (whole-vector arithmetic throughout)
        f4_t lo = {0.f, 0.f, 0.f, 0.f}, hi = {0.f, 0.f, 0.f, 0.f};
        for (int fr = 0; fr < p.R; ++fr) {
            const int ih = oh * p.stride_h - p.pad_h + fr * p.dil_h;
            if ((unsigned)ih >= (unsigned)p.H) continue;
            for (int fs = 0; fs < p.S; ++fs) {
                const int iw = ow * p.stride_w - p.pad_w + fs * p.dil_w;
                if ((unsigned)iw >= (unsigned)p.W) continue;
                const w4_t xv = *(const w4_t *)((const uint16_t *)p.x + xb + dim2_off(p.xh, ih) + dim2_off(p.xw, iw));
                const w4_t wv = *(const w4_t *)((const uint16_t *)p.w + wb + dim2_off(p.wr, fr) + dim2_off(p.ws, fs));
                lo += __builtin_bit_cast(f4_t, xv << 16) * __builtin_bit_cast(f4_t, wv << 16);
                hi += __builtin_bit_cast(f4_t, xv & 0xffff0000u) * __builtin_bit_cast(f4_t, wv & 0xffff0000u);
            }
        }
        if (p.epilogue & ALT_EPI_BIAS) {
            const f4_t b0 = *(const f4_t *)(p.bias + c), b1 = *(const f4_t *)(p.bias + c + 4);
            lo += __builtin_shufflevector(b0, b1, 0, 2, 4, 6);
            hi += __builtin_shufflevector(b0, b1, 1, 3, 5, 7);
        }
        if (p.epilogue & ALT_EPI_RELU) {
            lo = __builtin_elementwise_max(lo, (f4_t){0.f, 0.f, 0.f, 0.f});
            hi = __builtin_elementwise_max(hi, (f4_t){0.f, 0.f, 0.f, 0.f});
        }
        w4_t out;
#pragma unroll
        for (int q = 0; q < 4; ++q) out[q] = f32x2_to_bf16x2(lo[q], hi[q]);
        const int64_t yo = dim2_off(p.yn, n) + dim2_off(p.yk, c) + dim2_off(p.yh, oh) + dim2_off(p.yw, ow);
        *(w4_t *)((uint16_t *)p.y + yo) = out;
    }
}

// The common case of the vector kernel: 3x3 filter, dilation 1, H and W not blocked.  A thread
// owns eight channels of TW consecutive output pixels of one row: the nine weight vectors are
// loaded once, and neighbouring outputs share the input columns of their windows, so a thread
// makes 3 * ((TW - 1) * STRIDE + 3) + 9 loads for TW outputs instead of 18 per output.
// (At stride 1 the register count is held to four waves per SIMD: the benchmark layers are 3.4
// waves per SIMD of work, so every thread is then resident at once; at stride 2 the nine input
// columns of a row do not fit that budget without spilling.)
template <int STRIDE, int TW>
__global__ __launch_bounds__(kDwThreads, STRIDE == 1 ? 4 : 3) void dwconv_vec8_3x3_kernel(const DwParams p)
{
    typedef uint32_t w4_t __attribute__((ext_vector_type(4)));
    typedef float f4_t __attribute__((ext_vector_type(4)));
    constexpr int NCOL = (TW - 1) * STRIDE + 3;
    const int C8 = p.C >> 3, OWB = (p.OW + TW - 1) / TW;
    const int64_t total = (int64_t)p.N * p.OH * OWB * C8;
    const int64_t sxh = p.xh.si, sxw = p.xw.si, syh = p.yh.si, syw = p.yw.si;
    for (int64_t e = blockIdx.x * (int64_t)kDwThreads + threadIdx.x; e < total; e += (int64_t)gridDim.x * kDwThreads) {
        int c, ow0, oh, n;
        if (total <= 0x7fffffff) {                  // 32-bit divisions cost a fraction of 64-bit ones
            uint32_t r = (uint32_t)e;
            c = (int)(r % (uint32_t)C8) * 8; r /= (uint32_t)C8;
            ow0 = (int)(r % (uint32_t)OWB) * TW; r /= (uint32_t)OWB;
            oh = (int)(r % (uint32_t)p.OH);
            n = (int)(r / (uint32_t)p.OH);
        } else {
            int64_t r = e;
            c = (int)(r % C8) * 8; r /= C8;
            ow0 = (int)(r % OWB) * TW; r /= OWB;
            oh = (int)(r % p.OH);
            n = (int)(r / p.OH);
        }
        const uint16_t *xb = (const uint16_t *)p.x + dim2_off(p.xn, n) + dim2_off(p.xc, c);
        const uint16_t *wb = (const uint16_t *)p.w + dim2_off(p.wo, c);
        w4_t wv[9];                                 // kept packed: unpacked where used, half the registers
#pragma unroll
        for (int t = 0; t < 9; ++t) wv[t] = *(const w4_t *)(wb + dim2_off(p.wr, t / 3) + dim2_off(p.ws, t % 3));
        f4_t lo[TW], hi[TW];
#pragma unroll
        for (int j = 0; j < TW; ++j) { lo[j] = (f4_t){0.f, 0.f, 0.f, 0.f}; hi[j] = (f4_t){0.f, 0.f, 0.f, 0.f}; }
        const int ih0 = oh * STRIDE - p.pad_h, iw0 = ow0 * STRIDE - p.pad_w;
#pragma unroll
        for (int fr = 0; fr < 3; ++fr) {
            const int ih = ih0 + fr;
            if ((unsigned)ih >= (unsigned)p.H) continue;
            const uint16_t *row = xb + ih * sxh;
            f4_t xlo[NCOL], xhi[NCOL];
#pragma unroll
            for (int q = 0; q < NCOL; ++q) {
                const int iw = iw0 + q;
                w4_t xv = {0u, 0u, 0u, 0u};
                if ((unsigned)iw < (unsigned)p.W) xv = *(const w4_t *)(row + iw * sxw);
                xlo[q] = __builtin_bit_cast(f4_t, xv << 16);
                xhi[q] = __builtin_bit_cast(f4_t, xv & 0xffff0000u);
            }
#pragma unroll
            for (int fs = 0; fs < 3; ++fs) {
                const f4_t wl = __builtin_bit_cast(f4_t, wv[fr * 3 + fs] << 16);
                const f4_t wh = __builtin_bit_cast(f4_t, wv[fr * 3 + fs] & 0xffff0000u);
#pragma unroll
                for (int j = 0; j < TW; ++j) {
                    lo[j] += xlo[j * STRIDE + fs] * wl;
                    hi[j] += xhi[j * STRIDE + fs] * wh;
                }
            }
        }
        f4_t blo = {0.f, 0.f, 0.f, 0.f}, bhi = {0.f, 0.f, 0.f, 0.f};
        if (p.epilogue & ALT_EPI_BIAS) {
            const f4_t b0 = *(const f4_t *)(p.bias + c), b1 = *(const f4_t *)(p.bias + c + 4);
            blo = __builtin_shufflevector(b0, b1, 0, 2, 4, 6);
            bhi = __builtin_shufflevector(b0, b1, 1, 3, 5, 7);
        }
        const float floor_ = (p.epilogue & ALT_EPI_RELU) ? 0.f : -INFINITY;
        uint16_t *yb = (uint16_t *)p.y + dim2_off(p.yn, n) + dim2_off(p.yk, c) + oh * syh;
#pragma unroll
        for (int j = 0; j < TW; ++j) {
            if (ow0 + j >= p.OW) break;
            const f4_t a = __builtin_elementwise_max(lo[j] + blo, (f4_t){floor_, floor_, floor_, floor_});
            const f4_t b = __builtin_elementwise_max(hi[j] + bhi, (f4_t){floor_, floor_, floor_, floor_});
            w4_t out;
#pragma unroll
            for (int q = 0; q < 4; ++q) out[q] = f32x2_to_bf16x2(a[q], b[q]);
            *(w4_t *)(yb + (ow0 + j) * syw) = out;
        }
    }
}

// bf16 in and out, width contiguous, 3x3 without dilation, padding 1 along the width, W and OW multiples of TW
// (four or eight; checked by the host together with the alignment of every plane and row).  A thread computes
// outputs (oh, ow0 .. ow0+TW-1) of one (n, c) plane from input columns ow0*STRIDE - 1 .. : the columns from
// ow0*STRIDE on come as aligned vectors of TW elements (wholly inside or wholly outside the row), the one before
// them as a scalar.
template <int STRIDE, int TW>
__global__ __launch_bounds__(kDwThreads) void dwconv_rows_3x3_kernel(const DwParams p)
{
    typedef uint32_t wv_t __attribute__((ext_vector_type(TW / 2)));     // TW bf16: 8 bytes (TW = 4) or 16 (TW = 8)
    constexpr int NCOL = (TW - 1) * STRIDE + 3;            // input columns under TW outputs
    constexpr int NV = (NCOL - 1 + TW - 1) / TW;           // vectors that cover columns 1 .. NCOL-1
    const uint32_t OWB = (uint32_t)p.OW / TW;
    const int64_t total = (int64_t)p.N * p.C * p.OH * OWB;
    const int64_t sxh = p.xh.si, syh = p.yh.si;
    for (int64_t e = blockIdx.x * (int64_t)kDwThreads + threadIdx.x; e < total; e += (int64_t)gridDim.x * kDwThreads) {
        int c, ow0, oh, n;
        if (total <= 0x7fffffff) {
            uint32_t r = (uint32_t)e;
            ow0 = (int)(r % OWB) * TW; r /= OWB;
            oh = (int)(r % (uint32_t)p.OH); r /= (uint32_t)p.OH;
            c = (int)(r % (uint32_t)p.C);
            n = (int)(r / (uint32_t)p.C);
        } else {
            int64_t r = e;
            ow0 = (int)(r % OWB) * TW; r /= OWB;
            oh = (int)(r % p.OH); r /= p.OH;
            c = (int)(r % p.C);
            n = (int)(r / p.C);
        }
        const uint16_t *xb = (const uint16_t *)p.x + dim2_off(p.xn, n) + dim2_off(p.xc, c);
        const uint16_t *wb = (const uint16_t *)p.w + dim2_off(p.wo, c);
        float wq[9];
#pragma unroll
        for (int t = 0; t < 9; ++t)
            wq[t] = __builtin_bit_cast(float, (uint32_t)wb[(t / 3) * p.wr.si + (t % 3) * p.ws.si] << 16);
        float acc[TW];
#pragma unroll
        for (int j = 0; j < TW; ++j) acc[j] = 0.f;
        const int ih0 = oh * STRIDE - p.pad_h, iw1 = ow0 * STRIDE;      // column 1 of the window: a multiple of TW
#pragma unroll
        for (int fr = 0; fr < 3; ++fr) {
            const int ih = ih0 + fr;
            if ((unsigned)ih >= (unsigned)p.H) continue;
            const uint16_t *row = xb + ih * sxh;
            float xv[1 + TW * NV];
            xv[0] = iw1 > 0 ? __builtin_bit_cast(float, (uint32_t)row[iw1 - 1] << 16) : 0.f;
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                wv_t d;
                __builtin_memset(&d, 0, sizeof d);
                if (iw1 + TW * v < p.W) d = *(const wv_t *)(row + iw1 + TW * v);
#pragma unroll
                for (int q = 0; q < TW / 2; ++q) {
                    xv[1 + TW * v + 2 * q] = __builtin_bit_cast(float, d[q] << 16);
                    xv[2 + TW * v + 2 * q] = __builtin_bit_cast(float, d[q] & 0xffff0000u);
                }
            }
#pragma unroll
            for (int fs = 0; fs < 3; ++fs)
#pragma unroll
                for (int j = 0; j < TW; ++j) acc[j] += xv[j * STRIDE + fs] * wq[fr * 3 + fs];
        }
        const float bias = (p.epilogue & ALT_EPI_BIAS) ? p.bias[c] : 0.f;
        const float floor_ = (p.epilogue & ALT_EPI_RELU) ? 0.f : -INFINITY;
        wv_t out;
#pragma unroll
        for (int q = 0; q < TW / 2; ++q)
            out[q] = f32x2_to_bf16x2(fmaxf(acc[2 * q] + bias, floor_), fmaxf(acc[2 * q + 1] + bias, floor_));
        uint16_t *yb = (uint16_t *)p.y + dim2_off(p.yn, n) + dim2_off(p.yk, c) + oh * syh + ow0;
        *(wv_t *)yb = out;
    }
}

// every offset of a plane or row start is a multiple of m elements
bool rows_of(int m, const Dim2 *d, int n)
{
    for (int i = 0; i < n; ++i)
        if (d[i].so % m || d[i].si % m) return false;
    return true;
}

// eight consecutive channels from a multiple of eight are one contiguous, 16-byte aligned run
bool chan_runs_of_8(const Dim2 &c, int64_t C, const Dim2 *others, int n_others)
{
    const int64_t run = c.f >= C ? C : c.f;
    if (c.si != 1 || run % 8 || C % 8) return false;
    if (c.f < C && c.so % 8) return false;
    for (int i = 0; i < n_others; ++i)
        if (others[i].so % 8 || others[i].si % 8) return false;
    return true;
}

}  // namespace

// pb is the problem of one group (C = K = 1 per group, batch = channels) as conv_problem fills it for
// a depth-wise descriptor; x/w/y Dim2 entries describe the whole tensors.
alt_status_t depthwise_run(alt_handle_t h, const Problem &pb, int64_t N, int64_t C, hipStream_t st)
{
    if (!h->has_gpu) return fail(h, ALT_HIP_ERROR, "no GPU device available");
    const IgemmParams &q = pb.p;
    DwParams p;
    std::memset(&p, 0, sizeof p);
    p.x = q.x; p.w = q.w; p.bias = q.bias; p.y = q.y;
    p.N = (int32_t)N; p.C = (int32_t)C; p.H = q.H; p.W = q.W; p.R = q.R; p.S = q.S; p.OH = q.OH; p.OW = q.OW;
    p.stride_h = q.stride_h; p.stride_w = q.stride_w; p.pad_h = q.pad_h; p.pad_w = q.pad_w;
    p.dil_h = q.dil_h; p.dil_w = q.dil_w;
    p.epilogue = q.epilogue; p.in_bf16 = pb.dtype == ALT_BF16; p.out_bf16 = q.out_bf16;
    p.xn = q.xn; p.xc = q.xc; p.xh = q.xh; p.xw = q.xw;
    p.wo = q.wo; p.wr = q.wr; p.ws = q.ws;
    p.yn = q.yn; p.yk = q.yk; p.yh = q.yh; p.yw = q.yw;
    p.chan_fast = q.yk.si == 1;
    const Dim2 xo[3] = {q.xn, q.xh, q.xw}, wo_[2] = {q.wr, q.ws}, yo[3] = {q.yn, q.yh, q.yw};
    const bool vec = p.in_bf16 && p.out_bf16 && chan_runs_of_8(q.xc, C, xo, 3) && chan_runs_of_8(q.wo, C, wo_, 2) &&
                     chan_runs_of_8(q.yk, C, yo, 3) && (uintptr_t)q.x % 16 == 0 && (uintptr_t)q.w % 16 == 0 &&
                     (uintptr_t)q.y % 16 == 0 && (!(q.epilogue & ALT_EPI_BIAS) || (uintptr_t)q.bias % 16 == 0);
    constexpr int kTW = 4;
    const bool k3x3 = vec && q.R == 3 && q.S == 3 && q.dil_h == 1 && q.dil_w == 1 && q.stride_h == q.stride_w &&
                      (q.stride_h == 1 || q.stride_h == 2) && q.xh.f >= q.H && q.xw.f >= q.W && q.yh.f >= q.OH &&
                      q.yw.f >= q.OW;
    const Dim2 xr[3] = {q.xn, q.xc, q.xh}, yr[3] = {q.yn, q.yk, q.yh};
    const bool rows = !vec && p.in_bf16 && p.out_bf16 && q.R == 3 && q.S == 3 && q.dil_h == 1 && q.dil_w == 1 &&
                      q.stride_h == q.stride_w && (q.stride_h == 1 || q.stride_h == 2) && q.pad_w == 1 && q.xw.si == 1 &&
                      q.xw.f >= q.W && q.xh.f >= q.H && q.yw.si == 1 && q.yw.f >= q.OW && q.yh.f >= q.OH && q.wr.f >= 3 &&
                      q.ws.f >= 3 && q.W % 4 == 0 && q.OW % 4 == 0 && rows_of(4, xr, 3) && rows_of(4, yr, 3) &&
                      (uintptr_t)q.x % 8 == 0 && (uintptr_t)q.y % 8 == 0;
    // eight outputs per thread in 16-byte accesses where the rows allow it
    const bool rows8 = rows && q.W % 8 == 0 && q.OW % 8 == 0 && rows_of(8, xr, 3) && rows_of(8, yr, 3) &&
                       (uintptr_t)q.x % 16 == 0 && (uintptr_t)q.y % 16 == 0;
    const int64_t work = rows ? N * C * q.OH * (q.OW / (rows8 ? 8 : 4))
                       : k3x3 ? N * q.OH * ((q.OW + kTW - 1) / kTW) * (C / 8) : N * q.OH * q.OW * (vec ? C / 8 : C);
    const unsigned blocks = (unsigned)std::min<int64_t>((work + kDwThreads - 1) / kDwThreads, 256 * 64);
    if (rows8 && q.stride_h == 1) hipLaunchKernelGGL((dwconv_rows_3x3_kernel<1, 8>), dim3(blocks), dim3(kDwThreads), 0, st, p);
    else if (rows8) hipLaunchKernelGGL((dwconv_rows_3x3_kernel<2, 8>), dim3(blocks), dim3(kDwThreads), 0, st, p);
    else if (rows && q.stride_h == 1) hipLaunchKernelGGL((dwconv_rows_3x3_kernel<1, 4>), dim3(blocks), dim3(kDwThreads), 0, st, p);
    else if (rows) hipLaunchKernelGGL((dwconv_rows_3x3_kernel<2, 4>), dim3(blocks), dim3(kDwThreads), 0, st, p);
    else if (k3x3 && q.stride_h == 1) hipLaunchKernelGGL((dwconv_vec8_3x3_kernel<1, kTW>), dim3(blocks), dim3(kDwThreads), 0, st, p);
    else if (k3x3) hipLaunchKernelGGL((dwconv_vec8_3x3_kernel<2, kTW>), dim3(blocks), dim3(kDwThreads), 0, st, p);
    else if (vec) hipLaunchKernelGGL(dwconv_vec8_kernel, dim3(blocks), dim3(kDwThreads), 0, st, p);
    else hipLaunchKernelGGL(dwconv_elem_kernel, dim3(blocks), dim3(kDwThreads), 0, st, p);
    ALT_CHECK_HIP(h, hipGetLastError());
    return ALT_OK;
}

}  // namespace alt

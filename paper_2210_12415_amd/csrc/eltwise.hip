// Element-wise operators of a graph (Section 4.2 of the paper: simple operators
// take the layout of their producer, so they see flat buffers).  y = a + b,
// optionally followed by ReLU; b may be absent (y = relu(a)).  HBM-bound:
// 16 bytes per lane per access, write-through stores.
#include <hip/hip_runtime.h>

#include "common.h"
#include "igemm.h"

namespace alt {
namespace {

constexpr int kEltThreads = 256;

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }

// n16 = number of whole 16-byte vectors; the tail (fewer than 16 bytes) is handled element by element.
template <int ELSZ>
__global__ __launch_bounds__(kEltThreads) void eltwise_add_kernel(const void *a, const void *b, void *y, int64_t numel,
                                                                  int relu)
{
    typedef uint32_t w4_t __attribute__((ext_vector_type(4)));
    typedef float f4_t __attribute__((ext_vector_type(4)));
    constexpr int EPV = 16 / ELSZ;
    const float floor_ = relu ? 0.f : -INFINITY;
    const int64_t n16 = numel / EPV;
    for (int64_t v = blockIdx.x * (int64_t)kEltThreads + threadIdx.x; v < n16; v += (int64_t)gridDim.x * kEltThreads) {
        // (whole-vector arithmetic: element-wise float views of a loaded vector are miscompiled
        // into a single-dword load by this toolchain)
        w4_t out;
        if constexpr (ELSZ == 4) {
            f4_t s = ((const f4_t *)a)[v];
            if (b) s += ((const f4_t *)b)[v];
            s = __builtin_elementwise_max(s, (f4_t){floor_, floor_, floor_, floor_});
            out = __builtin_bit_cast(w4_t, s);
        } else {
            const w4_t va = ((const w4_t *)a)[v];
            f4_t lo = __builtin_bit_cast(f4_t, va << 16), hi = __builtin_bit_cast(f4_t, va & 0xffff0000u);
            if (b) {
                const w4_t vb = ((const w4_t *)b)[v];
                lo += __builtin_bit_cast(f4_t, vb << 16);
                hi += __builtin_bit_cast(f4_t, vb & 0xffff0000u);
            }
            lo = __builtin_elementwise_max(lo, (f4_t){floor_, floor_, floor_, floor_});
            hi = __builtin_elementwise_max(hi, (f4_t){floor_, floor_, floor_, floor_});
#pragma unroll
            for (int q = 0; q < 4; ++q) out[q] = f32x2_to_bf16x2(lo[q], hi[q]);
        }
        char *dst = (char *)y + v * 16;
        // (s_nop: the store reads its four data registers up to two cycles after it issues, and the
        // compiler does not guard registers of an asm statement against the next VALU write)
        asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1\n\ts_nop 1" : : "v"(dst), "v"(out) : "memory");
    }
    // tail
    const int64_t t0 = n16 * EPV;
    if (blockIdx.x == 0 && threadIdx.x < numel - t0) {
        const int64_t i = t0 + threadIdx.x;
        if constexpr (ELSZ == 4) {
            const float s = ((const float *)a)[i] + (b ? ((const float *)b)[i] : 0.f);
            ((float *)y)[i] = fmaxf(s, floor_);
        } else {
            const float s = bf16_lo(((const uint16_t *)a)[i]) + (b ? bf16_lo(((const uint16_t *)b)[i]) : 0.f);
            ((uint16_t *)y)[i] = f32_to_bf16_rne(fmaxf(s, floor_));
        }
    }
}

}  // namespace

alt_status_t eltwise_add(alt_handle_t h, int dtype, int64_t numel, const void *a, const void *b, void *y, int relu,
                         hipStream_t st)
{
    if (!h->has_gpu) return fail(h, ALT_HIP_ERROR, "no GPU device available");
    if (numel == 0) return ALT_OK;
    const int64_t vecs = numel / (dtype == ALT_F32 ? 4 : 8);
    const unsigned blocks = (unsigned)std::min<int64_t>(std::max<int64_t>((vecs + kEltThreads - 1) / kEltThreads, 1), 256 * 16);
    if (dtype == ALT_F32) hipLaunchKernelGGL(eltwise_add_kernel<4>, dim3(blocks), dim3(kEltThreads), 0, st, a, b, y, numel, relu);
    else hipLaunchKernelGGL(eltwise_add_kernel<2>, dim3(blocks), dim3(kEltThreads), 0, st, a, b, y, numel, relu);
    ALT_CHECK_HIP(h, hipGetLastError());
    return ALT_OK;
}

}  // namespace alt

using namespace alt;

extern "C" alt_status_t alt_eltwise_add(alt_handle_t h, alt_dtype_t dtype, int64_t numel, const void *a, const void *b,
                                        void *y, int relu, void *stream)
{
    if (!h) return ALT_INVALID_ARG;
    if (dtype != ALT_F32 && dtype != ALT_BF16) return fail(h, ALT_INVALID_ARG, "alt_eltwise_add: bad dtype");
    if (numel < 0) return fail(h, ALT_INVALID_ARG, "alt_eltwise_add: negative size");
    if (numel > 0 && (!a || !y)) return fail(h, ALT_INVALID_ARG, "alt_eltwise_add: null buffer");
    if (((uintptr_t)a | (uintptr_t)b | (uintptr_t)y) % 16) return fail(h, ALT_INVALID_ARG, "alt_eltwise_add: buffers must be 16-byte aligned");
    return eltwise_add(h, (int)dtype, numel, a, b, y, relu, (hipStream_t)stream);
}

// Attainable peaks of the device, measured with two micro-kernels: a large
// streaming copy (HBM) and a register-resident bf16 MFMA loop (matrix cores).
#include "igemm.h"

namespace alt {
namespace {

__global__ __launch_bounds__(256) void stream_copy_kernel(const uint4 *src, uint4 *dst, size_t n)
{
    for (size_t i = blockIdx.x * (size_t)256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void mfma_loop_kernel(float *sink, int iters)
{
    floatx16_t acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
    uint4 a = make_uint4(0x3f803f80u + threadIdx.x, 0x3f803f80u, 0x3f003f00u, 0x3f803f80u);
    uint4 b = make_uint4(0x3f803f80u, 0x3f003f00u + blockIdx.x, 0x3f803f80u, 0x3f803f80u);
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int j = 0; j < 4; ++j) mma_tile(acc[j], a, b, bf16_tag{});
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[j][e];
    if (s == 12345.678f) sink[0] = s;      // keeps the loop alive without a store in practice
}

}  // namespace
}  // namespace alt

using namespace alt;

extern "C" alt_status_t alt_get_peak(alt_handle_t h, void *arena, size_t arena_bytes, alt_peaks_t *out)
{
    if (!h) return ALT_INVALID_ARG;
    if (!out) return fail(h, ALT_INVALID_ARG, "null argument");
    std::memset(out, 0, sizeof *out);
    out->nominal_hbm_gbps = 8000.f;
    out->nominal_bf16_tflops = 2500.f;
    out->compute_units = h->compute_units;
    out->clock_mhz = h->clock_mhz;
    std::snprintf(out->arch, sizeof out->arch, "%s", h->arch.c_str());
    if (!h->has_gpu) return fail(h, ALT_HIP_ERROR, "no GPU device available");
    if (!arena || arena_bytes < (1u << 20)) return fail(h, ALT_INVALID_ARG, "alt_get_peak needs an arena of at least 1 MiB");
    hipEvent_t e0, e1;
    ALT_CHECK_HIP(h, hipEventCreate(&e0));
    ALT_CHECK_HIP(h, hipEventCreate(&e1));
    const size_t half = (arena_bytes / 2) & ~(size_t)255;
    const size_t n = half / 16;
    const int cus = h->compute_units > 0 ? h->compute_units : 256;
    float ms = 0.f;
    for (int pass = 0; pass < 2; ++pass) {
        ALT_CHECK_HIP(h, hipEventRecord(e0, 0));
        for (int r = 0; r < 10; ++r)
            hipLaunchKernelGGL(stream_copy_kernel, dim3(cus * 8), dim3(256), 0, 0, (const uint4 *)arena,
                               (uint4 *)((char *)arena + half), n);
        ALT_CHECK_HIP(h, hipEventRecord(e1, 0));
        ALT_CHECK_HIP(h, hipEventSynchronize(e1));
        ALT_CHECK_HIP(h, hipEventElapsedTime(&ms, e0, e1));
    }
    out->copy_gbps = (float)(2.0 * half * 10 / (ms * 1e-3) / 1e9);
    const int iters = 20000;
    for (int pass = 0; pass < 2; ++pass) {
        ALT_CHECK_HIP(h, hipEventRecord(e0, 0));
        hipLaunchKernelGGL(mfma_loop_kernel, dim3(cus * 4), dim3(256), 0, 0, (float *)arena, iters);
        ALT_CHECK_HIP(h, hipEventRecord(e1, 0));
        ALT_CHECK_HIP(h, hipEventSynchronize(e1));
        ALT_CHECK_HIP(h, hipEventElapsedTime(&ms, e0, e1));
    }
    const double flops = (double)cus * 4 * 4 * iters * 4 * (2.0 * 32 * 32 * 16);
    out->mfma_bf16_tflops = (float)(flops / (ms * 1e-3) / 1e12);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    ALT_CHECK_HIP(h, hipGetLastError());
    return ALT_OK;
}

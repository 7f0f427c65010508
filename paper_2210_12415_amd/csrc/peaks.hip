// Attainable peaks of the device, measured with micro-kernels: large streaming
// copy, read-only and write-only passes (HBM) and a register-resident bf16 MFMA
// loop (matrix cores).
#include "igemm.h"

namespace alt {
namespace {

// Plain streams over a large buffer.  A thread keeps four independent 16-byte accesses in
// flight per trip; consecutive threads touch consecutive 16-byte pieces, the four accesses of a
// trip are one grid-wide stride apart.
__global__ __launch_bounds__(256) void stream_copy_kernel(const uint4 *src, uint4 *dst, size_t n)
{
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = blockIdx.x * (size_t)256 + threadIdx.x;
    for (; i + 3 * stride < n; i += 4 * stride) {
        const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        dst[i] = a; dst[i + stride] = b; dst[i + 2 * stride] = c; dst[i + 3 * stride] = d;
    }
    for (; i < n; i += stride) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void stream_read_kernel(const uint4 *src, uint4 *sink, size_t n)
{
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = blockIdx.x * (size_t)256 + threadIdx.x;
    uint4 s = make_uint4(0, 0, 0, 0);
    for (; i + 3 * stride < n; i += 4 * stride) {
        const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        s.x ^= a.x ^ b.x ^ c.x ^ d.x; s.y ^= a.y ^ b.y ^ c.y ^ d.y;
        s.z ^= a.z ^ b.z ^ c.z ^ d.z; s.w ^= a.w ^ b.w ^ c.w ^ d.w;
    }
    for (; i < n; i += stride) { const uint4 a = src[i]; s.x ^= a.x; s.y ^= a.y; s.z ^= a.z; s.w ^= a.w; }
    // one 16-byte store per thread: 1/(trips*4) of the bytes read, and it keeps the loads alive
    sink[blockIdx.x * (size_t)256 + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void stream_write_kernel(uint4 *dst, size_t n, uint32_t v)
{
    const size_t stride = (size_t)gridDim.x * 256;
    const uint4 w = make_uint4(v, v + 1, v + 2, v + 3);
    for (size_t i = blockIdx.x * (size_t)256 + threadIdx.x; i < n; i += stride) dst[i] = w;
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
    const int blocks = cus * 8;
    for (int pass = 0; pass < 2; ++pass) {
        ALT_CHECK_HIP(h, hipEventRecord(e0, 0));
        for (int r = 0; r < 10; ++r)
            hipLaunchKernelGGL(stream_copy_kernel, dim3(blocks), dim3(256), 0, 0, (const uint4 *)arena,
                               (uint4 *)((char *)arena + half), n);
        ALT_CHECK_HIP(h, hipEventRecord(e1, 0));
        ALT_CHECK_HIP(h, hipEventSynchronize(e1));
        ALT_CHECK_HIP(h, hipEventElapsedTime(&ms, e0, e1));
    }
    out->copy_gbps = (float)(2.0 * half * 10 / (ms * 1e-3) / 1e9);
    // read-only and write-only streams over the whole arena (the reader's sink is the first
    // blocks * 4 KiB of the upper half, which the writer then overwrites)
    const size_t whole = (arena_bytes & ~(size_t)255), nw = whole / 16;
    if ((size_t)blocks * 4096 <= half) {
        for (int pass = 0; pass < 2; ++pass) {
            ALT_CHECK_HIP(h, hipEventRecord(e0, 0));
            for (int r = 0; r < 10; ++r)
                hipLaunchKernelGGL(stream_read_kernel, dim3(blocks), dim3(256), 0, 0, (const uint4 *)arena,
                                   (uint4 *)((char *)arena + half), n);
            ALT_CHECK_HIP(h, hipEventRecord(e1, 0));
            ALT_CHECK_HIP(h, hipEventSynchronize(e1));
            ALT_CHECK_HIP(h, hipEventElapsedTime(&ms, e0, e1));
        }
        out->read_gbps = (float)(1.0 * half * 10 / (ms * 1e-3) / 1e9);
    }
    for (int pass = 0; pass < 2; ++pass) {
        ALT_CHECK_HIP(h, hipEventRecord(e0, 0));
        for (int r = 0; r < 10; ++r)
            hipLaunchKernelGGL(stream_write_kernel, dim3(blocks), dim3(256), 0, 0, (uint4 *)arena, nw, (uint32_t)r);
        ALT_CHECK_HIP(h, hipEventRecord(e1, 0));
        ALT_CHECK_HIP(h, hipEventSynchronize(e1));
        ALT_CHECK_HIP(h, hipEventElapsedTime(&ms, e0, e1));
    }
    out->write_gbps = (float)(1.0 * whole * 10 / (ms * 1e-3) / 1e9);
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

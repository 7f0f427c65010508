// Direct convolution with the input patch resident in LDS ("overlapped tile").
//
// The implicit-GEMM kernels of igemm.h fetch the activation operand once per
// filter tap: a 3x3 layer pulls every input element through L2 nine times, and
// for layers with few output channels that traffic, not the matrix cores, sets
// the time.  Here a workgroup owns BM consecutive output pixels (in N*OH*OW
// order) x BN output channels and first brings the input pixels all its taps
// touch into LDS once: the BM pixels plus a halo of pad_h rows and pad_w
// columns on each side, i.e. the tile of the overlapped ("unfold") tiling of
// Section 4.1.2 of the paper, held on chip instead of materialised in memory.
// Every tap then reads its MFMA operand from that patch at a shifted pixel
// index; taps that fall outside the image read an all-zero row instead.  Only
// the weights stream through a ring of LDS stages (direct-to-LDS loads as in
// igemm_dma.h).
//
// Covers: bf16, stride 1 or 2, any dilation, padding from none to "same"
// (2*pad <= dil*(R-1), dil*(S-1), so the output is no larger than the input), activations NHWC,
// weights OHWI, output NHWC (fp32 or bf16), all dense, 64, 128, 256 or 512
// channels per split, output channels a multiple of 4.  The input pixel under
// an output pixel then grows monotonically with the output's linear index,
// across rows and images too (at stride 1 the two indices are equal), so the
// pixels a tile touches are one contiguous range of the input: the patch.  At
// stride 2 that range is four times the tile plus a row, which leaves room
// for 64- and 128-pixel tiles only.
//
// K groups: the waves of a workgroup may form several groups that split the
// slice's channels between them, each with a weight ring of its own; their
// tiles are summed through LDS before the epilogue (see dconv_kernel).  This
// file also holds what the streaming kernel of dstream.h shares with this one:
// the parameter block, the asynchronous LDS reads and the epilogue.
//
// Split-K: grid slices over channel groups (Cs channels each) compute partial
// sums; each writes its fp32 partial tile to the workspace and the last slice
// to arrive (a counter per output tile) sums all slices in slice order and
// runs the epilogue, so the result does not depend on arrival order and no
// second kernel is launched.
#pragma once

#include <utility>

#include "igemm_dma.h"

namespace alt {

// q = n / d for 0 <= n < 2^31: (umulhi(n, mul) + n) >> shift with
// shift = ceil(log2 d), mul = floor(2^32 * (2^shift - d) / d) + 1 (d = 1: mul = 1, shift = 0).
struct Div32 {
    uint32_t mul, shift;
};

inline Div32 make_div32(uint32_t d)
{
    uint32_t l = 0;
    while (((uint64_t)1 << l) < d) ++l;
    Div32 r;
    r.mul = (uint32_t)(((((uint64_t)1 << l) - d) << 32) / d + 1);
    r.shift = l;
    return r;
}

__device__ __forceinline__ uint32_t div32(uint32_t n, Div32 d) { return (__umulhi(n, d.mul) + n) >> d.shift; }

struct DconvParams {
    const void *x, *w;
    const float *bias;
    void *y;
    float *partial;               // [splitk][M][Nc] fp32 partial sums (splitk > 1)
    uint32_t *counters;           // one arrival counter per output tile, zero between launches
    uint32_t x_bytes, w_bytes, y_bytes, partial_bytes;   // partial_bytes: one slice
    int32_t M, Nc, C, Cs;         // Cs = C / splitk channels per slice
    int32_t H, W, R, S, pad_h, pad_w;
    int32_t tiles_m, tiles_n, splitk, flags;             // flags: ALT_EPI_BIAS | ALT_EPI_RELU | 4 (bf16 output)
    Div32 d_hw, d_w, d_tm, d_tn;  // divisions by OH*OW, OW, tiles_m, tiles_n
    int32_t log2_cpp;             // log2(Cs / 8): 16-byte chunks per patch pixel
    Div32 d_slots;                // division by Cs / 8 + 1, the 16-byte slots of a patch pixel in LDS
    int32_t ncc;                  // K steps per tap: (Cs / K groups) / channels per K step
    int32_t bk;                   // channels per K step: 64, or 32 for narrow K groups
    int32_t pad0_;
    Div32 d_sk;                   // division by splitk
    // streaming kernel (dstream.h) only: batch entries and the byte strides between them
    int32_t batch, pad1_;
    int64_t x_bstride, w_bstride, y_bstride;
    // direct kernel only: output image size and stride (H, W above are the input's; M counts
    // output pixels), and the number of input pixels
    int32_t OH, OW, stride, in_px;
    int32_t dil;                  // distance between filter taps, in input pixels (both directions)
    const void *addend;           // added before the activation: same layout and element type as y, or null
    Div32 d_ihw;                  // division by H*W (channel-planar kernel, blocked activations)
    // Channel-blocked tensors (N C/b H W b, b = 1 << blk, at least 8): 0 = channels contiguous per pixel (NHWC)
    int32_t x_blk, y_blk;
};

// Element offset of channel `ch` of input pixel g (= img * H*W + hw) under the activations' layout.
__device__ __forceinline__ uint32_t dconv_in_elem(const DconvParams &p, int g, int ch)
{
    if (p.x_blk == 0) return (uint32_t)(g * p.C + ch);
    const int hw_all = p.H * p.W;
    const int img = (int)div32((uint32_t)g, p.d_ihw), hw = g - img * hw_all;
    return (uint32_t)(img * (p.C * hw_all) + ((((ch >> p.x_blk) * hw_all + hw) << p.x_blk) | (ch & ((1 << p.x_blk) - 1))));
}

// Element offset of channel n of output pixel m (= img * OH*OW + q) under the output's layout.
__device__ __forceinline__ uint32_t dconv_out_elem(const DconvParams &p, int m, int n)
{
    if (p.y_blk == 0) return (uint32_t)(m * p.Nc + n);
    const int ohw = p.OH * p.OW;
    const int img = (int)div32((uint32_t)m, p.d_hw), q = m - img * ohw;
    return (uint32_t)(img * (p.Nc * ohw) + ((((n >> p.y_blk) * ohw + q) << p.y_blk) | (n & ((1 << p.y_blk) - 1))));
}

typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int kDconvOutBf16 = 4;
constexpr int kAgentScope = 16;          // cache-policy operand of buffer loads/stores: sc1 = device (agent) scope
// Output stores carry sc0 + sc1: the lines go through to memory as they are written instead of
// staying dirty in the XCD's L2 until the write-back at the end of the kernel, which
// shortens the gap before the next kernel on the stream (measured: 5 % of a five-layer step).
constexpr int kWriteThrough = 17;
constexpr int kDconvMaxTiles = 4096;     // output tiles a split-K launch may have (one counter each)
constexpr int kDconvSlots = 64;          // counter sets, one per stream that has issued a split-K launch

// Wave-wide 16-byte-per-lane load into LDS at `lds` (+ 16 * lane); the byte
// offset is voff (per lane) + soff (wave-uniform).
__device__ __forceinline__ void dma_load16_s(i32x4_t rsrc, uint32_t voff, uint32_t soff, uint32_t lds)
{
    const uint32_t lds_s = __builtin_amdgcn_readfirstlane(lds);
    const uint32_t soff_s = __builtin_amdgcn_readfirstlane(soff);
    asm volatile("s_mov_b32 m0, %0\n\t"
                 "s_nop 0\n\t"
                 "buffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_s), "v"(voff), "s"(rsrc), "s"(soff_s)
                 : "memory");
}

// LDS operand read whose completion the compiler does not track: the data is
// only valid after lds_wait<N>() on the same registers.
__device__ __forceinline__ void lds_read16_async(u32x4_t &dst, uint32_t addr)
{
    asm volatile("ds_read_b128 %0, %1" : "=v"(dst) : "v"(addr) : "memory");
}

// The same with a compile-time byte offset (an instruction field up to 65535, an add beyond).
template <int OFF>
__device__ __forceinline__ void lds_read16_async_at(u32x4_t &dst, uint32_t addr)
{
    if constexpr (OFF >= 0 && OFF < 65536) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF) : "memory");
    else lds_read16_async(dst, addr + (uint32_t)OFF);
}

typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));

// LDS transpose read of gfx950, 64 bits per lane, 16-bit elements (completion not tracked by the compiler,
// like lds_read16_async): within each group of 16 lanes, lane i receives element i % 4 of the 8 bytes
// that lanes 4j + i / 4 (j = 0..3) address, i.e. with lanes 4j .. 4j+3 on row j of a matrix, column i of rows 0..3.
template <int OFF>
__device__ __forceinline__ void lds_read8_tr_async_at(u32x2_t &dst, uint32_t addr)
{
    if constexpr (OFF >= 0 && OFF < 65536) asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF) : "memory");
    else asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(dst) : "v"(addr + (uint32_t)OFF) : "memory");
}

// lds_wait for fragments whose B halves are read separately.
template <int N, int NA, int NB>
__device__ __forceinline__ void lds_wait_tr(u32x4_t (&a)[NA], u32x2_t (&b)[NB][2])
{
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(a[0]) : "n"(N) : "memory");
#pragma unroll
    for (int i = 1; i < NA; ++i) asm volatile("" : "+v"(a[i]));
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        asm volatile("" : "+v"(b[j][0]));
        asm volatile("" : "+v"(b[j][1]));
    }
}

// f(std::integral_constant<int, 0>) ... f(std::integral_constant<int, N - 1>), in order.
template <typename F, int... I>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// Waits until at most N LDS operations of this wave are outstanding and ties
// the given fragment registers to that point (no use can move above it).
template <int N, int NA, int NB>
__device__ __forceinline__ void lds_wait(u32x4_t (&a)[NA], u32x4_t (&b)[NB])
{
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(a[0]) : "n"(N) : "memory");
#pragma unroll
    for (int i = 1; i < NA; ++i) asm volatile("" : "+v"(a[i]));
#pragma unroll
    for (int j = 0; j < NB; ++j) asm volatile("" : "+v"(b[j]));
}

// Second half of the epilogue.  The waves' tiles are staged in LDS ([WTM][SP] floats per
// wave); each lane handles CW consecutive columns (4, or 8 for bf16 output so that its
// store is still 16 bytes wide: stores run at a rate set by the bytes per lane).
template <int BM, int BN, int WGM, int WGN, int KW, int CW>
__device__ __forceinline__ bool dconv_epilogue_tail(const DconvParams &p, uint4 *smem_u4, int t, int lane, int kg, int wq,
                                                    int wm, int wn, int m0, int n0, int mt, int nt, int split, char *y)
{
    constexpr int NWG = WGM * WGN, NW = NWG * KW;
    constexpr int WTM = BM / WGM, WTN = BN / WGN;
    constexpr int SP = WTN + 4;                            // staging pitch in floats
    constexpr int V = CW / 4;                              // 16-byte pieces per lane per access
    constexpr int CPRW = WTN / CW;                         // lanes per staged row
    constexpr int RPI = 64 / CPRW;                         // rows per wave-wide access
    constexpr int NIT = WTM / RPI / KW;                    // wave-wide accesses per wave: its 1/KW of the wave tile's rows
    static_assert(NIT >= 1 && WTM % (RPI * KW) == 0, "the K groups share the rows of a wave tile evenly");
    const int cl = lane % CPRW, rl = lane / CPRW;          // this lane's column group and row inside an access
    const int n = n0 + wn * WTN + cl * CW;
    const bool n_ok = n < p.Nc;                            // Nc % CW == 0
    const int rrow0 = kg * (NIT * RPI) + rl;               // first row of this lane inside the wave tile
    const int mrow0 = m0 + wm * WTM + rrow0;
    const int tile = mt * p.tiles_n + nt;

    // The wave's share of the tile, summed over the K groups in group order.
    f32x4_t vs[NIT][V];
    {
        const float *src = (const float *)smem_u4 + wq * (WTM * SP) + rrow0 * SP + cl * CW;
#pragma unroll
        for (int it = 0; it < NIT; ++it)
#pragma unroll
            for (int v = 0; v < V; ++v) {
                const float4 f = *(const float4 *)(src + it * RPI * SP + v * 4);
                vs[it][v] = (f32x4_t){f.x, f.y, f.z, f.w};
            }
#pragma unroll
        for (int g = 1; g < KW; ++g)
#pragma unroll
            for (int it = 0; it < NIT; ++it)
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    const float4 f = *(const float4 *)(src + g * (NWG * WTM * SP) + it * RPI * SP + v * 4);
                    vs[it][v] += (f32x4_t){f.x, f.y, f.z, f.w};
                }
    }
    uint32_t offs[NIT];                                    // element offsets in a partial-sum plane ([M][Nc]) ...
    uint32_t yoffs[NIT];                                   // ... and in the output under its layout
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int m = mrow0 + it * RPI;
        const bool in = n_ok && m < p.M;
        offs[it] = in ? (uint32_t)(m * p.Nc + n) : kOutOfRange / 4u;
        yoffs[it] = in ? dconv_out_elem(p, m, n) : kOutOfRange / 4u;
    }

    if (p.splitk > 1) {
        // publish the partial tile; the last slice to arrive sums all slices in slice order
        const __amdgpu_buffer_rsrc_t pr = __builtin_amdgcn_make_buffer_rsrc(
            (void *)((char *)p.partial + (size_t)split * p.partial_bytes), 0, (int)p.partial_bytes, 0x00020000);
#pragma unroll
        for (int it = 0; it < NIT; ++it)
#pragma unroll
            for (int v = 0; v < V; ++v) {
                const u32x4_t w = __builtin_bit_cast(u32x4_t, vs[it][v]);
                __builtin_amdgcn_raw_buffer_store_b128(w, pr, (int)(offs[it] * 4u), v * 16, kAgentScope);
            }
        // Release half: the partial sums were stored with device (agent) scope, i.e. written
        // through to memory all XCDs share; once the stores are acknowledged they are
        // visible to device-scope loads anywhere (a full device-scope fence would write
        // back the whole L2 and costs tens of microseconds here).
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        uint32_t *flag = (uint32_t *)smem_u4 + NW * (WTM * SP);
        if (t == 0) {
            const uint32_t old = __hip_atomic_fetch_add(p.counters + tile, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            *flag = old == (uint32_t)(p.splitk - 1);
            if (*flag)                             // ready for the next launch
                __hip_atomic_store(p.counters + tile, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        if (*flag == 0) return false;                   // another workgroup finishes this tile
        // acquire half: the loads below have device scope and so do not hit stale cache lines

        // Sum of the slices in slice order.  All loads of a slice are issued before any of
        // them is consumed (one dependent load per access would cost a device-scope memory
        // round trip each).  Whole-vector adds: element-wise float views of a loaded
        // vector are miscompiled into a single-dword load by this toolchain.
#pragma unroll
        for (int it = 0; it < NIT; ++it)
#pragma unroll
            for (int v = 0; v < V; ++v) vs[it][v] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
        // G slices (up to 16 loads) are in flight at a time: a device-scope load takes over a
        // microsecond, so slices fetched one after the other would cost that much each.  (Not
        // more: these registers, not the main loop's, would then set the kernel's register
        // count and with it the waves a SIMD can hold.)
        constexpr int G = NIT * V >= 16 ? 1 : 16 / (NIT * V);
        for (int sl0 = 0; sl0 < p.splitk; sl0 += G) {
            u32x4_t w4[G][NIT][V];
#pragma unroll
            for (int g = 0; g < G; ++g) {
                // slices past the last one read with a zero-sized descriptor: all zeros
                const bool live = sl0 + g < p.splitk;
                const __amdgpu_buffer_rsrc_t sr = __builtin_amdgcn_make_buffer_rsrc(
                    (void *)((char *)p.partial + (size_t)(live ? sl0 + g : 0) * p.partial_bytes), 0,
                    live ? (int)p.partial_bytes : 0, 0x00020000);
#pragma unroll
                for (int it = 0; it < NIT; ++it)
#pragma unroll
                    for (int v = 0; v < V; ++v)
                        w4[g][it][v] = __builtin_amdgcn_raw_buffer_load_b128(sr, (int)(offs[it] * 4u), v * 16, kAgentScope);
            }
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int it = 0; it < NIT; ++it)
#pragma unroll
                    for (int v = 0; v < V; ++v) vs[it][v] += __builtin_bit_cast(f32x4_t, w4[g][it][v]);
        }
    }

    const __amdgpu_buffer_rsrc_t yr = __builtin_amdgcn_make_buffer_rsrc(y, 0, (int)p.y_bytes, 0x00020000);
    const float relu_floor = (p.flags & ALT_EPI_RELU) ? 0.f : -INFINITY;
    const bool out_bf16 = p.flags & kDconvOutBf16;
    float bv[CW];
#pragma unroll
    for (int q = 0; q < CW; ++q) bv[q] = 0.f;
    if (n_ok && (p.flags & ALT_EPI_BIAS)) {
#pragma unroll
        for (int v = 0; v < V; ++v) {
            const float4 b4 = *(const float4 *)(p.bias + n + v * 4);
            bv[v * 4 + 0] = b4.x; bv[v * 4 + 1] = b4.y; bv[v * 4 + 2] = b4.z; bv[v * 4 + 3] = b4.w;
        }
    }
    const __amdgpu_buffer_rsrc_t ar = __builtin_amdgcn_make_buffer_rsrc((void *)p.addend, 0, (int)p.y_bytes, 0x00020000);
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const bool ok = yoffs[it] != kOutOfRange / 4u;
        float ad[CW];                                      // the fused sum's other operand (zeros without one)
#pragma unroll
        for (int q = 0; q < CW; ++q) ad[q] = 0.f;
        if (!p.addend) {
        } else if (CW == 8 || out_bf16) {
            // bf16: element 2j is the low half of dword j, element 2j+1 the high half (whole-vector
            // shifts and masks; an out-of-range offset reads zeros)
            u32x4_t av = {0u, 0u, 0u, 0u};
            if constexpr (CW == 8) av = __builtin_amdgcn_raw_buffer_load_b128(ar, (int)(ok ? yoffs[it] * 2u : kOutOfRange), 0, 0);
            else {
                typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
                const u32x2_t a2 = __builtin_amdgcn_raw_buffer_load_b64(ar, (int)(ok ? yoffs[it] * 2u : kOutOfRange), 0, 0);
                av = __builtin_shufflevector(a2, a2, 0, 1, 0, 1);
            }
            const f32x4_t lo = __builtin_bit_cast(f32x4_t, av << 16), hi = __builtin_bit_cast(f32x4_t, av & 0xffff0000u);
#pragma unroll
            for (int q = 0; q < CW / 2; ++q) { ad[2 * q] = lo[q]; ad[2 * q + 1] = hi[q]; }
        } else {
            const f32x4_t a4 = __builtin_bit_cast(f32x4_t, __builtin_amdgcn_raw_buffer_load_b128(ar, (int)(ok ? yoffs[it] * 4u : kOutOfRange), 0, 0));
            const f32x4_t z = a4 + (f32x4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int q = 0; q < 4; ++q) ad[q] = z[q];
        }
        float o[CW];
#pragma unroll
        for (int q = 0; q < CW; ++q) o[q] = fmaxf(vs[it][q / 4][q % 4] + bv[q] + ad[q], relu_floor);
        if (CW == 8 || out_bf16) {                         // (eight columns per lane are only used for bf16 output)
            uint32_t w[CW / 2];
#pragma unroll
            for (int q = 0; q < CW / 2; ++q)
                w[q] = f32x2_to_bf16x2(o[2 * q], o[2 * q + 1]);
            if constexpr (CW == 8) {
                u32x4_t ov = {w[0], w[1], w[2], w[3]};
                __builtin_amdgcn_raw_buffer_store_b128(ov, yr, (int)(ok ? yoffs[it] * 2u : kOutOfRange), 0, kWriteThrough);
            } else {
                typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
                u32x2_t ov = {w[0], w[1]};
                __builtin_amdgcn_raw_buffer_store_b64(ov, yr, (int)(ok ? yoffs[it] * 2u : kOutOfRange), 0, kWriteThrough);
            }
        } else {
            u32x4_t ov = {__builtin_bit_cast(uint32_t, o[0]), __builtin_bit_cast(uint32_t, o[1]),
                          __builtin_bit_cast(uint32_t, o[2]), __builtin_bit_cast(uint32_t, o[3])};
            __builtin_amdgcn_raw_buffer_store_b128(ov, yr, (int)(ok ? yoffs[it] * 4u : kOutOfRange), 0, kWriteThrough);
        }
    }
    return true;
}

// The end of a tile kernel: every wave holds a WTM x WTN accumulator tile (wave (wm, wn) of
// K group kg; wq = its index inside the group); the K groups are summed, then either
// the finished tile is stored (bias, ReLU, fp32 or bf16) or, with split-K, the partial
// tile is published and the last slice to arrive sums all slices.  y = the output of this
// batch entry.  Uses the whole LDS allocation from its start (callers are done with it: the
// function opens with a barrier).  Returns false in workgroups that leave the tile to
// another slice's workgroup.
template <int BM, int BN, int WGM, int WGN, int KW>
__device__ __forceinline__ bool dconv_epilogue(const DconvParams &p, floatx16_t (&acc)[BM / WGM / 32][BN / WGN / 32],
                                               uint4 *smem_u4, int t, int lane, int wave, int kg, int wq, int wm, int wn,
                                               int m0, int n0, int mt, int nt, int split, char *y)
{
    constexpr int WTM = BM / WGM, WTN = BN / WGN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    // ---- the wave's tile goes through LDS to row-major order -----------------------------------------
    // The MFMAs take the weights as their first operand, so accumulator register e of lane l is
    // element (pixel l%32, channel 8*(e/4) + 4*(l/32) + e%4) of a 32x32 tile: four consecutive
    // channels of one pixel per register quad, but consecutive lanes on different pixels, and
    // stores whose lanes are 2*Nc bytes apart run at a fraction of the rate of contiguous
    // 16-byte ones.  So each wave transposes through a private LDS region ([WTM][WTN + 4]
    // floats, written 16 bytes at a time; the pitch keeps those writes and the 16-byte reads
    // of eight columns per lane conflict-free) and then handles four or eight consecutive
    // channels per lane, consecutive lanes side by side.
    constexpr int SP = WTN + 4;                            // staging pitch in floats
    __syncthreads();                                       // every wave is done with the stages and the patch
    float *stg = (float *)smem_u4 + wave * (WTM * SP);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                *(float4 *)(stg + (i * 32 + (lane & 31)) * SP + j * 32 + 8 * q + 4 * (lane >> 5)) =
                    make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
    // (with one K group a wave reads back only what it wrote itself; the compiler orders these LDS accesses)
    if constexpr (KW > 1) __syncthreads();
    bool mine;
    constexpr bool kWideFits = WTM % ((64 / (WTN / 8)) * KW) == 0;     // eight columns per lane divide the tile evenly
    if (kWideFits && (p.flags & kDconvOutBf16) && p.Nc % 8 == 0) {
        if constexpr (kWideFits)
            mine = dconv_epilogue_tail<BM, BN, WGM, WGN, KW, 8>(p, smem_u4, t, lane, kg, wq, wm, wn, m0, n0, mt, nt, split, y);
    } else {
        mine = dconv_epilogue_tail<BM, BN, WGM, WGN, KW, 4>(p, smem_u4, t, lane, kg, wq, wm, wn, m0, n0, mt, nt, split, y);
    }
    return mine;
}

// Whether a tile kernel's output staging (every wave's whole tile at once) exceeds LDS; such
// kernels stage and store their tiles 32 rows at a time instead (dconv_epilogue_banded).
template <int BM, int BN, int WGN, int KW>
constexpr bool kBandedEpilogue = (size_t)KW * BM * (BN + 8 * WGN) * 4 + 16 > 160 * 1024;

// The end of a tile kernel whose wave tiles are too large to stage whole (128 x 128 per wave):
// each wave takes its tile through a private LDS region one band of 32 rows at a time, then
// stores the band with 16-byte accesses (four fp32 or eight bf16 columns per lane) exactly as
// dconv_epilogue_tail does.  One K group and no split-K (the host does not offer these
// kernels with either); a wave only reads back what it wrote, so after the opening
// barrier (all waves done with the operand stages) no further one is needed.
template <int BM, int BN, int WGM, int WGN>
__device__ __forceinline__ void dconv_epilogue_banded(const DconvParams &p, floatx16_t (&acc)[BM / WGM / 32][BN / WGN / 32],
                                                      uint4 *smem_u4, int lane, int wave, int wm, int wn, int m0, int n0,
                                                      char *y)
{
    constexpr int WTM = BM / WGM, WTN = BN / WGN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int SP = WTN + 4;                            // staging pitch in floats
    __syncthreads();
    float *stg = (float *)smem_u4 + wave * (32 * SP);
    const __amdgpu_buffer_rsrc_t yr = __builtin_amdgcn_make_buffer_rsrc(y, 0, (int)p.y_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t ar = __builtin_amdgcn_make_buffer_rsrc((void *)p.addend, 0, (int)p.y_bytes, 0x00020000);
    const float relu_floor = (p.flags & ALT_EPI_RELU) ? 0.f : -INFINITY;
    const bool wide = (p.flags & kDconvOutBf16) && p.Nc % 8 == 0;      // eight bf16 columns per lane
    auto band = [&](auto cw, int i) {
        constexpr int CW = decltype(cw)::value;
        constexpr int V = CW / 4, CPRW = WTN / CW, RPI = 64 / CPRW, NIT = 32 / RPI;
        const int cl = lane % CPRW, rl = lane / CPRW;
        const int n = n0 + wn * WTN + cl * CW;
        const bool n_ok = n < p.Nc;
        float bv[CW];
#pragma unroll
        for (int q = 0; q < CW; ++q) bv[q] = 0.f;
        if (n_ok && (p.flags & ALT_EPI_BIAS)) {
#pragma unroll
            for (int v = 0; v < V; ++v) {
                const float4 b4 = *(const float4 *)(p.bias + n + v * 4);
                bv[v * 4 + 0] = b4.x; bv[v * 4 + 1] = b4.y; bv[v * 4 + 2] = b4.z; bv[v * 4 + 3] = b4.w;
            }
        }
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int row = it * RPI + rl;
            const int m = m0 + wm * WTM + i * 32 + row;
            const bool ok = n_ok && m < p.M;
            float o[CW];
#pragma unroll
            for (int v = 0; v < V; ++v) {
                const float4 f = *(const float4 *)(stg + row * SP + cl * CW + v * 4);
                o[v * 4 + 0] = f.x; o[v * 4 + 1] = f.y; o[v * 4 + 2] = f.z; o[v * 4 + 3] = f.w;
            }
            const uint32_t el = ok ? dconv_out_elem(p, m, n) : 0u;
            float ad[CW];                                  // the fused sum's other operand: y's layout and element type
#pragma unroll
            for (int q = 0; q < CW; ++q) ad[q] = 0.f;
            if (!p.addend) {
            } else if (CW == 8 || (p.flags & kDconvOutBf16)) {
                u32x4_t av = {0u, 0u, 0u, 0u};
                if constexpr (CW == 8) av = __builtin_amdgcn_raw_buffer_load_b128(ar, (int)(ok ? el * 2u : kOutOfRange), 0, 0);
                else {
                    typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
                    const u32x2_t a2 = __builtin_amdgcn_raw_buffer_load_b64(ar, (int)(ok ? el * 2u : kOutOfRange), 0, 0);
                    av = __builtin_shufflevector(a2, a2, 0, 1, 0, 1);
                }
                const f32x4_t lo = __builtin_bit_cast(f32x4_t, av << 16), hi = __builtin_bit_cast(f32x4_t, av & 0xffff0000u);
#pragma unroll
                for (int q = 0; q < CW / 2; ++q) { ad[2 * q] = lo[q]; ad[2 * q + 1] = hi[q]; }
            } else {
                const f32x4_t a4 = __builtin_bit_cast(f32x4_t, __builtin_amdgcn_raw_buffer_load_b128(ar, (int)(ok ? el * 4u : kOutOfRange), 0, 0));
                const f32x4_t z = a4 + (f32x4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int q = 0; q < 4; ++q) ad[q] = z[q];
            }
#pragma unroll
            for (int q = 0; q < CW; ++q) o[q] = fmaxf(o[q] + bv[q] + ad[q], relu_floor);
            if (CW == 8 || (p.flags & kDconvOutBf16)) {
                uint32_t w[CW / 2];
#pragma unroll
                for (int q = 0; q < CW / 2; ++q) w[q] = f32x2_to_bf16x2(o[2 * q], o[2 * q + 1]);
                if constexpr (CW == 8) {
                    u32x4_t ov = {w[0], w[1], w[2], w[3]};
                    __builtin_amdgcn_raw_buffer_store_b128(ov, yr, (int)(ok ? el * 2u : kOutOfRange), 0, kWriteThrough);
                } else {
                    typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
                    u32x2_t ov = {w[0], w[1]};
                    __builtin_amdgcn_raw_buffer_store_b64(ov, yr, (int)(ok ? el * 2u : kOutOfRange), 0, kWriteThrough);
                }
            } else {
                u32x4_t ov = {__builtin_bit_cast(uint32_t, o[0]), __builtin_bit_cast(uint32_t, o[1]),
                              __builtin_bit_cast(uint32_t, o[2]), __builtin_bit_cast(uint32_t, o[3])};
                __builtin_amdgcn_raw_buffer_store_b128(ov, yr, (int)(ok ? el * 4u : kOutOfRange), 0, kWriteThrough);
            }
        }
    };
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        // band i of the wave's tile to row-major order (same element mapping as in dconv_epilogue)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                *(float4 *)(stg + (lane & 31) * SP + j * 32 + 8 * q + 4 * (lane >> 5)) =
                    make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
        if (wide) band(std::integral_constant<int, 8>{}, i);
        else band(std::integral_constant<int, 4>{}, i);
    }
}

// Waves per SIMD the register allocation must leave room for (a SIMD has 512 registers per
// lane, accumulators included).  Without a bound the allocator spreads the accumulators
// over the second register file and takes what it likes: one wave per SIMD for 64x64 wave
// tiles.  Workgroups of up to four waves are held to three waves per SIMD when their
// accumulators are 32 registers and to two when they are 64, which the main loops fit
// without spilling.
#ifndef ALT_DCONV_MIN_WAVES
#define ALT_DCONV_MIN_WAVES(acc_regs, nw) ((nw) <= 4 ? ((acc_regs) <= 32 ? 3 : (acc_regs) <= 64 ? 2 : 1) : 1)
#endif

// The workgroup has KW groups of WGM x WGN waves.  Each group computes the whole BM x BN
// tile over its own 1/KW of the slice's channels (all taps), with a weight ring of its
// own; the groups' tiles are summed through LDS at the end.  This puts two waves on every
// SIMD of a CU even when the tile only has room for a few large wave tiles, which is
// what hides the operand-read latency (large wave tiles keep the LDS traffic per MFMA low).
//
// KR > 0: the filter is KR x KR and a group's channels are NCC chunks of BK, both known at
// compile time: all K steps are unrolled into straight-line code (no loop-carried
// register shuffling, every operand address precomputed).  KR = 0: any filter size and
// slice width, taps and chunks walked at run time.
template <int BM, int BN, int WGM, int WGN, int KW, int NS, int BK, int KR, int NCC>
__global__ __launch_bounds__(64 * WGM * WGN * KW, ALT_DCONV_MIN_WAVES((BM / WGM) * (BN / WGN) / 64, WGM * WGN * KW))
void dconv_kernel(const DconvParams p)
{
    constexpr int NWG = WGM * WGN, NW = NWG * KW;          // waves per group, per workgroup
    constexpr int WTM = BM / WGM, WTN = BN / WGN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int NKC = BK / 16;
    constexpr int CPR = BK / 8;                            // 16-byte chunks per weight row of a stage
    constexpr int RP = 256 / (BK * 2);                     // weight rows per 256 bytes of LDS
    constexpr int B_STAGE = BN * BK * 2;                   // bytes of one weight stage: [BN][CPR chunks of 16 B]
    constexpr int B_RING = NS * B_STAGE;                   // one group's stages
    constexpr int NLB = B_STAGE / 1024 / NWG;              // wave-loads per wave per stage
    static_assert(BK == 64 || BK == 32, "K step");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0 && TM >= 1 && TN >= 1, "wave tile");
    static_assert(B_STAGE % (1024 * NWG) == 0 && NLB >= 1, "a weight stage is a whole number of wave-loads per wave");
    static_assert(NS >= 3 && (NS - 1) * NLB < 48, "pipeline depth");
    static_assert(TM + TN <= 15, "fragment reads in flight against the lgkmcnt range");

    extern __shared__ uint4 smem_u4[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)smem_u4;    // the groups' weight rings first, then the patch
    const uint32_t patch0 = lds0 + KW * B_RING;

    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int kg = wave / NWG, wq = wave % NWG;            // K group, wave inside the group
    const int wm = wq / WGN, wn = wq % WGN;

    // workgroup -> (m tile, n tile, channel slice)
    int mt, nt, split;
    {
        // consecutive logical ids share an XCD
        const int ntot = p.tiles_m * p.tiles_n * p.splitk;
        const int logical = igemm_logical_tile(ntot);
        const int rest = (int)div32((uint32_t)logical, p.d_tm);
        mt = logical - rest * p.tiles_m;
        split = (int)div32((uint32_t)rest, p.d_tn);
        nt = rest - split * p.tiles_n;
    }
    const int m0 = mt * BM, n0 = nt * BN;

    const i32x4_t x_rsrc = make_rsrc(p.x, p.x_bytes);
    const i32x4_t w_rsrc = make_rsrc(p.w, p.w_bytes);

    // ---- the patch: input pixels [m0 - halo, m0 + BM + halo), Cs channels of this slice --------
    // A patch pixel takes Cs * 2 + 16 bytes of LDS: its chunks in order, then one unused
    // 16-byte slot.  The odd pitch spreads 16 consecutive pixels over all banks (so the
    // operand reads of an MFMA row tile do not collide) while a pixel's address stays
    // affine in its index: a filter tap is then one add per row tile and the chunk inside
    // the pixel an instruction offset, with no per-read address arithmetic.
    // Output pixel m of image img at (oh, ow) sits over input pixel img*H*W + oh*stride*W + ow*stride
    // (its tap (pad_h, pad_w)); the tile's patch runs from the first row's to the last row's.
    const int halo = p.pad_h * p.W + p.pad_w;                                  // pixels before the first tap's anchor
    const int halo_hi = ((p.R - 1) * p.dil - p.pad_h) * p.W + ((p.S - 1) * p.dil - p.pad_w);   // and behind the last one's
    const int ohw = p.OH * p.OW;
    auto anchor = [&](int m) {
        const int img = (int)div32((uint32_t)m, p.d_hw), rem = m - img * ohw;
        const int oh = (int)div32((uint32_t)rem, p.d_w), ow = rem - oh * p.OW;
        return img * (p.H * p.W) + (oh * p.W + ow) * p.stride;
    };
    const int a0 = anchor(m0);
    const int np = anchor(min(m0 + BM, p.M) - 1) - a0 + 1 + halo + halo_hi;
    const int spp = (1 << p.log2_cpp) + 1;                 // 16-byte slots per patch pixel
    const int pitch_b = spp * 16;
    const int nwl = (np * spp + 63) >> 6;                  // wave-loads (the region is padded to whole ones)
    const int pz = (int)div32((uint32_t)((nwl << 6) + spp - 1), p.d_slots);   // the first pixel row behind the patch
    // Behind the patch, at a multiple of 256 bytes (one pass over all banks), sits the zero area that taps
    // outside the image read: 256 bytes and a pixel's channels of zeros.  A lane whose tap is outside reads it at
    // the same offset modulo 256 as the pixel it would have read, i.e. from the same banks, so the lanes of an
    // operand read stay on distinct banks as they are without padding (one zero pixel shared by all such lanes
    // sits on the banks of some other lane's pixel: measured 170 against 245 bytes per clock with eight lanes
    // on it).
    const uint32_t zero0 = (patch0 + (uint32_t)(pz * pitch_b) + 255u) & ~255u;
    {
        const int g0 = a0 - halo;
        auto load_one = [&](int j) {
            const int slot = j * 64 + lane;
            const int px = (int)div32((uint32_t)slot, p.d_slots), c = slot - px * spp;
            const int g = g0 + px;
            const bool ok = c < spp - 1 && px < np && (unsigned)g < (unsigned)p.in_px;
            const uint32_t voff = ok ? dconv_in_elem(p, g, split * p.Cs + c * 8) * 2u : kOutOfRange;
            dma_load16(x_rsrc, voff, patch0 + j * 1024);
        };
        int j = wave;
        for (; j + 3 * NW < nwl; j += 4 * NW) {            // four at a time: independent address chains
            load_one(j); load_one(j + NW); load_one(j + 2 * NW); load_one(j + 3 * NW);
        }
        for (; j < nwl; j += NW) load_one(j);
        for (int i = t; i < 16 + (p.Cs >> 3) + 2; i += 64 * NW)
            *(uint4 *)((char *)smem_u4 + (zero0 - lds0) + i * 16) = make_uint4(0, 0, 0, 0);
    }

    // ---- weights: slot s = (i*NWG + wq)*64 + lane of a stage holds chunk (s % CPR) ^ swz(row) of row s / CPR
    // (rows that share LDS banks, RP apart, get different chunk orders)
    const int ncc = NCC > 0 ? NCC : p.ncc;                 // BK-channel chunks of the group
    const int csg = ncc * BK;                              // channels of the group
    const uint32_t kg_off = (uint32_t)(kg * csg) * 2u;     // the group's first channel inside a patch pixel, bytes
    uint32_t b_voff[NLB];
    const int rsc = p.R * p.S * p.C;
#pragma unroll
    for (int i = 0; i < NLB; ++i) {
        const int s = (i * NWG + wq) * 64 + lane;
        const int row = s / CPR, c = (s % CPR) ^ ((row / RP) & (CPR - 1));
        const int n = n0 + row;
        b_voff[i] = n < p.Nc ? (uint32_t)(n * rsc + split * p.Cs + kg * csg + c * 8) * 2u : kOutOfRange;
    }
    const uint32_t ring0 = lds0 + kg * B_RING;
    const uint32_t ldsB = ring0 + wq * 1024;
    const int nsteps = KR > 0 ? KR * KR * NCC : p.R * p.S * p.ncc;
    // load cursor: byte offset of K step `lstep` inside a weight row, (tap, chunk) walked chunk fastest
    int lstep = 0, lcc = 0, lstage = 0;
    uint32_t lsoff = 0;
    auto issue_b = [&]() {
#pragma unroll
        for (int i = 0; i < NLB; ++i) dma_load16_s(w_rsrc, b_voff[i], lsoff, ldsB + lstage * B_STAGE + i * (NWG * 1024));
        ++lstep;
        lstage = lstage + 1 == NS ? 0 : lstage + 1;
        // next K step's offset inside a weight row; past the last step it stays where it is
        const bool more = lstep < nsteps;
        const bool wrap = lcc + 1 == ncc;
        lsoff += more ? (uint32_t)(BK * 2) + (wrap ? (uint32_t)(p.C - csg) * 2u : 0u) : 0u;
        lcc = more ? (wrap ? 0 : lcc + 1) : lcc;
    };
    // NS - 1 stages in flight from here on (past the last step: repeats of it, never read)
#pragma unroll
    for (int s = 0; s < NS - 1; ++s) issue_b();

    // ---- per-lane rows of the MFMA tiles ---------------------------------------------------------
    int32_t row_px[TM], row_oh[TM], row_ow[TM];           // patch pixel under tap (pad_h, pad_w); its input row and column
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int r = wm * WTM + i * 32 + (lane & 31);
        const int m = m0 + r;
        if (m < p.M) {
            const int img = (int)div32((uint32_t)m, p.d_hw), rem = m - img * ohw;
            const int oh = (int)div32((uint32_t)rem, p.d_w), ow = rem - oh * p.OW;
            row_oh[i] = oh * p.stride;
            row_ow[i] = ow * p.stride;
            row_px[i] = img * (p.H * p.W) + row_oh[i] * p.W + row_ow[i] - a0 + halo;
        } else {
            row_oh[i] = -(1 << 20);
            row_ow[i] = -(1 << 20);
            row_px[i] = 0;
        }
    }
    // weight operand addresses inside stage 0 (LDS byte addresses), per n tile and k chunk
    uint32_t b_rd[TN][NKC];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int r = wn * WTN + j * 32 + (lane & 31);
        const uint32_t swz = ((r / RP) & (CPR - 1)) * 16;
#pragma unroll
        for (int kc = 0; kc < NKC; ++kc) b_rd[j][kc] = ring0 + r * (BK * 2) + ((kc * 32 + (lane >> 5) * 16) ^ swz);
    }

    floatx16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const uint32_t khalf = (lane >> 5) * 16 + kg_off;      // this lane's first byte inside a patch pixel

    // Where the MFMA row tiles of one K step read: the patch row under the step's tap (rows
    // whose tap falls outside the image use the zero row) at this lane's channel half,
    // the channel offset inside the pixel and the weight stage.
    struct StepAddr {
        uint32_t a_row[TM], c_off, st_off;
    };
    auto set_tap = [&](StepAddr &sa, int r, int s) {
        const int dr = r * p.dil - p.pad_h, ds = s * p.dil - p.pad_w;          // the tap's offset from the anchor
        const int shift = dr * p.W + ds;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const bool ok = (unsigned)(row_oh[i] + dr) < (unsigned)p.H && (unsigned)(row_ow[i] + ds) < (unsigned)p.W;
            const uint32_t at = patch0 + (uint32_t)((row_px[i] + shift) * pitch_b);
            sa.a_row[i] = (ok ? at : zero0 + (at & 255u)) + khalf;
        }
    };
    // Operand reads run D k-chunks ahead of the MFMAs that use them, each k-chunk in a
    // register buffer of its own (kc % NKC): with one wave per SIMD the LDS latency
    // under load (several hundred cycles) is only covered by that many MFMA groups.
    constexpr int D0 = (TM + TN) * 3 <= 15 ? 3 : (TM + TN) * 2 <= 15 ? 2 : 1;
    constexpr int D = D0 < NKC ? D0 : NKC;
    constexpr int NBUF = 4;                                // k chunk g (counted over all steps) uses buffer g % NBUF
    static_assert(D <= NKC && D < NBUF && NBUF % NKC == 0, "look-ahead stays within the next step");
    u32x4_t af[NBUF][TM], bf[NBUF][TN];
    auto read_frags = [&](int kc, const StepAddr &sa) {
#pragma unroll
        for (int i = 0; i < TM; ++i) lds_read16_async(af[kc][i], sa.a_row[i] + (sa.c_off + kc * 32));
#pragma unroll
        for (int j = 0; j < TN; ++j) lds_read16_async(bf[kc][j], b_rd[j][kc] + sa.st_off);
    };

    // ---- main loop -------------------------------------------------------------------------------------
    // K steps walk the taps, 64-channel chunks of the slice innermost.  Step t's weights
    // sit in stage t % NS.  At the barrier that opens step t every wave has its share of
    // stage t+1 landed, so after it stages t and t+1 are complete for everybody and the
    // look-ahead reads may run into step t+1 before the next barrier.  The same barrier
    // says stage t-1 is consumed, and its refill (step t+NS-1) is issued after it.
    //
    // A wave issues in order, so whatever sits between two MFMA groups delays the
    // second one unless it can run in the first one's shadow.  The body of a step is
    // therefore one straight basic block: the bookkeeping of the next step (tap, row
    // addresses) uses selects, not branches, and stands after the first MFMA group; past
    // the last step the weight refills and look-ahead reads repeat the last step's
    // addresses (loaded, never used) instead of being skipped.
    if constexpr (KR > 0) {
        // Patch rows of every tap, computed while the patch is still in flight; the channel
        // offset of a k chunk and the weight stage are instruction offsets.
        constexpr int RS = KR * KR, NSTEPS = RS * NCC;
        uint32_t t_row[RS][TM];
#pragma unroll
        for (int tap = 0; tap < RS; ++tap) {
            StepAddr sa;
            set_tap(sa, tap / KR, tap % KR);
#pragma unroll
            for (int i = 0; i < TM; ++i) t_row[tap][i] = sa.a_row[i];
        }
        wait_vmcnt<(NS - 2) * NLB>();                      // the patch and stage 0
        lds_barrier();
        // reads of k chunk g (counted over all steps); past the last step they repeat it (never used)
        auto read_one = [&](auto gc, auto rc) {            // operand read r of chunk g: the TM patch rows, then the TN weight rows
            constexpr int g = decltype(gc)::value, r = decltype(rc)::value;
            constexpr int step = g / NKC < NSTEPS ? g / NKC : NSTEPS - 1, kc = g % NKC, buf = g % NBUF;
            constexpr int tap = step / NCC, cc = step % NCC, st = step % NS;
            if constexpr (r < TM) lds_read16_async_at<cc * (BK * 2) + kc * 32>(af[buf][r], t_row[tap][r]);
            else lds_read16_async_at<st * B_STAGE>(bf[buf][r - TM], b_rd[r - TM][kc]);
        };
        auto reads = [&](auto gc) {
            static_for<TM + TN>([&](auto rc) { read_one(gc, rc); });
        };
        // Large wave tiles run a hand-pinned instruction order (see the streaming kernel, dstream.h):
        // after each row of TN MFMAs a few of the next chunk's operand reads and one weight load.
        constexpr bool kPinned = KW == 1 && TM * TN >= 8 && TM >= 2 && NLB <= NKC * TM;
        constexpr int DP = kPinned ? 1 : D;
        static_for<DP>([&](auto gc) { reads(gc); });
        static_for<NSTEPS>([&](auto sc) {
            constexpr int step = decltype(sc)::value;
            wait_vmcnt<(NS - 3) * NLB>();                  // stage step+1 has landed (this wave's share)
            if constexpr (NWG > 1) asm volatile("s_barrier" ::: "memory");   // (a one-wave group loads its ring alone)
            if constexpr (!kPinned) {
                issue_b();
                static_for<NKC>([&](auto kcc) {
                    constexpr int kc = decltype(kcc)::value;
                    constexpr int buf = (step * NKC + kc) % NBUF;
                    reads(std::integral_constant<int, step * NKC + kc + D>{});
                    lds_wait<D * (TM + TN)>(af[buf], bf[buf]);
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int j = 0; j < TN; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, bf[buf][j]),
                                                                                __builtin_bit_cast(bf16x8_t, af[buf][i]),
                                                                                acc[i][j], 0, 0, 0);
                });
            } else {
                static_for<NKC>([&](auto kcc) {
                    constexpr int kc = decltype(kcc)::value, g = step * NKC + kc, buf = g % NBUF;
                    constexpr int RPS = (TM + TN + TM - 2) / (TM - 1);         // reads per row slot, rows 0 .. TM - 2
                    lds_wait<0>(af[buf], bf[buf]);
                    static_for<TM>([&](auto IR) {
                        constexpr int i = decltype(IR)::value;
#pragma unroll
                        for (int j = 0; j < TN; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, bf[buf][j]),
                                                                                __builtin_bit_cast(bf16x8_t, af[buf][i]),
                                                                                acc[i][j], 0, 0, 0);
                        __builtin_amdgcn_sched_barrier(0);
                        static_for<RPS>([&](auto RR) {
                            constexpr int r = i * RPS + decltype(RR)::value;
                            if constexpr (r < TM + TN) read_one(std::integral_constant<int, g + 1>{}, std::integral_constant<int, r>{});
                        });
                        if constexpr (kc * TM + i < NLB)
                            dma_load16_s(w_rsrc, b_voff[kc * TM + i], lsoff, ldsB + lstage * B_STAGE + (kc * TM + i) * (NWG * 1024));
                        __builtin_amdgcn_sched_barrier(0);
                    });
                });
                // the cursor moves on as in issue_b
                ++lstep;
                lstage = lstage + 1 == NS ? 0 : lstage + 1;
                const bool more = lstep < nsteps;
                const bool wrap = lcc + 1 == ncc;
                lsoff += more ? (uint32_t)(BK * 2) + (wrap ? (uint32_t)(p.C - csg) * 2u : 0u) : 0u;
                lcc = more ? (wrap ? 0 : lcc + 1) : lcc;
            }
        });
    } else {
        static_assert(KR > 0 || NKC == NBUF, "the run-time path takes 64-channel steps");
        int r = 0, s = 0, cc = 0;
        StepAddr cur, nxt;
        set_tap(cur, 0, 0);
        cur.c_off = 0;
        cur.st_off = 0;
        wait_vmcnt<(NS - 2) * NLB>();                          // the patch and stage 0
        lds_barrier();
    #pragma unroll
        for (int kc = 0; kc < D; ++kc) read_frags(kc, cur);
        for (int step = 0; step < nsteps; ++step) {
            wait_vmcnt<(NS - 3) * NLB>();                      // stage step+1 has landed (this wave's share)
            if constexpr (NWG > 1) asm volatile("s_barrier" ::: "memory");
            issue_b();
    #pragma unroll
            for (int kc = 0; kc < NKC; ++kc) {
                if (kc + D < NKC) read_frags(kc + D, cur);
                else read_frags(kc + D - NKC, nxt);
                lds_wait<D * (TM + TN)>(af[kc], bf[kc]);
    #pragma unroll
                for (int i = 0; i < TM; ++i)
    #pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, bf[kc][j]),
                                                                            __builtin_bit_cast(bf16x8_t, af[kc][i]),
                                                                            acc[i][j], 0, 0, 0);
                if (kc == 0) {
                    // where step + 1 reads (after the last step: where this one does)
                    const bool more = step + 1 < nsteps;
                    const bool wrap_c = cc + 1 == ncc;
                    const bool wrap_s = wrap_c && s + 1 == p.S;
                    cc = more ? (wrap_c ? 0 : cc + 1) : cc;
                    s = more && wrap_c ? (wrap_s ? 0 : s + 1) : s;
                    r = more && wrap_s ? r + 1 : r;
                    set_tap(nxt, r, s);
                    nxt.c_off = (uint32_t)cc * (BK * 2);
                    const uint32_t st1 = cur.st_off + B_STAGE == NS * B_STAGE ? 0 : cur.st_off + B_STAGE;
                    nxt.st_off = more ? st1 : cur.st_off;
                }
            }
            cur = nxt;
        }
    }
    wait_vmcnt<0>();                                       // the refills past the last step
    // The look-ahead reads past the last step are never used, but they still land in
    // their registers some hundred cycles after they were issued: the registers must
    // stay reserved until then, so they are tied to a wait here like any other read.
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int kc = 0; kc < NBUF; ++kc) {
#pragma unroll
        for (int i = 0; i < TM; ++i) asm volatile("" : "+v"(af[kc][i]));
#pragma unroll
        for (int j = 0; j < TN; ++j) asm volatile("" : "+v"(bf[kc][j]));
    }

    dconv_epilogue<BM, BN, WGM, WGN, KW>(p, acc, smem_u4, t, lane, wave, kg, wq, wm, wn, m0, n0, mt, nt, split, (char *)p.y);
}

// Pixels of the largest patch over the tiles of BM output pixels: the span of input pixels
// under a tile's first and last output pixel (found tile by tile: it depends on where rows and
// images end inside the tile) plus the taps' reach before and behind.
inline size_t dconv_patch_pixels(int BM, int64_t M, int H, int W, int OH, int OW, int R, int S, int pad_h, int pad_w,
                                 int stride, int dil)
{
    auto anchor = [&](int64_t m) {
        const int64_t img = m / ((int64_t)OH * OW), rem = m - img * OH * OW, oh = rem / OW, ow = rem - oh * OW;
        return img * H * W + (oh * W + ow) * stride;
    };
    int64_t span = 1;
    if (stride == 1 && OH == H && OW == W) span = BM;      // output and input indices coincide
    else
        for (int64_t m0 = 0; m0 < M; m0 += BM) {
            const int64_t m1 = (m0 + BM < M ? m0 + BM : M) - 1;
            const int64_t d = anchor(m1) - anchor(m0) + 1;
            if (d > span) span = d;
        }
    return (size_t)span + (size_t)pad_h * W + pad_w + (size_t)((R - 1) * dil - pad_h) * W + ((S - 1) * dil - pad_w);
}

// LDS bytes of one workgroup: the K groups' weight rings, the patch rounded up to
// whole wave-loads, the zero area.
// np = the largest patch of any tile, in pixels (dconv_patch_pixels).
inline size_t dconv_lds_bytes(int BM, int BN, int NS, int waves_n, int kw, int bk, int Cs, size_t np)
{
    const size_t spp = (size_t)Cs / 8 + 1;                 // 16-byte slots per patch pixel (one unused)
    const size_t nwl = (np * spp + 63) / 64;
    const size_t pz = (nwl * 64 + spp - 1) / spp;          // the zero area sits behind the whole wave-loads,
    // at the next multiple of 256 bytes: 256 bytes, a pixel's channels and the two K halves' reach
    const size_t main_loop = ((size_t)kw * NS * BN * bk * 2 + pz * spp * 16 + 255) / 256 * 256 + 512 + (size_t)Cs * 2 + 32;
    // output staging: per K group [BM][BN + 8 floats per wave column], + the split-K flag
    const size_t staging = (size_t)kw * BM * (BN + 8 * waves_n) * 4 + 16;
    return main_loop > staging ? main_loop : staging;
}

template <int BM, int BN, int WGM, int WGN, int KW, int NS, int BK, int KR, int NCC>
hipError_t dconv_launch_kr(const DconvParams &p, size_t lds, hipStream_t st)
{
    auto kern = dconv_kernel<BM, BN, WGM, WGN, KW, NS, BK, KR, NCC>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int tiles = p.tiles_m * p.tiles_n;
    const unsigned grid = (unsigned)(tiles * p.splitk);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * WGM * WGN * KW), lds, st, p);
    return hipGetLastError();
}

// 1x1 filters over up to 512 channels per K group and 3x3 filters over 64 or 128 have
// fully unrolled kernels; everything else walks taps and chunks at run time.  Kernels
// with 32-channel K steps (BK = 32: smaller weight stages) exist for 3x3 filters over
// 32 or 64 channels per K group.
template <int BM, int BN, int WGM, int WGN, int KW, int NS, int BK>
hipError_t dconv_launch(const DconvParams &p, size_t lds, hipStream_t st)
{
    if (p.bk != BK) return hipErrorInvalidValue;
    if constexpr (BK == 32) {
        if (p.R == 3 && p.S == 3 && p.ncc == 1) return dconv_launch_kr<BM, BN, WGM, WGN, KW, NS, 32, 3, 1>(p, lds, st);
        if (p.R == 3 && p.S == 3 && p.ncc == 2) return dconv_launch_kr<BM, BN, WGM, WGN, KW, NS, 32, 3, 2>(p, lds, st);
        return hipErrorInvalidValue;
    } else {
        if (p.R == 3 && p.S == 3) {
            if (p.ncc == 1) return dconv_launch_kr<BM, BN, WGM, WGN, KW, NS, 64, 3, 1>(p, lds, st);
            if (p.ncc == 2) return dconv_launch_kr<BM, BN, WGM, WGN, KW, NS, 64, 3, 2>(p, lds, st);
        } else if (p.R == 1 && p.S == 1) {
            if (p.ncc == 1) return dconv_launch_kr<BM, BN, WGM, WGN, KW, NS, 64, 1, 1>(p, lds, st);
            if (p.ncc == 2) return dconv_launch_kr<BM, BN, WGM, WGN, KW, NS, 64, 1, 2>(p, lds, st);
            if (p.ncc == 4) return dconv_launch_kr<BM, BN, WGM, WGN, KW, NS, 64, 1, 4>(p, lds, st);
            if constexpr (KW == 1)
                if (p.ncc == 8) return dconv_launch_kr<BM, BN, WGM, WGN, KW, NS, 64, 1, 8>(p, lds, st);
        }
        return dconv_launch_kr<BM, BN, WGM, WGN, KW, NS, 64, 0, 0>(p, lds, st);
    }
}

}  // namespace alt

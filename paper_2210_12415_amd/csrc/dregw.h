// Direct 3x3 convolution for layers whose whole weight tensor fits the register file:
// at most 64 output channels over 32 or 64 input channels (the first stage of a ResNet),
// bf16 operands, fp32 accumulation, at large batches.
//
// In the tile kernels (dconv.h) a 32x32x16 MFMA needs one 1 KB operand fragment of pixels and
// one of weights out of LDS, and for 64 output channels no wave tile can amortise them
// further: four SIMDs at full MFMA rate would ask the LDS for more than it delivers, and a
// workgroup's start-up, address arithmetic and epilogue are only hidden by a second
// workgroup on the same compute unit.  Here
//
//  * a wave holds every weight fragment it will ever need in registers (one wave per SIMD,
//    512 registers per lane), so the main loop reads only pixels: half the LDS traffic, no
//    weight ring, no barrier per K step;
//  * one workgroup of four waves per compute unit stays resident and walks a contiguous range of
//    output tiles of 128 pixels.  Consecutive tiles' patches overlap in all but 128 pixels, so
//    the input streams through a ring of pixels in LDS, each pixel fetched once; the loads run
//    several tiles ahead of the tile being computed (a tile is shorter than the memory
//    latency under load);
//  * everything a tile needs besides its MFMAs runs in the shadow of the neighbouring tiles'
//    MFMAs: the patch rows of tile k + 1 are computed during tile k, and tile k's reduction,
//    bias, activation, conversion and stores are spread over the K steps of tile k + 1 (the
//    accumulators are double-buffered).
//
// The four waves are two pixel halves (64 pixels each) by two channel halves: a wave
// multiplies its 64 pixels by all 64 output channels over half of the input channels (all
// taps), which halves its weight registers (144 for 64 input channels) and leaves the LDS
// traffic where it was (each wave reads only its channels of a pixel).  The two waves of a
// pair then trade halves through LDS: each finishes 32 of the pair's 64 pixels.  So that both
// run the same code, wave kg of a pair calls pixels [32 * kg, 32 * kg + 32) of the pair its
// row tile 0 and the others its row tile 1: everybody keeps row tile 0 and sends row tile 1.
//
// For bf16 output a lane swaps half of its values with lane ^ 32 (v_permlane32_swap) so that
// both hold eight consecutive channels of a pixel, and stores 16 bytes.
//
// Covers stride 1, no dilation, output size = input size (padding 1), activations and
// output NHWC or N C/b H W b, weights OHWI, bias and ReLU; no split-K, no fused sum.
#pragma once

#include "dconv.h"

namespace alt {

constexpr int kRegwBM = 128;             // output pixels of a tile
constexpr int kRegwExchange = 32 * 1024; // LDS bytes of the pairs' exchange: four waves x 32 registers x 64 lanes

template <int KR, int CCH>
__global__ __launch_bounds__(256, 1) void dregw_kernel(const DconvParams p)
{
    constexpr int TM = 2, TN = 2, RS = KR * KR;
    constexpr int KCL = CCH / 2, NC = RS * KCL;            // k chunks per tap and per tile of one wave
    constexpr int NG = RS * CCH;                           // k chunks of the layer
    constexpr int BM = kRegwBM;
    constexpr int WLW = NG * TN / 4;                       // weight wave-loads per wave
    static_assert(CCH % 2 == 0 && (NG * TN) % 4 == 0 && NC * TN * 4 <= 160, "the weight fragments of a wave against the register file");

    extern __shared__ uint4 smem_u4[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)smem_u4;    // the pixel ring, the zero row, the pairs' exchange, the bias
    float *bias_lds = (float *)((char *)smem_u4 + p.regw_bias_off);
    char *xch = (char *)smem_u4 + p.regw_bias_off - kRegwExchange;

    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int kg = wave & 1, wm = wave >> 1;               // channel half, pixel half
    const int h = lane >> 5;

    // ---- this workgroup's tiles: the contiguous range [t0, t1) (the grid never exceeds the tiles)
    const int G = (int)gridDim.x, b = (int)blockIdx.x;
    const int t0 = (int)((int64_t)b * p.tiles_m / G), t1 = (int)((int64_t)(b + 1) * p.tiles_m / G);
    const int count = t1 - t0;
    if (count == 0) return;

    // ---- the pixel stream.  Output pixel m sits over input pixel m, so tile k of the range needs input pixels
    // [k BM, (k + 1) BM + halo + halo_hi) counted from the range's first one, g_start.  Stream slot s is 16-byte
    // slot s % spp of pixel s / spp (spp slots per pixel, the last one unused: the odd pitch spreads the MFMA
    // operand reads over the banks) and lives at LDS slot s modulo the ring, which holds P pixels.  A unit is
    // 256 slots, one wave-load per wave.
    const int halo = p.pad_h * p.W + p.pad_w;
    const int halo_hi = (KR - 1 - p.pad_h) * p.W + (KR - 1 - p.pad_w);
    const int hw = p.H * p.W;
    const int spp = (1 << p.log2_cpp) + 1;
    const int pitch_b = spp * 16;
    const int P = p.regw_ring_px;
    const uint32_t ring_bytes = (uint32_t)(P * pitch_b);
    const int ahead = p.regw_ahead;                        // the loads run this many tiles ahead of the MFMAs
    const int g_start = t0 * BM - halo;
    const int range_px = halo + count * BM + halo_hi;
    auto units_upto = [&](int k) { return ((halo + (k + 1) * BM + halo_hi) * spp + 255) >> 8; };   // units that complete tile k's patch

    const i32x4_t x_rsrc = make_rsrc(p.x, p.x_bytes);
    int ucur = 0;                                          // next unit to issue
    uint32_t uoff = (uint32_t)wave * 1024;                 // where this wave's share of it goes in the ring
    // Issues units [ucur, upto).  Past the end of the range the loads are out of range (they fetch nothing and
    // write zeros over pixels no longer needed): every tile issues its share, which keeps the count of loads in
    // flight behind a tile's own a function of the tile number alone.
    auto issue_units = [&](int upto) {
        for (; ucur < upto; ++ucur) {
            const int slot = (ucur * 4 + wave) * 64 + lane;
            const int px = (int)div32((uint32_t)slot, p.d_slots), c = slot - px * spp;
            const int gp = g_start + px;
            const bool ok = c < spp - 1 && px < range_px && (unsigned)gp < (unsigned)p.in_px;
            const uint32_t voff = ok ? dconv_in_elem(p, gp, c * 8) * 2u : kOutOfRange;
            dma_load16(x_rsrc, voff, lds0 + uoff);
            uoff += 4096;
            uoff -= uoff >= ring_bytes ? ring_bytes : 0u;
        }
    };
    // Waits until at most n of this wave's loads and stores are outstanding.
    auto wait_outstanding = [&](int n) {
        switch (n < 20 ? n : 20) {
        case 20: wait_vmcnt<20>(); break;
        case 19: wait_vmcnt<19>(); break;
        case 18: wait_vmcnt<18>(); break;
        case 17: wait_vmcnt<17>(); break;
        case 16: wait_vmcnt<16>(); break;
        case 15: wait_vmcnt<15>(); break;
        case 14: wait_vmcnt<14>(); break;
        case 13: wait_vmcnt<13>(); break;
        case 12: wait_vmcnt<12>(); break;
        case 11: wait_vmcnt<11>(); break;
        case 10: wait_vmcnt<10>(); break;
        case 9: wait_vmcnt<9>(); break;
        case 8: wait_vmcnt<8>(); break;
        case 7: wait_vmcnt<7>(); break;
        case 6: wait_vmcnt<6>(); break;
        case 5: wait_vmcnt<5>(); break;
        case 4: wait_vmcnt<4>(); break;
        case 3: wait_vmcnt<3>(); break;
        case 2: wait_vmcnt<2>(); break;
        case 1: wait_vmcnt<1>(); break;
        default: wait_vmcnt<0>(); break;
        }
    };
    const int pz = P;                                      // the all-zero pixel row sits behind the ring

    // ---- prologue: the weights go to LDS in fragment order (slot (g * 2 + j) * 64 + lane is what lane `lane`
    // feeds the MFMAs of k chunk g and column tile j: row j * 32 + lane % 32, k half lane / 32), behind the
    // first tile's patch; every wave then copies its channel half of them into its registers
    const uint32_t wst = (uint32_t)units_upto(0) * 4096;   // byte offset of the weights' staging area in the ring
    {
        const i32x4_t w_rsrc = make_rsrc(p.w, p.w_bytes);
        const int rsc = RS * p.C;
#pragma unroll
        for (int q = 0; q < WLW; ++q) {
            const int idx = wave * WLW + q;                // column tile first: consecutive loads walk along the rows
            const int j = idx / NG, g = idx - j * NG;
            const int n = j * 32 + (lane & 31);
            const uint32_t voff = n < p.Nc ? (uint32_t)(n * rsc + g * 16 + h * 8) * 2u : kOutOfRange;
            dma_load16(w_rsrc, voff, lds0 + wst + (uint32_t)(g * TN + j) * 1024);
        }
        issue_units(units_upto(0));
        if (t < spp - 1) *(uint4 *)((char *)smem_u4 + pz * pitch_b + t * 16) = make_uint4(0, 0, 0, 0);
        if (t < 64) bias_lds[t] = (p.flags & ALT_EPI_BIAS) && t < p.Nc ? p.bias[t] : 0.f;
    }
    wait_vmcnt<0>();
    __syncthreads();
    u32x4_t wreg[NC][TN];                                  // chunk c = tap * KCL + kcl of this wave is chunk tap * CCH + kg * KCL + kcl
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int g = (c / KCL) * CCH + kg * KCL + c % KCL;
            wreg[c][j] = *(const u32x4_t *)((const char *)smem_u4 + wst + (uint32_t)((g * TN + j) * 64 + lane) * 16);
        }
    __syncthreads();                                       // the staging area is ring again from here on
    issue_units(units_upto(ahead));                        // tiles 1 .. ahead

    const uint32_t koff = h * 16 + kg * (KCL * 32);        // this lane's first byte inside a patch pixel
    const __amdgpu_buffer_rsrc_t yr = __builtin_amdgcn_make_buffer_rsrc(p.y, 0, (int)p.y_bytes, 0x00020000);
    const float relu_floor = (p.flags & ALT_EPI_RELU) ? 0.f : -INFINITY;
    const bool out_bf16 = p.flags & kDconvOutBf16;
    const int row0 = wm * 64 + (lane & 31);                // row tile i of this wave: pixels row0 + 32 * (i ^ kg) of the tile

    // Ring row under every tap for this lane's pixels of tile k of the range, whose first pixel sits at ring
    // pixel kbase = k BM mod P (taps outside the image, and pixels past the end: the zero row)
    auto tap_rows = [&](uint32_t (&rows)[RS][TM], int k, int kbase) {
        const int m0 = (t0 + k) * BM;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int m = m0 + row0 + 32 * (i ^ kg);
            const bool m_ok = m < p.M;
            const int mm = m_ok ? m : 0;
            const int rem = mm - (int)div32((uint32_t)mm, p.d_hw) * hw;
            const int oh = (int)div32((uint32_t)rem, p.d_w), ow = rem - oh * p.W;
            const int row_px = kbase + row0 + 32 * (i ^ kg) + halo;
            const bool up = m_ok && oh >= p.pad_h, down = m_ok && oh + (KR - 1 - p.pad_h) < p.H;
            const bool left = ow >= p.pad_w, right = ow + (KR - 1 - p.pad_w) < p.W;
#pragma unroll
            for (int tap = 0; tap < RS; ++tap) {
                const int r = tap / KR, s = tap % KR;
                // (3x3, padding 1: the tap's row or column leaves the image only at the first and last ones)
                const bool ok = (r == 0 ? up : r == KR - 1 ? down : m_ok) && (s == 0 ? left : s == KR - 1 ? right : true);
                const uint32_t lin = (uint32_t)(row_px + (r - p.pad_h) * p.W + (s - p.pad_w));     // below 2 P
                const uint32_t px = ok ? min(lin, lin - (uint32_t)P) : (uint32_t)pz;
                rows[tap][i] = lds0 + px * (uint32_t)pitch_b + koff;
            }
        }
    };

    // ---- a finished tile: its accumulators, and the pieces of its way to memory --------------------------------
    int prev_m0 = p.M;                                     // (no previous tile yet: every store is out of range)
    // the wave's row tile 1 goes to its partner
    auto send_half = [&](floatx16_t (&accP)[TM][TN]) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                *(float4 *)(xch + wave * 8192 + ((j * 4 + q) * 64 + lane) * 16) =
                    make_float4(accP[1][j][4 * q], accP[1][j][4 * q + 1], accP[1][j][4 * q + 2], accP[1][j][4 * q + 3]);
    };
    // the partner's row tile 1 is this wave's row tile 0; column tile j goes to memory.
    // Register e of lane l holds (pixel l % 32, channel 8 * (e / 4) + 4 * (l / 32) + e % 4) of a 32x32 tile.
    auto finish = [&](floatx16_t (&accP)[TM][TN], auto jc) {
        constexpr int j = decltype(jc)::value;
        const int m = prev_m0 + row0 + 32 * kg;
        const bool m_ok = m < p.M;
        float v[16];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 o = *(const float4 *)(xch + (wave ^ 1) * 8192 + ((j * 4 + q) * 64 + lane) * 16);
            const float4 b4 = *(const float4 *)(bias_lds + j * 32 + 8 * q + 4 * h);
            v[4 * q + 0] = fmaxf(accP[0][j][4 * q + 0] + o.x + b4.x, relu_floor);
            v[4 * q + 1] = fmaxf(accP[0][j][4 * q + 1] + o.y + b4.y, relu_floor);
            v[4 * q + 2] = fmaxf(accP[0][j][4 * q + 2] + o.z + b4.z, relu_floor);
            v[4 * q + 3] = fmaxf(accP[0][j][4 * q + 3] + o.w + b4.w, relu_floor);
        }
        if (out_bf16) {
            // Lanes l and l + 32 hold the two halves of every group of eight channels of one pixel.  Swapping the
            // upper lanes of group q's registers with the lower lanes of group q + 2's leaves the lower lane with
            // both halves of group q (its own in the first register, the partner's in the second) and the upper
            // lane with both halves of group q + 2, in channel order either way.
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                u32x2_t r0 = __builtin_amdgcn_permlane32_swap(f32x2_to_bf16x2(v[4 * q], v[4 * q + 1]),
                                                              f32x2_to_bf16x2(v[4 * q + 8], v[4 * q + 9]), false, false);
                u32x2_t r1 = __builtin_amdgcn_permlane32_swap(f32x2_to_bf16x2(v[4 * q + 2], v[4 * q + 3]),
                                                              f32x2_to_bf16x2(v[4 * q + 10], v[4 * q + 11]), false, false);
                const int n = j * 32 + 8 * (q + 2 * h);
                const u32x4_t ov = {r0.x, r1.x, r0.y, r1.y};
                const bool ok = m_ok && n < p.Nc;
                __builtin_amdgcn_raw_buffer_store_b128(ov, yr, (int)(ok ? dconv_out_elem(p, m, n) * 2u : kOutOfRange), 0, 0);
            }
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = j * 32 + 8 * q + 4 * h;
                const u32x4_t ov = {__builtin_bit_cast(uint32_t, v[4 * q]), __builtin_bit_cast(uint32_t, v[4 * q + 1]),
                                    __builtin_bit_cast(uint32_t, v[4 * q + 2]), __builtin_bit_cast(uint32_t, v[4 * q + 3])};
                const bool ok = m_ok && n < p.Nc;
                __builtin_amdgcn_raw_buffer_store_b128(ov, yr, (int)(ok ? dconv_out_elem(p, m, n) * 4u : kOutOfRange), 0, 0);
            }
        }
    };

    constexpr int D = 3, NBUF = 4;                         // pixel fragments run D k chunks ahead of their MFMAs
    static_assert(D * TM <= 15 && D < NBUF && NC > D + 5, "fragment reads in flight; room for the previous tile's steps");
    u32x4_t af[NBUF][TM];
    int kbase = 0;                                         // ring pixel of the present tile's first pixel

    // Tile k: its sums go to `acc`, its patch rows are `rows`; `accP` holds tile k - 1 and `rows_next` takes
    // the patch rows of tile k + 1.
    auto tile = [&](int k, floatx16_t (&acc)[TM][TN], floatx16_t (&accP)[TM][TN], uint32_t (&rows)[RS][TM],
                    uint32_t (&rows_next)[RS][TM]) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

        // ---- main loop.  It is one basic block: no fragment read is in flight across a branch (the compiler
        // copies registers at joins, and a copy of a register whose read has not landed is stale), and the
        // previous tile's steps run for the first tile too, on zeros and with every store out of range.
        auto reads = [&](auto cc) {
            constexpr int c = decltype(cc)::value, tap = c / KCL, kcl = c % KCL, buf = c % NBUF;
            static_for<TM>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                lds_read16_async_at<kcl * 32>(af[buf][i], rows[tap][i]);
            });
        };
        static_for<D>([&](auto cc) { reads(cc); });
        static_for<NC>([&](auto cc) {
            constexpr int c = decltype(cc)::value, buf = c % NBUF;
            if constexpr (c + D < NC) reads(std::integral_constant<int, c + D>{});
            constexpr int ahead = c + D < NC ? D : NC - 1 - c;
            asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(af[buf][0]) : "n"(ahead * TM) : "memory");
#pragma unroll
            for (int i = 1; i < TM; ++i) asm volatile("" : "+v"(af[buf][i]));
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, wreg[c][j]),
                                                                        __builtin_bit_cast(bf16x8_t, af[buf][i]), acc[i][j], 0, 0, 0);
            // the previous tile, and the next one's patch rows, in the shadow of these MFMAs
            if constexpr (c == 0) send_half(accP);
            if constexpr (c == 1) lds_barrier();
            if constexpr (c == 2) finish(accP, std::integral_constant<int, 0>{});
            if constexpr (c == 3) finish(accP, std::integral_constant<int, 1>{});
            if constexpr (c == 4) {
                kbase += BM;
                kbase -= kbase >= P ? P : 0;
                tap_rows(rows_next, k + 1, kbase);
            }
        });

        // The next tile's patch has landed once this wave's loads for the tiles behind it are all that is
        // outstanding (loads complete in order; the stores issued since are younger still and only make the wait
        // stricter).  Behind the barrier everybody's share has landed and every wave is through with this
        // tile's pixels and with the exchange, so the loads of tile k + 1 + ahead may overwrite them.
        wait_outstanding(units_upto(k + ahead) - units_upto(k + 1));
        lds_barrier();
        issue_units(units_upto(k + 1 + ahead));
        prev_m0 = (t0 + k) * BM;
    };
    auto last = [&](floatx16_t (&accP)[TM][TN]) {
        send_half(accP);
        lds_barrier();
        finish(accP, std::integral_constant<int, 0>{});
        finish(accP, std::integral_constant<int, 1>{});
    };

    // two tiles per trip, the two sets of accumulators and patch rows trading places
    floatx16_t acc_a[TM][TN], acc_b[TM][TN];
    uint32_t rows_a[RS][TM], rows_b[RS][TM];
    tap_rows(rows_a, 0, 0);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc_b[i][j][e] = 0.f;
    int k = 0;
    for (; k + 1 < count; k += 2) {
        tile(k, acc_a, acc_b, rows_a, rows_b);
        tile(k + 1, acc_b, acc_a, rows_b, rows_a);
    }
    if (k < count) {
        tile(k, acc_a, acc_b, rows_a, rows_b);
        last(acc_a);
    } else {
        last(acc_b);
    }
    wait_vmcnt<0>();                                       // the loads issued past the end of the range
}

// Ring size and look-ahead for a layer (W = image width, padding 1), or false if no ring fits LDS: the ring must
// hold the tiles from the one about to start to the one being loaded (ahead + 1 tiles and the taps' reach, plus
// the pixels a load unit may run past a tile), and, before the first tile, the first patch and the weights in
// fragment order side by side.  *bias_off: where the bias sits (the exchange just before it); *lds: bytes in all.
inline bool dregw_plan(int C, int W, int *ring_px, int *ahead, uint32_t *bias_off, size_t *lds)
{
    const int spp = C / 8 + 1, pitch = spp * 16, reach = 2 * (W + 1);
    const size_t first = (size_t)(((reach + kRegwBM) * spp + 255) / 256) * 4096;
    const size_t wb = (size_t)9 * (C / 16) * 2 * 1024;
    for (int a = 4; a >= 2; --a) {
        size_t need = (size_t)(a + 1) * kRegwBM + reach + 256 / spp + 2;
        const size_t stage_px = (first + wb + pitch - 1) / pitch;
        if (stage_px > need) need = stage_px;
        const size_t P = (need + 63) / 64 * 64;
        const size_t total = (P + 1) * pitch + kRegwExchange + 256;
        if (total <= 160 * 1024) {
            *ring_px = (int)P;
            *ahead = a;
            *bias_off = (uint32_t)((P + 1) * pitch + kRegwExchange);
            *lds = total;
            return true;
        }
    }
    return false;
}

template <int KR, int CCH>
hipError_t dregw_launch_c(const DconvParams &p, size_t lds, hipStream_t st)
{
    auto kern = dregw_kernel<KR, CCH>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    if (p.regw_grid < 1 || p.regw_grid > p.tiles_m) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kern, dim3((unsigned)p.regw_grid), dim3(256), lds, st, p);
    return hipGetLastError();
}

inline hipError_t dregw_launch(const DconvParams &p, size_t lds, hipStream_t st)
{
    if (p.R != 3 || p.S != 3) return hipErrorInvalidValue;
    if (p.C == 64) return dregw_launch_c<3, 4>(p, lds, st);
    if (p.C == 32) return dregw_launch_c<3, 2>(p, lds, st);
    return hipErrorInvalidValue;
}

}  // namespace alt

// Direct convolution for channel-planar tensors: activations NCHW, weights OIHW, output NCHW,
// the layouts a network arrives in before any layout is chosen (Section 5.1 of the paper
// takes them as the starting point of the layout search).
//
// The matrix cores want eight consecutive reduction channels per lane for both operands,
// and in these layouts consecutive channels are a whole image plane (activations) or a whole
// filter (weights) apart.  The kernel therefore converts on the way into LDS and then runs
// the same loop as the patch-resident kernel of dconv.h:
//
//  * activations: the tile's patch (its BM output pixels plus the taps' reach) is read
//    plane by plane in 16-byte runs of eight pixels, eight planes per thread, transposed
//    8x8 in registers and written as 16-byte channel chunks: in LDS the patch is
//    [pixel][channel], exactly what dconv.h holds;
//  * weights: a filter row is contiguous over (channel, tap), so the 64 channels x all taps
//    of a "super-step" are read as one contiguous run per output channel and scattered
//    element by element into one [row][64 channels] stage per tap; the loads of the next
//    super-step are in registers while the present one computes;
//  * output: the accumulators (pixels along the MFMA rows, so a lane holds four consecutive
//    pixels of one channel) go through LDS as [channel][pixel] and are stored with
//    consecutive lanes on consecutive pixels of a plane.
//
// K groups: KW groups of waves each take every KW-th 16-channel chunk of a tap's 64
// channels; their tiles are summed in group order when the staged output is read back.
//
// The output may also be NHWC (eight output channels per store): the layer then converts the
// layout for an NHWC consumer by itself, which is how layout propagation (Section 4.2) lets a
// chain that starts in NCHW do without a conversion operator.
//
// Covers: bf16, 1x1 and 3x3 filters, stride 1 or 2, any dilation, padding from none to
// same-size, channels a multiple of 64, images of at least eight pixels, fp32 or bf16
// output, bias and ReLU.  No split-K and no fused addend.
#pragma once

#include "dconv.h"

namespace alt {

// Sixteen bytes at any even address (the hardware takes unaligned global loads).
struct __attribute__((packed, aligned(2))) PlanarRun {
    u32x4_t v;
};
__device__ __forceinline__ uint4 planar_run(const uint16_t *src)
{
    const u32x4_t v = ((const PlanarRun *)src)->v;
    return make_uint4(v.x, v.y, v.z, v.w);
}

// Four floats at any address that is a multiple of four.
struct __attribute__((packed, aligned(4))) PlanarRunF {
    f32x4_t v;
};

constexpr int kPlanarOutNhwc = 8;                // flag: the output is NHWC, not NCHW

constexpr int kPlanarWP = 144;                   // bytes of a weight row in LDS: 64 channels and one unused 16-byte slot

// LDS bytes of one tap's weight stage: BN rows, then 16 bytes that skew consecutive taps over the banks.
constexpr int planar_stage_bytes(int BN) { return BN * kPlanarWP + 16; }

inline size_t dplanar_lds_bytes(int BM, int BN, int kw, int taps, int C, size_t np)
{
    const size_t npr = (np + 7) / 8 * 8;
    // (the zero area behind the patch: at the next multiple of 256 bytes, 256 bytes and a pixel's channels)
    const size_t main_loop = ((size_t)taps * planar_stage_bytes(BN) + npr * ((size_t)C * 2 + 16) + 255) / 256 * 256 + 512 + (size_t)C * 2 + 32;
    // output staging: [channel][pixel] (NCHW output) or [pixel][channel] (NHWC output), the larger of the two
    const size_t staging = std::max((size_t)kw * BN * (BM + 4) * 4, (size_t)kw * BM * (BN + 4) * 4);
    return main_loop > staging ? main_loop : staging;
}

template <int BM, int BN, int WGM, int WGN, int KW, int KR>
__global__ __launch_bounds__(64 * WGM * WGN * KW) void dplanar_kernel(const DconvParams p)
{
    constexpr int NWG = WGM * WGN, NW = NWG * KW, NT = 64 * NW;
    constexpr int WTM = BM / WGM, WTN = BN / WGN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int RS = KR * KR;
    constexpr int WP = kPlanarWP, WST = planar_stage_bytes(BN);
    static_assert(WTM % 32 == 0 && WTN % 32 == 0 && TM >= 1 && TN >= 1, "wave tile");
    static_assert(KW == 1 || KW == 2 || KW == 4, "K groups divide the four 16-channel chunks of a step");
    static_assert(NT % BM == 0, "the output pass gives every thread one pixel");

    extern __shared__ uint4 smem_u4[];
    char *smem = (char *)smem_u4;                          // the taps' weight stages first, then the patch

    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int kg = wave / NWG, wq = wave % NWG;
    const int wm = wq / WGN, wn = wq % WGN;

    int mt, nt;
    {
        const int ntot = p.tiles_m * p.tiles_n;
        const int logical = igemm_logical_tile(ntot);
        nt = (int)div32((uint32_t)logical, p.d_tm);
        mt = logical - nt * p.tiles_m;
    }
    const int m0 = mt * BM, n0 = nt * BN;
    const uint16_t *xg = (const uint16_t *)p.x;
    const uint16_t *wg = (const uint16_t *)p.w;
    const int HW = p.H * p.W;

    // ---- weights of super-step sb (channels 64*sb ..): global -> registers -> the taps' stages ----------
    // Thread (row, cg) owns the run of eight channels x all taps of one filter row: RS consecutive
    // 16-byte pieces.  Per tap it picks its eight channels out of them (elements RS apart) and
    // writes them as one 16-byte chunk of that tap's stage.
    static_assert(NT >= BN * 8, "one thread per (row, eight channels)");
    const int w_row = t >> 3, w_cg = t & 7;
    const bool w_live = t < BN * 8 && n0 + w_row < p.Nc;
    uint4 wreg[RS];
    auto load_w = [&](int sb) {
        const uint16_t *src = wg + ((size_t)(n0 + w_row) * p.C + (size_t)sb * 64 + w_cg * 8) * RS;
#pragma unroll
        for (int i = 0; i < RS; ++i) {
            const uint4 v = *(const uint4 *)(w_live ? src + i * 8 : wg);
            wreg[i] = w_live ? v : make_uint4(0, 0, 0, 0);
        }
    };
    auto scatter_w = [&]() {
        if (t < BN * 8) {
            uint32_t d[RS * 4];
#pragma unroll
            for (int i = 0; i < RS; ++i) { d[4 * i] = wreg[i].x; d[4 * i + 1] = wreg[i].y; d[4 * i + 2] = wreg[i].z; d[4 * i + 3] = wreg[i].w; }
#pragma unroll
            for (int tap = 0; tap < RS; ++tap) {
                uint32_t o[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int fl = (2 * k) * RS + tap, fh = (2 * k + 1) * RS + tap;   // elements of channels 2k and 2k + 1
                    const uint32_t sel = ((fl & 1) ? 0x0302u : 0x0100u) | ((fh & 1) ? 0x07060000u : 0x05040000u);
                    o[k] = __builtin_amdgcn_perm(d[fh >> 1], d[fl >> 1], sel);
                }
                *(uint4 *)(smem + tap * WST + w_row * WP + w_cg * 16) = make_uint4(o[0], o[1], o[2], o[3]);
            }
        }
    };
    load_w(0);

    // ---- the patch: input pixels [a0 - halo, a0 - halo + np), all C channels, as [pixel][channel] ----------
    const int halo = p.pad_h * p.W + p.pad_w;
    const int halo_hi = ((p.R - 1) * p.dil - p.pad_h) * p.W + ((p.S - 1) * p.dil - p.pad_w);
    const int ohw = p.OH * p.OW;
    auto anchor = [&](int m) {
        const int img = (int)div32((uint32_t)m, p.d_hw), rem = m - img * ohw;
        const int oh = (int)div32((uint32_t)rem, p.d_w), ow = rem - oh * p.OW;
        return img * HW + (oh * p.W + ow) * p.stride;
    };
    const int a0 = anchor(m0);
    const int np = anchor(min(m0 + BM, p.M) - 1) - a0 + 1 + halo + halo_hi;
    const int npr = (np + 7) & ~7;                         // whole blocks of eight pixels
    const int pitch_b = p.C * 2 + 16;
    char *patch = smem + RS * WST;
    // behind the patch, at a multiple of 256 bytes: the zero area that taps outside the image read, each lane at
    // the offset modulo 256 (i.e. on the banks) of the pixel it would have read (see dconv.h)
    const uint32_t patch_a = (uint32_t)(uintptr_t)patch;
    const uint32_t zero0 = (patch_a + (uint32_t)(npr * pitch_b) + 255u) & ~255u;
    {
        // Work items: (pixel block of eight, channel block of eight), one per lane: the lane loads its eight
        // planes' runs, transposes them 8x8 in registers and writes eight 16-byte channel chunks.  A set of 64
        // items is eight pixel blocks (lane % 8) x eight channel blocks (lane / 8): its loads cover 128
        // contiguous bytes of each plane, and each of its LDS writes covers every bank four times, which is the
        // least a 16-byte-per-lane write takes.
        const int g0 = a0 - halo;
        const int npb = npr >> 3;                          // pixel blocks
        const int npbg = (npb + 7) >> 3;                   // sets along the pixels; C / 64 along the channels
        const int nitems = npbg * (p.C >> 6) * 64;
        struct Item {
            int px0, cb, q;
            bool live, inside, straddle;
            size_t e0;
        };
        auto item_of = [&](int first) {
            Item it;
            const int set = first >> 6;
            const int cbg = set / npbg, pbg = set - cbg * npbg;
            const int pb = pbg * 8 + (lane & 7);
            it.cb = cbg * 8 + (lane >> 3);
            it.px0 = pb * 8;
            const int cb = it.cb;
            const int g = g0 + it.px0;                     // first input pixel of the block
            it.live = first < nitems && pb < npb;
            it.inside = it.live && g >= 0 && g + 7 < p.in_px;
            const int img = it.inside ? (int)div32((uint32_t)g, p.d_ihw) : 0;
            it.q = (img + 1) * HW - g;                     // pixels of the block that lie in image `img`
            it.straddle = it.inside && it.q < 8;
            // element index of pixel g + e, channel c: g + e + (img * (C - 1) + c) * HW
            it.e0 = (size_t)g + ((size_t)img * (p.C - 1) + (size_t)cb * 8) * HW;
            return it;
        };
        auto item_load = [&](const Item &it, uint4 (&blk)[8], uint4 (&nx)[8], bool any_straddle) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                // (lanes without a block load the tensor's first bytes instead of branching round the load)
                const uint4 v = planar_run(it.inside ? xg + it.e0 + (size_t)i * HW : xg);
                blk[i] = it.inside ? v : make_uint4(0, 0, 0, 0);
            }
            if (any_straddle) {
                // pixels q .. 7 belong to the next image: the same run, (C - 1) planes further on
                const size_t e1 = it.e0 + (it.straddle ? (size_t)(p.C - 1) * HW : 0);
#pragma unroll
                for (int i = 0; i < 8; ++i) nx[i] = planar_run(it.inside ? xg + e1 + (size_t)i * HW : xg);
            }
        };
        auto item_write = [&](const Item &it, uint4 (&blk)[8]) {
            transpose8x8_b16(blk);                         // blk[j]: pixel px0 + j, channels 8*cb .. 8*cb + 7
            if (it.live) {
#pragma unroll
                for (int j = 0; j < 8; ++j) *(uint4 *)(patch + (size_t)(it.px0 + j) * pitch_b + it.cb * 16) = blk[j];
            }
        };
        auto item_store = [&](const Item &it, uint4 (&blk)[8], uint4 (&nx)[8], bool any_straddle) {
            if (any_straddle) {
                uint32_t msk[4];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    msk[j] = !it.straddle || it.q >= 2 * j + 2 ? 0xffffffffu : it.q == 2 * j + 1 ? 0x0000ffffu : 0u;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    blk[i].x = (blk[i].x & msk[0]) | (nx[i].x & ~msk[0]);
                    blk[i].y = (blk[i].y & msk[1]) | (nx[i].y & ~msk[1]);
                    blk[i].z = (blk[i].z & msk[2]) | (nx[i].z & ~msk[2]);
                    blk[i].w = (blk[i].w & msk[3]) | (nx[i].w & ~msk[3]);
                }
            }
            item_write(it, blk);
        };
        // a set with a block that reaches before the first or behind the last input pixel: element by element,
        // every load unconditional (at element 0 where the pixel does not exist) so that all are in flight together
        auto item_slow = [&](const Item &it) {
            const int g = g0 + it.px0;
            size_t eb[8];
            bool eok[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int ge = g + e;
                eok[e] = it.live && ge >= 0 && ge < p.in_px;
                const int gs = eok[e] ? ge : 0;
                const int im = (int)div32((uint32_t)gs, p.d_ihw);
                eb[e] = (size_t)gs + ((size_t)im * (p.C - 1) + (size_t)it.cb * 8) * HW;
            }
            uint4 blk[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                uint32_t v[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const uint32_t ld = xg[eok[e] ? eb[e] + (size_t)i * HW : 0];
                    v[e] = eok[e] ? ld : 0u;
                }
                blk[i] = make_uint4(v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16));
            }
            item_write(it, blk);
        };
        for (int first = wave * 64; first < nitems; first += NW * 64) {
            const Item a = item_of(first);
            if (__builtin_amdgcn_ballot_w64(a.live && !a.inside) != 0) {
                item_slow(a);
            } else {
                const bool str_a = __builtin_amdgcn_ballot_w64(a.straddle) != 0;
                uint4 blk[8], nx[8];
                item_load(a, blk, nx, str_a);
                item_store(a, blk, nx, str_a);
            }
        }
        for (int i = t; i < 16 + (p.C >> 3) + 2; i += NT)
            *(uint4 *)(patch + (zero0 - patch_a) + i * 16) = make_uint4(0, 0, 0, 0);
    }
    scatter_w();
    const int nsb = p.C >> 6;
    if (nsb > 1) load_w(1);
    __syncthreads();

    // ---- per-lane rows of the MFMA tiles -----------------------------------------------------------------
    int32_t row_px[TM], row_oh[TM], row_ow[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int m = m0 + wm * WTM + i * 32 + (lane & 31);
        if (m < p.M) {
            const int img = (int)div32((uint32_t)m, p.d_hw), rem = m - img * ohw;
            const int oh = (int)div32((uint32_t)rem, p.d_w), ow = rem - oh * p.OW;
            row_oh[i] = oh * p.stride;
            row_ow[i] = ow * p.stride;
            row_px[i] = img * HW + row_oh[i] * p.W + row_ow[i] - a0 + halo;
        } else {
            row_oh[i] = -(1 << 20);
            row_ow[i] = -(1 << 20);
            row_px[i] = 0;
        }
    }
    // LDS byte addresses of the operand rows: the patch row under every tap (rows whose tap falls
    // outside the image use the zero area) and the weight rows, both at this lane's eight channels
    // of this K group's first 16-channel chunk.
    const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
    const uint32_t khalf = (lane >> 5) * 16 + kg * 32;
    uint32_t t_row[RS][TM];
#pragma unroll
    for (int tap = 0; tap < RS; ++tap) {
        const int dr = (tap / KR) * p.dil - p.pad_h, ds = (tap % KR) * p.dil - p.pad_w;
        const int shift = dr * p.W + ds;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const bool ok = (unsigned)(row_oh[i] + dr) < (unsigned)p.H && (unsigned)(row_ow[i] + ds) < (unsigned)p.W;
            const uint32_t at = lds0 + RS * WST + (uint32_t)((row_px[i] + shift) * pitch_b);
            t_row[tap][i] = (ok ? at : zero0 + (at & 255u)) + khalf;
        }
    }
    uint32_t b_rd[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) b_rd[j] = lds0 + (wn * WTN + j * 32 + (lane & 31)) * WP + khalf;

    floatx16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // ---- main loop: super-steps of 64 channels x all taps ----------------------------------------------
    // Inside a super-step nothing is loaded or synchronised: the group's k chunks (tap by tap, CPT
    // chunks of 16 channels per tap) follow one another with their operand reads D chunks ahead of
    // the MFMAs that use them, in register buffers of their own (as in dconv.h).
    constexpr int CPT = 4 / KW, NG = RS * CPT;
    constexpr int D0 = (TM + TN) * 3 <= 15 ? 3 : (TM + TN) * 2 <= 15 ? 2 : 1;
    constexpr int D = D0 < NG ? D0 : NG;
    constexpr int NBUF = 4;
    static_assert(D < NBUF, "look-ahead against the register buffers");
    u32x4_t af[NBUF][TM], bf[NBUF][TN];
    auto reads = [&](auto gc) {
        constexpr int g = decltype(gc)::value, tap = g / CPT, kc = g % CPT, buf = g % NBUF;
        static_for<TM>([&](auto ic) { lds_read16_async_at<kc * KW * 32>(af[buf][decltype(ic)::value], t_row[tap][decltype(ic)::value]); });
        static_for<TN>([&](auto jc) { lds_read16_async_at<tap * WST + kc * KW * 32>(bf[buf][decltype(jc)::value], b_rd[decltype(jc)::value]); });
    };
    for (int sb = 0; sb < nsb; ++sb) {
        static_for<D>([&](auto gc) { reads(gc); });
        static_for<NG>([&](auto gc) {
            constexpr int g = decltype(gc)::value, buf = g % NBUF;
            if constexpr (g + D < NG) reads(std::integral_constant<int, g + D>{});
            constexpr int ahead = g + D < NG ? D : NG - 1 - g;     // chunks read after this one and still in flight
            lds_wait<ahead * (TM + TN)>(af[buf], bf[buf]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, af[buf][i]),
                                                                        __builtin_bit_cast(bf16x8_t, bf[buf][j]), acc[i][j], 0, 0, 0);
        });
        if (sb + 1 < nsb) {
            __syncthreads();                               // every wave is done with this super-step's stages
            scatter_w();
            if (sb + 2 < nsb) load_w(sb + 2);
#pragma unroll
            for (int tap = 0; tap < RS; ++tap)
#pragma unroll
                for (int i = 0; i < TM; ++i) t_row[tap][i] += 128;             // the next 64 channels of every patch pixel
            __syncthreads();
        }
    }

    __syncthreads();
    float *stg = (float *)smem;
    if (p.flags & kPlanarOutNhwc) {
        // ---- output with the channels of a pixel contiguous (the consumer's layout: no conversion operator
        // between this layer and an NHWC one): [K group][pixel][channel] through LDS, then eight channels
        // (16 bytes of bf16, two 16-byte stores of fp32) per thread ----------------------------------------
        constexpr int SPN = BN + 4;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    stg[((size_t)kg * BM + wm * WTM + i * 32 + 8 * (e / 4) + 4 * (lane >> 5) + e % 4) * SPN + wn * WTN + j * 32 +
                        (lane & 31)] = acc[i][j][e];
        __syncthreads();
        constexpr int N8 = BN / 8;
        const bool relu = p.flags & ALT_EPI_RELU, bias = p.flags & ALT_EPI_BIAS, obf = p.flags & kDconvOutBf16;
        for (int idx = t; idx < BM * N8; idx += NT) {
            const int ml = idx / N8, nl = (idx % N8) * 8;
            const int m = m0 + ml, n = n0 + nl;
            if (m >= p.M || n >= p.Nc) continue;
            float v[8];
            {
                const float *sg = stg + (size_t)ml * SPN + nl;
                const float4 lo = *(const float4 *)sg, hi = *(const float4 *)(sg + 4);
                v[0] = lo.x; v[1] = lo.y; v[2] = lo.z; v[3] = lo.w; v[4] = hi.x; v[5] = hi.y; v[6] = hi.z; v[7] = hi.w;
            }
#pragma unroll
            for (int g = 1; g < KW; ++g) {
                const float *sg = stg + ((size_t)g * BM + ml) * SPN + nl;
                const float4 lo = *(const float4 *)sg, hi = *(const float4 *)(sg + 4);
                v[0] += lo.x; v[1] += lo.y; v[2] += lo.z; v[3] += lo.w; v[4] += hi.x; v[5] += hi.y; v[6] += hi.z; v[7] += hi.w;
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if (bias) v[e] += p.bias[n + e];
                if (relu) v[e] = fmaxf(v[e], 0.f);
            }
            const size_t off = (size_t)m * p.Nc + n;       // (Nc is a multiple of 8 and y is 16-byte aligned here)
            if (obf) {
                *(uint4 *)((uint16_t *)p.y + off) = make_uint4(f32x2_to_bf16x2(v[0], v[1]), f32x2_to_bf16x2(v[2], v[3]),
                                                               f32x2_to_bf16x2(v[4], v[5]), f32x2_to_bf16x2(v[6], v[7]));
            } else {
                *(float4 *)((float *)p.y + off) = make_float4(v[0], v[1], v[2], v[3]);
                *(float4 *)((float *)p.y + off + 4) = make_float4(v[4], v[5], v[6], v[7]);
            }
        }
        return;
    }
    // ---- output: [K group][channel][pixel] through LDS, then plane by plane ------------------------------
    constexpr int SPM = BM + 4;                            // staging pitch in floats
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
                *(float4 *)(stg + ((size_t)kg * BN + wn * WTN + j * 32 + (lane & 31)) * SPM + wm * WTM + i * 32 + 8 * q4 +
                            4 * (lane >> 5)) =
                    make_float4(acc[i][j][4 * q4], acc[i][j][4 * q4 + 1], acc[i][j][4 * q4 + 2], acc[i][j][4 * q4 + 3]);
    __syncthreads();
    // a thread takes eight consecutive pixels of one channel: one 16-byte store (two for fp32 output)
    // where they lie in one image, element by element where an image or the problem ends among them;
    // the wide stores are non-temporal (measured: 0.3-0.6 us off a 12 us layer against plain stores)
    constexpr int M8 = BM / 8;
    static_assert(NT % M8 == 0, "the output pass gives every thread one run of eight pixels");
    const int ml = (t % M8) * 8, m = m0 + ml;
    if (m < p.M) {
        const int img = (int)div32((uint32_t)m, p.d_hw), rem = m - img * ohw;
        const bool wide = m + 7 < p.M && rem + 7 < ohw;
        const bool relu = p.flags & ALT_EPI_RELU, bias = p.flags & ALT_EPI_BIAS, obf = p.flags & kDconvOutBf16;
        for (int nl = t / M8; nl < BN; nl += NT / M8) {
            const int n = n0 + nl;
            if (n >= p.Nc) break;
            float v[8];
            {
                const float4 lo = *(const float4 *)(stg + (size_t)nl * SPM + ml), hi = *(const float4 *)(stg + (size_t)nl * SPM + ml + 4);
                v[0] = lo.x; v[1] = lo.y; v[2] = lo.z; v[3] = lo.w; v[4] = hi.x; v[5] = hi.y; v[6] = hi.z; v[7] = hi.w;
            }
#pragma unroll
            for (int g = 1; g < KW; ++g) {
                const float *sg = stg + ((size_t)g * BN + nl) * SPM + ml;
                const float4 lo = *(const float4 *)sg, hi = *(const float4 *)(sg + 4);
                v[0] += lo.x; v[1] += lo.y; v[2] += lo.z; v[3] += lo.w; v[4] += hi.x; v[5] += hi.y; v[6] += hi.z; v[7] += hi.w;
            }
            const float bv = bias ? p.bias[n] : 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                v[e] += bv;
                if (relu) v[e] = fmaxf(v[e], 0.f);
            }
            if (wide) {
                const size_t off = (size_t)img * p.Nc * ohw + (size_t)n * ohw + rem;
                if (obf) {
                    PlanarRun r;
                    r.v.x = f32x2_to_bf16x2(v[0], v[1]); r.v.y = f32x2_to_bf16x2(v[2], v[3]);
                    r.v.z = f32x2_to_bf16x2(v[4], v[5]); r.v.w = f32x2_to_bf16x2(v[6], v[7]);
                    __builtin_nontemporal_store(r.v, &((PlanarRun *)((uint16_t *)p.y + off))->v);
                } else {
                    float *dst = (float *)p.y + off;
                    const f32x4_t lo = {v[0], v[1], v[2], v[3]}, hi = {v[4], v[5], v[6], v[7]};
                    __builtin_nontemporal_store(lo, &((PlanarRunF *)dst)->v);
                    __builtin_nontemporal_store(hi, &((PlanarRunF *)(dst + 4))->v);
                }
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int me = m + e;
                    if (me < p.M) {
                        const int ie = (int)div32((uint32_t)me, p.d_hw);
                        const size_t off = (size_t)ie * p.Nc * ohw + (size_t)n * ohw + (me - ie * ohw);
                        if (obf) ((uint16_t *)p.y)[off] = f32_to_bf16_rne(v[e]);
                        else ((float *)p.y)[off] = v[e];
                    }
                }
            }
        }
    }
}

template <int BM, int BN, int WGM, int WGN, int KW, int KR>
hipError_t dplanar_launch_kr(const DconvParams &p, size_t lds, hipStream_t st)
{
    auto kern = dplanar_kernel<BM, BN, WGM, WGN, KW, KR>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)(p.tiles_m * p.tiles_n)), dim3(64 * WGM * WGN * KW), lds, st, p);
    return hipGetLastError();
}

template <int BM, int BN, int WGM, int WGN, int KW>
hipError_t dplanar_launch(const DconvParams &p, size_t lds, hipStream_t st)
{
    if (p.R == 3 && p.S == 3) return dplanar_launch_kr<BM, BN, WGM, WGN, KW, 3>(p, lds, st);
    if (p.R == 1 && p.S == 1) return dplanar_launch_kr<BM, BN, WGM, WGN, KW, 1>(p, lds, st);
    return hipErrorInvalidValue;
}

}  // namespace alt

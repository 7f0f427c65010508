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
// Covers: bf16, stride 1, dilation 1, "same" padding (2*pad = R-1, S-1; so 1x1
// pad 0 too), activations NHWC, weights OHWI, output NHWC (fp32 or bf16), all
// dense, channels a multiple of 64 per split.  The linear pixel index of the
// input is then the linear index of the output pixel plus a per-tap constant,
// across image boundaries too, which is what makes the patch one contiguous
// range of input pixels.
//
// Split-K: grid slices over channel groups (Cs channels each) compute partial
// sums; each writes its fp32 partial tile to the workspace and the last slice
// to arrive (a counter per output tile) sums all slices in slice order and
// runs the epilogue, so the result does not depend on arrival order and no
// second kernel is launched.
#pragma once

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
    Div32 d_hw, d_w, d_tm, d_tn;  // divisions by H*W, W, tiles_m, tiles_n
    int32_t log2_cpp;             // log2(Cs / 8): 16-byte chunks per patch pixel
    int32_t swz_shift, swz_mask;  // patch swizzle: chunk position = chunk ^ ((pixel >> swz_shift) & swz_mask)
    int32_t ncc;                  // Cs / 64: K steps per tap
};

constexpr int kDconvOutBf16 = 4;
constexpr int kAgentScope = 16;          // cache-policy operand of buffer loads/stores: sc1 = device (agent) scope
constexpr int kDconvMaxTiles = 4096;     // output tiles a split-K launch may have (one counter each)
constexpr int kDconvSlots = 8;           // counter sets, handed to launches round-robin

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

template <int BM, int BN, int WGM, int WGN, int NS>
__global__ __launch_bounds__(64 * WGM * WGN) void dconv_kernel(const DconvParams p)
{
#ifdef ALT_PHASE_TIMING
    uint64_t stamps[5] = {0, 0, 0, 0, 0};
#endif
    ALT_STAMP(0);
    constexpr int NW = WGM * WGN;
    constexpr int WTM = BM / WGM, WTN = BN / WGN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int BK = 64, NKC = BK / 16;
    constexpr int B_STAGE = BN * BK * 2;                   // bytes of one weight stage: [BN][8 chunks of 16 B]
    constexpr int NLB = B_STAGE / 1024 / NW;               // wave-loads per wave per stage
    static_assert(WTM % 32 == 0 && WTN % 32 == 0 && TM >= 1 && TN >= 1, "wave tile");
    static_assert(B_STAGE % (1024 * NW) == 0 && NLB >= 1, "a weight stage is a whole number of wave-loads per wave");
    static_assert(NS >= 2 && (NS - 1) * NLB < 48, "pipeline depth against the vmcnt range");

    extern __shared__ uint4 smem_u4[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)smem_u4;    // weight stages first, then the patch
    const uint32_t patch0 = lds0 + NS * B_STAGE;

    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave / WGN, wn = wave % WGN;

    // workgroup -> (m tile, n tile, channel slice); consecutive logical ids share an XCD
    const int ntot = p.tiles_m * p.tiles_n * p.splitk;
    const int logical = igemm_logical_tile(ntot);
    const int rest = (int)div32((uint32_t)logical, p.d_tm);
    const int mt = logical - rest * p.tiles_m;
    const int split = (int)div32((uint32_t)rest, p.d_tn);
    const int nt = rest - split * p.tiles_n;
    const int m0 = mt * BM, n0 = nt * BN;

    const i32x4_t x_rsrc = make_rsrc(p.x, p.x_bytes);
    const i32x4_t w_rsrc = make_rsrc(p.w, p.w_bytes);

    // ---- the patch: input pixels [m0 - halo, m0 + BM + halo), Cs channels of this slice --------
    const int halo = p.pad_h * p.W + p.pad_w;
    const int np = BM + 2 * halo;
    const int log2_pitch = p.log2_cpp + 4;                 // bytes per patch pixel = Cs * 2
    const int nslots = np << p.log2_cpp;                   // 16-byte slots
    const int nwl = (nslots + 63) >> 6;                    // wave-loads (the region is padded to whole ones)
    const int pz = (nwl << 10) >> log2_pitch;              // index of the all-zero pixel row behind the patch
    {
        const int cmask = (1 << p.log2_cpp) - 1;
        const int g0 = m0 - halo;
        for (int j = wave; j < nwl; j += NW) {
            const int sidx = j * 64 + lane;
            const int px = sidx >> p.log2_cpp, cpos = sidx & cmask;
            const int q = cpos ^ ((px >> p.swz_shift) & p.swz_mask);
            const int g = g0 + px;
            const bool ok = sidx < nslots && (unsigned)g < (unsigned)p.M;
            const uint32_t voff = ok ? (uint32_t)(g * p.C + split * p.Cs + q * 8) * 2u : kOutOfRange;
            dma_load16(x_rsrc, voff, patch0 + j * 1024);
        }
        if (t < (1 << p.log2_cpp)) ((uint4 *)((char *)smem_u4 + NS * B_STAGE + (pz << log2_pitch)))[t] = make_uint4(0, 0, 0, 0);
    }

    // ---- weights: slot s = (i*NW + wave)*64 + lane of a stage holds chunk (s % 8) ^ swz(row) of row s / 8
    uint32_t b_voff[NLB];
    const int rsc = p.R * p.S * p.C;
#pragma unroll
    for (int i = 0; i < NLB; ++i) {
        const int s = (i * NW + wave) * 64 + lane;
        const int row = s >> 3, c = (s & 7) ^ ((row >> 1) & 7);
        const int n = n0 + row;
        b_voff[i] = n < p.Nc ? (uint32_t)(n * rsc + split * p.Cs + c * 8) * 2u : kOutOfRange;
    }
    const uint32_t ldsB = lds0 + wave * 1024;
    const int nsteps = p.R * p.S * p.ncc;
    // load cursor: byte offset of K step `lstep` inside a weight row, (tap, chunk) walked chunk fastest
    int lstep = 0, lcc = 0;
    uint32_t lsoff = 0;
    auto issue_b = [&]() {
        const int stage = lstep % NS;
#pragma unroll
        for (int i = 0; i < NLB; ++i) dma_load16_s(w_rsrc, b_voff[i], lsoff, ldsB + stage * B_STAGE + i * (NW * 1024));
        ++lstep;
        if (++lcc == p.ncc) { lcc = 0; lsoff += (uint32_t)(p.C - p.Cs) * 2u; }
        lsoff += BK * 2;
    };
#pragma unroll
    for (int s = 0; s < NS - 1; ++s)
        if (s < nsteps) issue_b();

    // ---- per-lane rows of the MFMA tiles ---------------------------------------------------------
    int32_t row_px[TM], row_oh[TM], row_ow[TM];
    const int hw = p.H * p.W;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int r = wm * WTM + i * 32 + (lane & 31);
        const int m = m0 + r;
        row_px[i] = r + halo;                              // patch pixel under the centre tap
        if (m < p.M) {
            const int img = (int)div32((uint32_t)m, p.d_hw), rem = m - img * hw;
            row_oh[i] = (int)div32((uint32_t)rem, p.d_w);
            row_ow[i] = rem - row_oh[i] * p.W;
        } else {
            row_oh[i] = -(1 << 20);
            row_ow[i] = -(1 << 20);
        }
    }
    // weight operand addresses inside a stage (byte offsets from lds0), per n tile and k chunk
    uint32_t b_rd[TN][NKC];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int r = wn * WTN + j * 32 + (lane & 31);
        const uint32_t swz = ((r >> 1) & 7) * 16;
#pragma unroll
        for (int kc = 0; kc < NKC; ++kc) b_rd[j][kc] = r * 128 + ((kc * 32 + (lane >> 5) * 16) ^ swz);
    }

    floatx16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const char *lds_base = (const char *)smem_u4;
    const char *patch_base = lds_base + NS * B_STAGE;
    const uint32_t khalf = (lane >> 5) * 16;

    ALT_STAMP(1);
    // ---- main loop: taps outer, 64-channel chunks inner; one barrier per K step ---------------------
    int step = 0;
    for (int r = 0; r < p.R; ++r) {
        for (int s = 0; s < p.S; ++s) {
            const int shift = (r - p.pad_h) * p.W + (s - p.pad_w);
            uint32_t a_row[TM], a_swz[TM];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const bool ok = (unsigned)(row_oh[i] + r - p.pad_h) < (unsigned)p.H &&
                                (unsigned)(row_ow[i] + s - p.pad_w) < (unsigned)p.W;
                const int px = ok ? row_px[i] + shift : pz;
                a_row[i] = (uint32_t)px << log2_pitch;
                a_swz[i] = (uint32_t)((px >> p.swz_shift) & p.swz_mask) << 4;
            }
            for (int cc = 0; cc < p.ncc; ++cc, ++step) {
                if (step + NS - 2 < nsteps) wait_vmcnt<(NS - 2) * NLB>();
                else wait_vmcnt<0>();
                lds_barrier();                 // step's weights (and at step 0 the patch) are in LDS; step-1 is consumed
#ifdef ALT_PHASE_TIMING
                if (step == 0) ALT_STAMP(2);
#endif
                if (lstep < nsteps) issue_b();
                const uint32_t st_off = (uint32_t)(step % NS) * B_STAGE;
                const uint32_t c_off = (uint32_t)cc * (BK * 2) + khalf;
                uint4 af[2][TM], bf[2][TN];
#pragma unroll
                for (int i = 0; i < TM; ++i) af[0][i] = *(const uint4 *)(patch_base + a_row[i] + (c_off ^ a_swz[i]));
#pragma unroll
                for (int j = 0; j < TN; ++j) bf[0][j] = *(const uint4 *)(lds_base + st_off + b_rd[j][0]);
#pragma unroll
                for (int kc = 0; kc < NKC; ++kc) {
                    if (kc + 1 < NKC) {
#pragma unroll
                        for (int i = 0; i < TM; ++i)
                            af[(kc + 1) & 1][i] = *(const uint4 *)(patch_base + a_row[i] + ((c_off + (kc + 1) * 32) ^ a_swz[i]));
#pragma unroll
                        for (int j = 0; j < TN; ++j)
                            bf[(kc + 1) & 1][j] = *(const uint4 *)(lds_base + st_off + b_rd[j][kc + 1 < NKC ? kc + 1 : 0]);
                    }
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int j = 0; j < TN; ++j) mma_tile(acc[i][j], af[kc & 1][i], bf[kc & 1][j], bf16_tag{});
                }
            }
        }
    }

    ALT_STAMP(3);
    // ---- split-K: publish the partial tile; the last slice to arrive sums all slices ------------------
    const int tile = mt * p.tiles_n + nt;
    if (p.splitk > 1) {
        const __amdgpu_buffer_rsrc_t pr = __builtin_amdgcn_make_buffer_rsrc(
            (void *)((char *)p.partial + (size_t)split * p.partial_bytes), 0, (int)p.partial_bytes, 0x00020000);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int n = n0 + wn * WTN + j * 32 + (lane & 31);
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int m = m0 + wm * WTM + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                    const uint32_t off = (m < p.M && n < p.Nc) ? (uint32_t)(m * p.Nc + n) * 4u : kOutOfRange;
                    const float v = acc[i][j][e];
                    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, v), pr, (int)off, 0, kAgentScope);
                }
            }
        // The partial sums were stored with device (agent) scope, i.e. written through to
        // memory all XCDs share; once the stores are acknowledged they are visible to
        // device-scope loads anywhere.  That is the release half; a full device-scope
        // fence would write back the whole L2 and costs tens of microseconds here.
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        uint32_t *flag = (uint32_t *)smem_u4;  // the weight stages are free now
        if (t == 0) {
            const uint32_t old = __hip_atomic_fetch_add(p.counters + tile, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            *flag = old == (uint32_t)(p.splitk - 1);
            if (*flag) __hip_atomic_store(p.counters + tile, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next launch
        }
        __syncthreads();
        if (*flag == 0) return;
        // acquire half: the loads below have device scope and so do not hit stale cache lines
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
        for (int sl = 0; sl < p.splitk; ++sl) {
            const __amdgpu_buffer_rsrc_t sr = __builtin_amdgcn_make_buffer_rsrc(
                (void *)((char *)p.partial + (size_t)sl * p.partial_bytes), 0, (int)p.partial_bytes, 0x00020000);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int n = n0 + wn * WTN + j * 32 + (lane & 31);
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int m = m0 + wm * WTM + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                        const uint32_t off = (m < p.M && n < p.Nc) ? (uint32_t)(m * p.Nc + n) * 4u : kOutOfRange;
                        const uint32_t bits = __builtin_amdgcn_raw_buffer_load_b32(sr, (int)off, 0, kAgentScope);
                        acc[i][j][e] += __builtin_bit_cast(float, bits);
                    }
                }
        }
    }

    // ---- epilogue: bias, ReLU, rounding, NHWC store ---------------------------------------------------------
    const __amdgpu_buffer_rsrc_t yr = __builtin_amdgcn_make_buffer_rsrc(p.y, 0, (int)p.y_bytes, 0x00020000);
    const float relu_floor = (p.flags & ALT_EPI_RELU) ? 0.f : -INFINITY;
    const bool out_bf16 = p.flags & kDconvOutBf16;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = n0 + wn * WTN + j * 32 + (lane & 31);
        const bool n_ok = n < p.Nc;
        const float bv = (n_ok && (p.flags & ALT_EPI_BIAS)) ? p.bias[n] : 0.f;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int m = m0 + wm * WTM + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                const uint32_t idx = (uint32_t)(m * p.Nc + n);
                const bool ok = n_ok && m < p.M;
                const float v = fmaxf(acc[i][j][e] + bv, relu_floor);
                if (out_bf16)
                    __builtin_amdgcn_raw_buffer_store_b16(f32_to_bf16_rne(v), yr, (int)(ok ? idx * 2u : kOutOfRange), 0, 0);
                else
                    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, v), yr, (int)(ok ? idx * 4u : kOutOfRange), 0, 0);
            }
    }
#ifdef ALT_PHASE_TIMING
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    ALT_STAMP(4);
    if (threadIdx.x == 0 && p.partial && p.splitk == 1) {
        uint64_t *out = (uint64_t *)p.partial + (size_t)blockIdx.x * 8;
        for (int i = 0; i < 5; ++i) out[i] = stamps[i];
        out[5] = __builtin_amdgcn_s_getreg(GETREG_IMMED(31, 0, 4));    // HW_ID
        out[6] = __builtin_amdgcn_s_getreg(GETREG_IMMED(3, 0, 20));    // XCC_ID
    }
#endif
}

// LDS bytes of one workgroup: weight stages, the patch rounded up to whole
// wave-loads, the all-zero row.
inline size_t dconv_lds_bytes(int BM, int BN, int NS, int Cs, int W, int pad_h, int pad_w)
{
    const size_t pitch = (size_t)Cs * 2;
    const size_t np = (size_t)BM + 2 * ((size_t)pad_h * W + pad_w);
    const size_t patch = (np * pitch + 1023) / 1024 * 1024;
    return (size_t)NS * BN * 128 + patch + pitch;
}

template <int BM, int BN, int WGM, int WGN, int NS>
hipError_t dconv_launch(const DconvParams &p, size_t lds, hipStream_t st)
{
    auto kern = dconv_kernel<BM, BN, WGM, WGN, NS>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)(p.tiles_m * p.tiles_n * p.splitk)), dim3(64 * WGM * WGN), lds, st, p);
    return hipGetLastError();
}

struct DconvLaunch {
    const char *name;
    int BM, BN, NS, waves;
    hipError_t (*launch)(const DconvParams &p, size_t lds, hipStream_t st);
};

}  // namespace alt

// Implicit-GEMM kernel whose operand tiles go from global memory straight into
// LDS (buffer loads with the LDS bit), NS stages deep.
//
// Same tiling and MFMA mapping as igemm.h; what differs is the pipeline.  A
// wave-wide 16-byte buffer load with the LDS bit writes the 64 lanes' data to
// 1 KB of consecutive LDS starting at the address in M0, without passing
// through VGPRs, so a stage costs no registers and no ds_write, and NS - 1
// K steps of loads stay in flight while the MFMAs of the current step run.
// Because the destination of a wave-load is contiguous, rows cannot be padded;
// bank conflicts of the 16-byte MFMA operand reads are avoided by an XOR
// swizzle instead: 16-byte chunk c of tile row r is stored at chunk position
// c ^ swz(r), and since every lane picks its own global address, the loader
// simply fetches, for LDS slot s, the chunk that belongs there.  Padding taps
// and rows outside the tile use an offset beyond the buffer descriptor's size,
// for which the hardware writes zeros.
//
// The loads are issued from inline assembly, and completion is waited for with
// explicit s_waitcnt vmcnt(n): the compiler's own bookkeeping of LDS-bound
// loads waits for the newest one before any LDS read, which would serialise
// the pipeline.  Only for layouts both of whose operands are contiguous along
// the reduction channel in 16-byte blocks (the "vv" case of igemm.h).
#pragma once

#include "igemm.h"

namespace alt {

struct KEntry32 {             // per K step, byte-offset arithmetic in 32 bits (operands < 2 GiB)
    int32_t a_off, b_off;     // element offsets added to every row base
    int32_t dh, dw;
};

typedef int i32x4_t __attribute__((ext_vector_type(4)));

// One wave-wide 16-byte-per-lane load into LDS at byte address `lds` (+ 16 * lane);
// `lds` must be wave-uniform (it is moved to M0).
__device__ __forceinline__ void dma_load16(i32x4_t rsrc, uint32_t voff, uint32_t lds)
{
    // (the compiler drops the readfirstlane where it already knows the value to be scalar)
    const uint32_t lds_s = __builtin_amdgcn_readfirstlane(lds);
    asm volatile("s_mov_b32 m0, %0\n\t"
                 "s_nop 0\n\t"
                 "buffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(lds_s), "v"(voff), "s"(rsrc)
                 : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

__device__ __forceinline__ i32x4_t make_rsrc(const void *base, uint32_t bytes)
{
    const uint64_t a = (uint64_t)base;
    i32x4_t r;
    r.x = __builtin_amdgcn_readfirstlane((int)(uint32_t)a);
    r.y = __builtin_amdgcn_readfirstlane((int)(uint32_t)(a >> 32) & 0xffff);   // stride 0
    r.z = __builtin_amdgcn_readfirstlane((int)bytes);
    r.w = 0x00020000;                                                           // 32-bit data format
    return r;
}

template <typename T, int BM, int BN, int BK, int WGM, int WGN, int NS>
__global__ __launch_bounds__(64 * WGM * WGN) void igemm_dma_kernel(const IgemmParams p)
{
    using TR = ElemTraits<T>;
    constexpr int EPV = TR::EPV;
    constexpr int ES = TR::SIZE;
    constexpr int NW = WGM * WGN;                          // wavefronts per workgroup (4 or 8)
    constexpr int NT = 64 * NW;
    constexpr int WTM = BM / WGM, WTN = BN / WGN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int KC = 2 * EPV;
    constexpr int NKC = BK / KC;                           // MFMA k-chunks per step
    constexpr int CPR = BK / EPV;                          // 16-byte chunks per tile row
    constexpr int SWZ_DIV = CPR >= 16 ? 1 : 16 / CPR;      // rows that share one swizzle value
    constexpr int A_STAGE = BM * BK * ES, B_STAGE = BN * BK * ES;      // bytes
    constexpr int NLA = A_STAGE / 1024 / NW, NLB = B_STAGE / 1024 / NW;  // wave-loads per wave per stage
    constexpr int LPS = NLA + NLB;
    constexpr int LPK = (LPS + NKC - 1) / NKC;             // wave-loads issued per k-chunk
    static_assert((NW == 4 || NW == 8 || NW == 16) && WTM % 32 == 0 && WTN % 32 == 0 && BK % KC == 0, "tile shape");
    static_assert(A_STAGE % (1024 * NW) == 0 && B_STAGE % (1024 * NW) == 0, "a stage is a whole number of wave-loads per wave");
    static_assert(NS >= 2 && (NS - 2) * LPS < 64, "pipeline depth against the vmcnt range");
    static_assert(CPR >= 2 && (CPR & (CPR - 1)) == 0 && CPR <= 16, "chunks per row");

    extern __shared__ uint4 smem_u4[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)smem_u4;
    KEntry32 *ktab = (KEntry32 *)((char *)smem_u4 + NS * (A_STAGE + B_STAGE));

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);          // scalar: LDS destinations stay in SGPRs
    const int wm = wave / WGN, wn = wave % WGN;
    const int logical = igemm_logical_tile(p.tiles_m * p.tiles_n);
    const int nt = logical % p.tiles_n, mt = logical / p.tiles_n;
    const int m0 = mt * BM, n0 = nt * BN;
    const int split = blockIdx.y % p.splitk, bz = blockIdx.y / p.splitk;
    const int kbeg = split * p.ksteps_per_split;
    const int nk = min(p.ksteps_per_split, p.ksteps_total - kbeg);

    const i32x4_t x_rsrc = make_rsrc((const char *)p.x + (int64_t)bz * p.x_bstride * ES, p.x_bytes);
    const i32x4_t w_rsrc = make_rsrc((const char *)p.w + (int64_t)bz * p.w_bstride * ES, p.w_bytes);
    // LDS byte addresses of this wave's first wave-load of stage 0
    const uint32_t ldsA = lds0 + wave * 1024, ldsB = lds0 + NS * A_STAGE + wave * 1024;

    // ---- what each lane fetches: LDS slot s = (i*NW + wave)*64 + lane holds chunk
    // (s % CPR) ^ swz(row) of tile row s / CPR
    int32_t a_base[NLA], a_ih0[NLA], a_iw0[NLA];
    int32_t b_base[NLB];
    const int ohow = p.OH * p.OW;
#pragma unroll
    for (int i = 0; i < NLA; ++i) {
        const int s = (i * NW + wave) * 64 + lane;
        const int row = s / CPR, c = (s % CPR) ^ ((row / SWZ_DIV) % CPR);
        const int m = m0 + row;
        if (m < p.M) {
            const int img = (int)fast_div(m, p.fd_ohow), rem = m - img * ohow;
            const int oh = (int)fast_div(rem, p.fd_ow), ow = rem - oh * p.OW;
            a_ih0[i] = oh * p.stride_h - p.pad_h;
            a_iw0[i] = ow * p.stride_w - p.pad_w;
            int32_t base = dim2_off32(p.xn, img) + dim2_off32(p.xc, c * EPV);
            if (p.spatial_split) base += dim2_off32(p.xh, a_ih0[i]) + dim2_off32(p.xw, a_iw0[i]);
            else base += a_ih0[i] * (int32_t)p.xh.si + a_iw0[i] * (int32_t)p.xw.si;
            a_base[i] = base;
        } else {
            a_ih0[i] = -(1 << 28); a_iw0[i] = -(1 << 28); a_base[i] = 0;
        }
    }
#pragma unroll
    for (int i = 0; i < NLB; ++i) {
        const int s = (i * NW + wave) * 64 + lane;
        const int row = s / CPR, c = (s % CPR) ^ ((row / SWZ_DIV) % CPR);
        const int n = n0 + row;
        b_base[i] = n < p.Nc ? dim2_off32(p.wo, n) + dim2_off32(p.wi, c * EPV) : -1;
    }

    auto fill_ktab = [&](int first) {
        for (int j = t; j < kKTab && first + j < nk; j += NT) {
            const int k0 = (kbeg + first + j) * BK;
            const int rs = (int)fast_div(k0, p.fd_c), c0 = k0 - rs * p.C;
            const int r = (int)fast_div(rs, p.fd_s), s = rs - r * p.S;
            KEntry32 e;
            e.dh = r * p.dil_h;
            e.dw = s * p.dil_w;
            e.a_off = e.dh * (int32_t)p.xh.si + e.dw * (int32_t)p.xw.si + dim2_off32(p.xc, c0);
            e.b_off = dim2_off32(p.wr, r) + dim2_off32(p.ws, s) + dim2_off32(p.wi, c0);
            ktab[j] = e;
        }
    };

    // Issues wave-loads [first, last) of the K step described by table entry e into stage
    // `stage`; loads 0..NLA-1 are the A tile, NLA..LPS-1 the B tile.
    auto issue = [&](const KEntry32 &e, int stage, int first, int last) {
#pragma unroll
        for (int l = 0; l < LPS; ++l) {
            if (l < first || l >= last) continue;
            if (l < NLA) {
                const int i = l;
                const bool ok = (unsigned)(a_ih0[i] + e.dh) < (unsigned)p.H && (unsigned)(a_iw0[i] + e.dw) < (unsigned)p.W;
                const uint32_t voff = ok ? (uint32_t)(a_base[i] + e.a_off) * ES : kOutOfRange;
                dma_load16(x_rsrc, voff, ldsA + stage * A_STAGE + i * (NW * 1024));
            } else {
                const int i = l - NLA;
                const uint32_t voff = b_base[i] >= 0 ? (uint32_t)(b_base[i] + e.b_off) * ES : kOutOfRange;
                dma_load16(w_rsrc, voff, ldsB + stage * B_STAGE + i * (NW * 1024));
            }
        }
    };

    floatx16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // operand read addresses inside a stage, per 32-row MFMA tile and k-chunk (loop
    // invariant; the stage offset is a compile-time addend of the unrolled step)
    const char *a_rd[TM][NKC], *b_rd[TN][NKC];
    {
        const uint32_t khalf = (lane >> 5) * 16;
        const char *lds_base = (const char *)smem_u4;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int r = wm * WTM + i * 32 + (lane & 31);
            const uint32_t swz = ((r / SWZ_DIV) % CPR) * 16;
#pragma unroll
            for (int kc = 0; kc < NKC; ++kc) a_rd[i][kc] = lds_base + r * (CPR * 16) + ((kc * 32 + khalf) ^ swz);
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int r = wn * WTN + j * 32 + (lane & 31);
            const uint32_t swz = ((r / SWZ_DIV) % CPR) * 16;
#pragma unroll
            for (int kc = 0; kc < NKC; ++kc) b_rd[j][kc] = lds_base + NS * A_STAGE + r * (CPR * 16) + ((kc * 32 + khalf) ^ swz);
        }
    }

    if (nk > 0) {
        fill_ktab(0);
        lds_barrier();
#pragma unroll
        for (int s = 0; s < NS - 1; ++s)
            if (s < nk) issue(ktab[s], s, 0, LPS);
        // One K step; `st`, the stage of step ks, is a compile-time constant at every call site.
        auto do_step = [&](int ks, int st) {
            // step ks has landed once at most the loads of the later steps in flight remain
            if (ks + NS - 2 < nk) wait_vmcnt<(NS - 2) * LPS>();
            else wait_vmcnt<0>();
            lds_barrier();                             // everyone's part of step ks is in LDS; step ks-1 is consumed
            const int nf = ks + NS - 1;
            const bool more = nf < nk;
            if (more && nf % kKTab == 0) {             // next window of the K-step table
                fill_ktab(nf);
                lds_barrier();
            }
            const KEntry32 e = ktab[(more ? nf : ks) % kKTab];
            const int fstage = (st + NS - 1) % NS;
            // operand fragments one k-chunk ahead of the MFMAs that use them, and the
            // next stage's loads spread between the MFMA groups, so that a wavefront
            // alone on its SIMD still overlaps LDS reads, load issue and matrix math
            uint4 af[2][TM], bf[2][TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) af[0][i] = *(const uint4 *)(a_rd[i][0] + st * A_STAGE);
#pragma unroll
            for (int j = 0; j < TN; ++j) bf[0][j] = *(const uint4 *)(b_rd[j][0] + st * B_STAGE);
#pragma unroll
            for (int kc = 0; kc < NKC; ++kc) {
                if (kc + 1 < NKC) {
#pragma unroll
                    for (int i = 0; i < TM; ++i) af[(kc + 1) & 1][i] = *(const uint4 *)(a_rd[i][kc + 1 < NKC ? kc + 1 : 0] + st * A_STAGE);
#pragma unroll
                    for (int j = 0; j < TN; ++j) bf[(kc + 1) & 1][j] = *(const uint4 *)(b_rd[j][kc + 1 < NKC ? kc + 1 : 0] + st * B_STAGE);
                }
                if (more) issue(e, fstage, kc * LPK, (kc + 1) * LPK);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) mma_tile(acc[i][j], af[kc & 1][i], bf[kc & 1][j], T{});
            }
        };
        int ks0 = 0;
        for (; ks0 + NS <= nk; ks0 += NS) {            // whole rounds over the stages, no exit inside
#pragma unroll
            for (int st = 0; st < NS; ++st) do_step(ks0 + st, st);
        }
#pragma unroll
        for (int st = 0; st < NS - 1; ++st)            // the last, partial round
            if (ks0 + st < nk) do_step(ks0 + st, st);
        lds_barrier();                                 // last reads done before the stages are reused
    }
    igemm_epilogue<BM, TM, TN, WTM, WTN, NT>(p, acc, (void *)smem_u4, m0, n0, wm, wn, split, bz);
}

template <typename T, int BM, int BN, int BK, int NS>
constexpr size_t igemm_dma_lds_bytes()
{
    return (size_t)NS * (BM + BN) * BK * ElemTraits<T>::SIZE + kKTab * sizeof(KEntry32);
}

template <typename T, int BM, int BN, int BK, int WGM, int WGN, int NS>
hipError_t igemm_dma_launch(const IgemmParams &p, dim3 grid, hipStream_t st)
{
    constexpr int NT = 64 * WGM * WGN;
    constexpr size_t lds = igemm_dma_lds_bytes<T, BM, BN, BK, NS>();
    static_assert(lds <= 160 * 1024, "LDS per workgroup");
    auto kern = igemm_dma_kernel<T, BM, BN, BK, WGM, WGN, NS>;
    static bool attr_set = false;
    if (!attr_set && lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, grid, dim3(NT), lds, st, p);
    return hipGetLastError();
}

}  // namespace alt

// Implicit-GEMM kernel for C2D and GMM on gfx950 matrix cores.
//
// The output is an M x Nc matrix (M = N*OH*OW output pixels or GMM rows,
// Nc = output channels or GMM columns) reduced over Kg = R*S*C (GMM: K),
// walked in the order (r, s, c) with c fastest.  One workgroup of 256 threads
// (4 wavefronts of 64) owns a BM x BN output tile; each K step stages a
// BM x BK slice of the "A" operand (activations) and a BN x BK slice of the
// "B" operand (weights) in LDS, both stored [row][k] with k contiguous,
// because every 32x32 MFMA lane consumes 8 (bf16) or 4 (fp32) consecutive k
// of one row.  LDS rows are padded by 16 bytes so that the 16-byte operand
// reads of a wavefront fall on distinct banks.  Global loads run PF steps
// ahead of the MFMAs: the loads of step t+PF are issued before the MFMAs of
// step t into a register slot of their own, and the registers of step t+1 go
// to the other LDS stage after them (register prefetch of depth PF + LDS double
// buffering, one barrier per step).  With few workgroups per CU the load
// latency is what a step costs, so PF > 1 is what keeps the matrix cores fed.
//
// How an operand tile is fetched depends on its layout (the point of the
// paper: the loop nest follows the layout):
//   LOAD_VEC    – the reduction channel is the memory-contiguous dimension in
//                 blocks of >= 8/4 elements (NHWC, NCHW[x]c, OHWI,
//                 OIHW[y]o[x]i, row-major A, "NK" B): 16-byte loads.
//   LOAD_GATHER – any other two-level layout (NCHW, OIHW, ...): one element
//                 per load, lanes walk the rows of the tile.
//   LOAD_TRANS  – rows are memory-contiguous and k is strided (row-major B
//                 "KN", A stored "KM"): 16-byte loads along the rows and an
//                 8x8 (4x4 for fp32) transpose in registers.
#pragma once

#include "common.h"

namespace alt {

enum { LOAD_VEC = 0, LOAD_GATHER = 1, LOAD_TRANS = 2 };

struct IgemmParams {
    const void *x;            // A operand (activations / GMM A)
    const void *w;            // B operand (weights / GMM B)
    const float *bias;
    void *y;
    float *partial;           // split-K partial sums [split][batch][M][Nc]
    int32_t M, Nc, Kg;        // per batch entry
    int32_t C, H, W, R, S, OH, OW;
    int32_t stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
    int32_t batch, splitk, ksteps_per_split, ksteps_total;
    int32_t tiles_m, tiles_n;
    int32_t epilogue, out_bf16;
    int32_t uniform_rs;       // C % BK == 0: one (r, s) per K step
    int32_t spatial_split;    // H or W of x is blocked (only with R = S = 1, no padding)
    int64_t x_bstride, w_bstride, y_bstride;
    uint32_t x_bytes, w_bytes;   // size of one batch entry of each operand (vector loaders: < 2 GiB)
    uint32_t y_bytes;            // size of one batch entry of the output, 0 if it does not fit 31 bits
    int32_t bias_bstride;        // elements between the bias vectors of consecutive batch entries (groups)
    FastDiv fd_ohow, fd_ow, fd_c, fd_s, fd_nc;   // divisions by OH*OW, OW, C, S, Nc
    Dim2 xn, xc, xh, xw;      // activations (N, C, H, W)
    Dim2 wo, wi, wr, ws;      // weights (O, I, R, S)
    Dim2 yn, yk, yh, yw;      // output (N, K, OH, OW)
    const void *addend;       // tensor added before the activation (same layout and type as y), or null
};

struct KEntry {               // one K step: what is uniform over the tile
    int64_t a_off, b_off;     // element offsets added to every row base
    int32_t dh, dw;           // r*dil_h, s*dil_w
};

constexpr int kIgemmThreads = 256;
constexpr int kKTab = 256;    // K steps whose KEntry is kept in LDS at a time

// Offset of index i (0 <= i < extent) of one logical dimension.
__device__ __forceinline__ int64_t dim2_off(const Dim2 &d, int32_t i)
{
    const int32_t q = (int32_t)fast_div((uint32_t)i, d.fd);
    return (int64_t)q * d.so + (int64_t)(i - q * d.f) * d.si;
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also
// carries a workgroup-scope release fence, which drains every outstanding
// global load (s_waitcnt vmcnt(0)) and so would cancel the register prefetch;
// here only this wave's LDS operations are waited for before the barrier.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// 16-byte load through a buffer descriptor: an offset at or beyond the
// descriptor's size returns zeros, which is how padding taps and rows outside
// the tile are filled without a branch or a select on the loaded data.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
constexpr uint32_t kOutOfRange = 0x80000000u;
__device__ __forceinline__ uint4 buffer_load16(__amdgpu_buffer_rsrc_t rsrc, uint32_t byte_off)
{
    u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)byte_off, 0, 0);
    return make_uint4(v.x, v.y, v.z, v.w);
}

// Same in 32 bits, for tensors known to be smaller than 2^31 elements.
__device__ __forceinline__ int32_t dim2_off32(const Dim2 &d, int32_t i)
{
    const int32_t q = (int32_t)fast_div((uint32_t)i, d.fd);
    return q * (int32_t)d.so + (i - q * d.f) * (int32_t)d.si;
}

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx16_t __attribute__((ext_vector_type(16)));

struct bf16_tag {};

template <typename T> struct ElemTraits;
template <> struct ElemTraits<bf16_tag> {
    using store_t = uint16_t;
    static constexpr int EPV = 8;        // elements per 16-byte vector
    static constexpr int SIZE = 2;
};
template <> struct ElemTraits<float> {
    using store_t = float;
    static constexpr int EPV = 4;
    static constexpr int SIZE = 4;
};

// One 16-byte operand fragment pair -> 32x32 accumulator.  Lane l holds row
// l%32 and the k group l/32 of both operands; accumulator register i of lane l
// is element (8*(i/4) + 4*(l/32) + i%4, l%32).
__device__ __forceinline__ void mma_tile(floatx16_t &acc, const uint4 &a, const uint4 &b, bf16_tag)
{
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                  __builtin_bit_cast(bf16x8_t, b), acc, 0, 0, 0);
}
__device__ __forceinline__ void mma_tile(floatx16_t &acc, const uint4 &a, const uint4 &b, float)
{
    const float *fa = (const float *)&a, *fb = (const float *)&b;
#pragma unroll
    for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[j], fb[j], acc, 0, 0, 0);
}

// fp32 -> bf16, round to nearest even, NaN kept quiet; selects instead of a branch.
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    const uint32_t w = __builtin_bit_cast(uint32_t, f);
    const uint32_t rounded = (w + 0x7fffu + ((w >> 16) & 1u)) >> 16;
    const uint32_t quiet = (w >> 16) | 0x40u;
    return (uint16_t)(((w & 0x7fffffffu) > 0x7f800000u) ? quiet : rounded);
}

// Two fp32 -> bf16 conversions (round to nearest even, NaN kept quiet) packed into one
// dword, lo in the low half: one hardware conversion instruction on gfx950.
__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float lo, float hi)
{
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// 8x8 transpose of 16-bit elements held as 8 uint4 rows (in place).
__device__ __forceinline__ void transpose8x8_b16(uint4 *r)
{
    uint32_t in[8][4], out[8][4];
#pragma unroll
    for (int i = 0; i < 8; ++i) { in[i][0] = r[i].x; in[i][1] = r[i].y; in[i][2] = r[i].z; in[i][3] = r[i].w; }
#pragma unroll
    for (int n = 0; n < 8; ++n)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t lo = in[2 * j][n / 2], hi = in[2 * j + 1][n / 2];
            out[n][j] = (n & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u)    // high halves
                                : __builtin_amdgcn_perm(hi, lo, 0x05040100u);   // low halves
        }
#pragma unroll
    for (int i = 0; i < 8; ++i) r[i] = make_uint4(out[i][0], out[i][1], out[i][2], out[i][3]);
}

__device__ __forceinline__ void transpose4x4_b32(uint4 *r)
{
    uint32_t in[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i) { in[i][0] = r[i].x; in[i][1] = r[i].y; in[i][2] = r[i].z; in[i][3] = r[i].w; }
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = make_uint4(in[0][i], in[1][i], in[2][i], in[3][i]);
}

// Writes one workgroup's accumulators: to y under its layout with bias, ReLU
// and the output conversion fused (the consumer's layout is written directly),
// or to the split-K partial-sum buffer.  Row offsets of the tile go through
// LDS (`scratch`, BM entries of 8 bytes; the operand stages are free by now);
// the column offset is per lane.  All waves must have passed their last LDS
// read.  When the destination spans less than 2 GiB the stores go through a
// buffer descriptor with 32-bit offsets and rows/columns outside the problem
// get an out-of-range offset, which the hardware drops: no branch per element.
template <int BM, int TM, int TN, int WTM, int WTN, int NT = kIgemmThreads>
__device__ __forceinline__ void igemm_epilogue(const IgemmParams &p, floatx16_t (&acc)[TM][TN], void *scratch,
                                               int m0, int n0, int wm, int wn, int split, int bz)
{
    const int t = threadIdx.x, lane = t & 63;
    const int ohow = p.OH * p.OW;
    const bool to_partial = p.splitk > 1;
    const bool narrow = to_partial || p.y_bytes != 0;
    if (narrow) {
        int32_t *rowoff = (int32_t *)scratch;
        for (int r = t; r < BM; r += NT) {
            const int m = m0 + r;
            int32_t off = -1;                              // row outside M
            if (m < p.M) {
                if (to_partial) {
                    off = m * p.Nc;
                } else {
                    const int img = (int)fast_div(m, p.fd_ohow), rem = m - img * ohow;
                    const int oh = (int)fast_div(rem, p.fd_ow), ow = rem - oh * p.OW;
                    off = dim2_off32(p.yn, img) + dim2_off32(p.yh, oh) + dim2_off32(p.yw, ow);
                }
            }
            rowoff[r] = off;
        }
        lds_barrier();
        const int esz = to_partial ? 4 : (p.out_bf16 ? 2 : 4);
        const char *dst = to_partial
            ? (const char *)(p.partial + ((int64_t)split * p.batch + bz) * (int64_t)p.M * p.Nc)
            : (const char *)p.y + (int64_t)bz * p.y_bstride * esz;
        const uint32_t dst_bytes = to_partial ? (uint32_t)p.M * p.Nc * 4u : p.y_bytes;
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)dst, 0, (int)dst_bytes, 0x00020000);
        // the 16 rows of a 32x32 accumulator tile a lane holds: 4 groups of 4 consecutive rows
        int32_t ro[TM][16];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int4 v = *(const int4 *)(rowoff + wm * WTM + i * 32 + 8 * g + 4 * (lane >> 5));
                ro[i][4 * g + 0] = v.x; ro[i][4 * g + 1] = v.y; ro[i][4 * g + 2] = v.z; ro[i][4 * g + 3] = v.w;
            }
        // straight-line store loops (no branch per element, so the compiler's
        // wait-count bookkeeping never makes a store wait for the one before it)
        const float relu_floor = (p.epilogue & ALT_EPI_RELU) ? 0.f : -INFINITY;
        const int mode = to_partial ? 0 : (p.out_bf16 ? 2 : 1);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = n0 + wn * WTN + j * 32 + (lane & 31);
            const bool n_ok = n < p.Nc;
            const int32_t coff = n_ok ? (to_partial ? n : dim2_off32(p.yk, n)) : 0;
            const float bv = (n_ok && !to_partial && (p.epilogue & ALT_EPI_BIAS)) ? p.bias[bz * p.bias_bstride + n] : 0.f;
            uint32_t voff[TM][16];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    voff[i][e] = (n_ok && ro[i][e] >= 0) ? (uint32_t)(ro[i][e] + coff) * (uint32_t)esz : kOutOfRange;
            if (mode == 0) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const float v = acc[i][j][e];      // (a vector element is not a bit_cast operand)
                        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, v), rsrc, (int)voff[i][e], 0, 0);
                    }
            } else if (mode == 1) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const float v = fmaxf(acc[i][j][e] + bv, relu_floor);
                        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, v), rsrc, (int)voff[i][e], 0, 0);
                    }
            } else {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const float v = fmaxf(acc[i][j][e] + bv, relu_floor);
                        __builtin_amdgcn_raw_buffer_store_b16(f32_to_bf16_rne(v), rsrc, (int)voff[i][e], 0, 0);
                    }
            }
        }
        return;
    }
    // outputs of 2 GiB and more: 64-bit addresses, one guarded store per element
    int64_t *rowoff = (int64_t *)scratch;
    for (int r = t; r < BM; r += NT) {
        const int m = m0 + r;
        int64_t off = -1;
        if (m < p.M) {
            const int img = (int)fast_div(m, p.fd_ohow), rem = m - img * ohow;
            const int oh = (int)fast_div(rem, p.fd_ow), ow = rem - oh * p.OW;
            off = dim2_off(p.yn, img) + dim2_off(p.yh, oh) + dim2_off(p.yw, ow);
        }
        rowoff[r] = off;
    }
    lds_barrier();
    char *yb = (char *)p.y + (int64_t)bz * p.y_bstride * (p.out_bf16 ? 2 : 4);
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = n0 + wn * WTN + j * 32 + (lane & 31);
        if (n >= p.Nc) continue;
        const int64_t coff = dim2_off(p.yk, n);
        const float bv = (p.epilogue & ALT_EPI_BIAS) ? p.bias[bz * p.bias_bstride + n] : 0.f;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int r = wm * WTM + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                const int64_t ro = rowoff[r];
                if (ro < 0) continue;
                float v = acc[i][j][e] + bv;
                if (p.epilogue & ALT_EPI_RELU) v = fmaxf(v, 0.f);
                if (p.out_bf16) ((uint16_t *)yb)[ro + coff] = f32_to_bf16_rne(v);
                else ((float *)yb)[ro + coff] = v;
            }
    }
}

// Consecutive logical tiles stay on one XCD (workgroup ids are dealt round-robin
// to the 8 XCDs), n-tiles of one m-tile adjacent, so the activation rows they
// share are served by the same L2.
__device__ __forceinline__ int igemm_logical_tile(int ntiles)
{
    const int id = blockIdx.x, xcd = id & 7, slot = id >> 3;
    const int q = ntiles >> 3, rem = ntiles & 7;
    return xcd * q + min(xcd, rem) + slot;
}

template <typename T, int BM, int BN, int BK, int WGM, int WGN, int AMODE, int BMODE, int PF>
__global__ __launch_bounds__(kIgemmThreads) void igemm_kernel(const IgemmParams p)
{
    using TR = ElemTraits<T>;
    using E = typename TR::store_t;
    constexpr int EPV = TR::EPV;
    constexpr int ES = TR::SIZE;
    constexpr int LDA = BK + EPV, LDB = BK + EPV;          // LDS row pitch in elements
    constexpr int WTM = BM / WGM, WTN = BN / WGN;          // wavefront tile
    constexpr int TM = WTM / 32, TN = WTN / 32;            // 32x32 MFMA tiles per wavefront
    constexpr int KC = 2 * EPV;                            // k consumed per fragment read
    constexpr int CPR = BK / EPV;                          // 16-byte chunks per LDS row
    constexpr int RPP = kIgemmThreads / CPR;               // rows covered per pass (VEC)
    constexpr int NVA = BM / RPP, NVB = BN / RPP;          // vectors per thread (VEC)
    constexpr int NGA = BM * BK / kIgemmThreads;           // elements per thread (GATHER)
    constexpr int NGB = BN * BK / kIgemmThreads;
    static_assert(WGM * WGN == 4, "four wavefronts");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0 && BK % KC == 0, "tile shape");
    static_assert(AMODE != LOAD_VEC || (BM % RPP == 0 && BM >= RPP), "vector loader shape");
    static_assert(BMODE != LOAD_VEC || (BN % RPP == 0 && BN >= RPP), "vector loader shape");
    static_assert(kIgemmThreads % BM == 0 && kIgemmThreads % BN == 0, "gather loader shape");
    // transposing loader: blocks of EPV rows x EPV k, dealt to threads row-group first
    constexpr int RVA = BM / EPV, RVB = BN / EPV;
    constexpr int NQA = ((BM / EPV) * (BK / EPV) + kIgemmThreads - 1) / kIgemmThreads;
    constexpr int NQB = ((BN / EPV) * (BK / EPV) + kIgemmThreads - 1) / kIgemmThreads;

    extern __shared__ uint4 smem_u4[];
    E *As = (E *)smem_u4;                                  // [2][BM][LDA]
    E *Bs = As + 2 * BM * LDA;                             // [2][BN][LDB]
    KEntry *ktab = (KEntry *)(Bs + 2 * BN * LDB);          // [kKTab]

    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const int wm = wave / WGN, wn = wave % WGN;

    const int ntiles = p.tiles_m * p.tiles_n;
    const int logical = igemm_logical_tile(ntiles);
    const int nt = logical % p.tiles_n, mt = logical / p.tiles_n;
    const int m0 = mt * BM, n0 = nt * BN;
    const int split = blockIdx.y % p.splitk, bz = blockIdx.y / p.splitk;
    const int kbeg = split * p.ksteps_per_split;
    const int nk = min(p.ksteps_per_split, p.ksteps_total - kbeg);

    const char *xb = (const char *)p.x + (int64_t)bz * p.x_bstride * ES;
    const char *wb = (const char *)p.w + (int64_t)bz * p.w_bstride * ES;
    // raw buffer descriptors (stride 0, 32-bit data format) over one batch entry of each operand
    const __amdgpu_buffer_rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)xb, 0, (int)p.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)wb, 0, (int)p.w_bytes, 0x00020000);

    // ---- per-thread row bases --------------------------------------------------
    constexpr int NRA = AMODE == LOAD_VEC ? NVA : 1;
    constexpr int NRB = BMODE == LOAD_VEC ? NVB : 1;
    int64_t a_base[NRA];
    int32_t a_ih0[NRA], a_iw0[NRA];
    int64_t b_base[NRB];
    bool b_ok[NRB];
    const int ohow = p.OH * p.OW;

    auto decode_a_row = [&](int row, int64_t &base, int32_t &ih0, int32_t &iw0) {
        const int m = m0 + row;
        if (m < p.M) {
            const int img = (int)fast_div(m, p.fd_ohow), rem = m - img * ohow;
            const int oh = (int)fast_div(rem, p.fd_ow), ow = rem - oh * p.OW;
            ih0 = oh * p.stride_h - p.pad_h;
            iw0 = ow * p.stride_w - p.pad_w;
            base = dim2_off(p.xn, img);
            if (p.spatial_split) base += dim2_off(p.xh, ih0) + dim2_off(p.xw, iw0);
            else base += (int64_t)ih0 * p.xh.si + (int64_t)iw0 * p.xw.si;
        } else {
            ih0 = -(1 << 28); iw0 = -(1 << 28); base = 0;
        }
    };

    if constexpr (AMODE == LOAD_VEC) {
        const int cc = (t % CPR) * EPV;
        const int64_t coff = dim2_off(p.xc, cc);
#pragma unroll
        for (int i = 0; i < NVA; ++i) {
            decode_a_row(t / CPR + i * RPP, a_base[i], a_ih0[i], a_iw0[i]);
            a_base[i] += coff;
        }
    } else if constexpr (AMODE == LOAD_GATHER) {
        decode_a_row(t % BM, a_base[0], a_ih0[0], a_iw0[0]);
    } else {
        // TRANS: thread owns 8 (4) consecutive rows; rows are memory-contiguous
        // (GMM A stored "KM"): only meaningful without spatial structure
        decode_a_row((t % RVA) * EPV, a_base[0], a_ih0[0], a_iw0[0]);
    }
    if constexpr (BMODE == LOAD_VEC) {
        const int cc = (t % CPR) * EPV;
        const int64_t coff = dim2_off(p.wi, cc);
#pragma unroll
        for (int i = 0; i < NVB; ++i) {
            const int n = n0 + t / CPR + i * RPP;
            b_ok[i] = n < p.Nc;
            b_base[i] = b_ok[i] ? dim2_off(p.wo, n) + coff : 0;
        }
    } else if constexpr (BMODE == LOAD_GATHER) {
        const int n = n0 + t % BN;
        b_ok[0] = n < p.Nc;
        b_base[0] = b_ok[0] ? dim2_off(p.wo, n) : 0;
    } else {
        const int n = n0 + (t % RVB) * EPV;
        b_ok[0] = n < p.Nc;                       // Nc % EPV == 0 is required by the host
        b_base[0] = b_ok[0] ? dim2_off(p.wo, n) : 0;
    }

    // ---- K-step table ----------------------------------------------------------
    auto fill_ktab = [&](int first) {
        for (int j = t; j < kKTab && first + j < nk; j += kIgemmThreads) {
            const int k0 = (kbeg + first + j) * BK;
            const int rs = (int)fast_div(k0, p.fd_c), c0 = k0 - rs * p.C;
            const int r = (int)fast_div(rs, p.fd_s), s = rs - r * p.S;
            KEntry e;
            e.dh = r * p.dil_h;
            e.dw = s * p.dil_w;
            e.a_off = (int64_t)e.dh * p.xh.si + (int64_t)e.dw * p.xw.si + dim2_off(p.xc, c0);
            e.b_off = dim2_off(p.wr, r) + dim2_off(p.ws, s) + dim2_off(p.wi, c0);
            ktab[j] = e;
        }
    };

    // ---- operand fetch: global -> registers ------------------------------------
    constexpr int NA_REG = AMODE == LOAD_VEC ? NVA : AMODE == LOAD_GATHER ? (NGA * ES + 15) / 16 : NQA * EPV;
    constexpr int NB_REG = BMODE == LOAD_VEC ? NVB : BMODE == LOAD_GATHER ? (NGB * ES + 15) / 16 : NQB * EPV;
    uint4 a_regs[PF][NA_REG], b_regs[PF][NB_REG];     // PF K steps of operand data in flight

    auto gather_one = [&](const char *basep, int64_t rowbase, int32_t ih0, int32_t iw0, bool rowok,
                          int kk, int kstep, const KEntry &e, bool is_a) -> E {
        // element (row, kk) of the current K step, any two-level layout
        E v = 0;
        if (p.uniform_rs) {
            if (is_a) {
                bool ok = (unsigned)(ih0 + e.dh) < (unsigned)p.H && (unsigned)(iw0 + e.dw) < (unsigned)p.W;
                if (ok) v = *(const E *)(basep + (rowbase + e.a_off + dim2_off(p.xc, kk)) * ES);
            } else if (rowok) {
                v = *(const E *)(basep + (rowbase + e.b_off + dim2_off(p.wi, kk)) * ES);
            }
        } else {
            const int k = (kbeg + kstep) * BK + kk;
            if (k < p.Kg) {
                const int rs = (int)fast_div(k, p.fd_c), c = k - rs * p.C;
                const int r = (int)fast_div(rs, p.fd_s), s = rs - r * p.S;
                if (is_a) {
                    const int ih = ih0 + r * p.dil_h, iw = iw0 + s * p.dil_w;
                    if ((unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W) {
                        int64_t off = rowbase + dim2_off(p.xc, c);
                        if (p.spatial_split) off += 0;   // r = s = 0 here, row base already complete
                        else off += (int64_t)(r * p.dil_h) * p.xh.si + (int64_t)(s * p.dil_w) * p.xw.si;
                        v = *(const E *)(basep + off * ES);
                    }
                } else if (rowok) {
                    v = *(const E *)(basep + (rowbase + dim2_off(p.wr, r) + dim2_off(p.ws, s) + dim2_off(p.wi, c)) * ES);
                }
            }
        }
        return v;
    };

    auto fetch = [&](int kstep, uint4 *a_reg, uint4 *b_reg) {
        const KEntry e = ktab[kstep % kKTab];
        if constexpr (AMODE == LOAD_VEC) {
#pragma unroll
            for (int i = 0; i < NVA; ++i) {
                const bool ok = (unsigned)(a_ih0[i] + e.dh) < (unsigned)p.H &&
                                (unsigned)(a_iw0[i] + e.dw) < (unsigned)p.W;
                a_reg[i] = buffer_load16(x_rsrc, ok ? (uint32_t)((a_base[i] + e.a_off) * ES) : kOutOfRange);
            }
        } else if constexpr (AMODE == LOAD_GATHER) {
            E *dst = (E *)a_reg;
            constexpr int KSTR = kIgemmThreads / BM;
#pragma unroll
            for (int i = 0; i < NGA; ++i) {
                const int kk = t / BM + i * KSTR;
                dst[i] = gather_one(xb, a_base[0], a_ih0[0], a_iw0[0], true, kk, kstep, e, true);
            }
        } else {
            // rows contiguous: vector j covers rows r0..r0+EPV-1 at k = kq*EPV + j
#pragma unroll
            for (int q = 0; q < NQA; ++q) {
                const int kq = t / RVA + q * (kIgemmThreads / RVA);
#pragma unroll
                for (int j = 0; j < EPV; ++j) {
                    const int k = (kbeg + kstep) * BK + kq * EPV + j;
                    const bool ok = a_ih0[0] >= 0 && kq < BK / EPV && k < p.Kg;
                    a_reg[q * EPV + j] = ok ? *(const uint4 *)(xb + (a_base[0] + dim2_off(p.xc, k)) * ES)
                                            : make_uint4(0, 0, 0, 0);
                }
            }
        }
        if constexpr (BMODE == LOAD_VEC) {
#pragma unroll
            for (int i = 0; i < NVB; ++i)
                b_reg[i] = buffer_load16(w_rsrc, b_ok[i] ? (uint32_t)((b_base[i] + e.b_off) * ES) : kOutOfRange);
        } else if constexpr (BMODE == LOAD_GATHER) {
            E *dst = (E *)b_reg;
            constexpr int KSTR = kIgemmThreads / BN;
#pragma unroll
            for (int i = 0; i < NGB; ++i) {
                const int kk = t / BN + i * KSTR;
                dst[i] = gather_one(wb, b_base[0], 0, 0, b_ok[0], kk, kstep, e, false);
            }
        } else {
#pragma unroll
            for (int q = 0; q < NQB; ++q) {
                const int kq = t / RVB + q * (kIgemmThreads / RVB);
#pragma unroll
                for (int j = 0; j < EPV; ++j) {
                    const int k = (kbeg + kstep) * BK + kq * EPV + j;
                    const bool ok = b_ok[0] && kq < BK / EPV && k < p.Kg;
                    b_reg[q * EPV + j] = ok ? *(const uint4 *)(wb + (b_base[0] + dim2_off(p.wi, k)) * ES)
                                            : make_uint4(0, 0, 0, 0);
                }
            }
        }
    };

    // ---- registers -> LDS stage --------------------------------------------------
    auto stash = [&](int stage, const uint4 *a_reg, const uint4 *b_reg) {
        E *as = As + stage * BM * LDA;
        E *bs = Bs + stage * BN * LDB;
        if constexpr (AMODE == LOAD_VEC) {
#pragma unroll
            for (int i = 0; i < NVA; ++i)
                *(uint4 *)(as + (t / CPR + i * RPP) * LDA + (t % CPR) * EPV) = a_reg[i];
        } else if constexpr (AMODE == LOAD_GATHER) {
            const E *srcv = (const E *)a_reg;
            constexpr int KSTR = kIgemmThreads / BM;
#pragma unroll
            for (int i = 0; i < NGA; ++i)
                as[(t % BM) * LDA + t / BM + i * KSTR] = srcv[i];
        } else {
#pragma unroll
            for (int q = 0; q < NQA; ++q) {
                const int kq = t / RVA + q * (kIgemmThreads / RVA);
                uint4 blk[EPV];
#pragma unroll
                for (int j = 0; j < EPV; ++j) blk[j] = a_reg[q * EPV + j];
                if constexpr (EPV == 8) transpose8x8_b16(blk); else transpose4x4_b32(blk);
                if (kq < BK / EPV) {
#pragma unroll
                    for (int j = 0; j < EPV; ++j)
                        *(uint4 *)(as + ((t % RVA) * EPV + j) * LDA + kq * EPV) = blk[j];
                }
            }
        }
        if constexpr (BMODE == LOAD_VEC) {
#pragma unroll
            for (int i = 0; i < NVB; ++i)
                *(uint4 *)(bs + (t / CPR + i * RPP) * LDB + (t % CPR) * EPV) = b_reg[i];
        } else if constexpr (BMODE == LOAD_GATHER) {
            const E *srcv = (const E *)b_reg;
            constexpr int KSTR = kIgemmThreads / BN;
#pragma unroll
            for (int i = 0; i < NGB; ++i)
                bs[(t % BN) * LDB + t / BN + i * KSTR] = srcv[i];
        } else {
#pragma unroll
            for (int q = 0; q < NQB; ++q) {
                const int kq = t / RVB + q * (kIgemmThreads / RVB);
                uint4 blk[EPV];
#pragma unroll
                for (int j = 0; j < EPV; ++j) blk[j] = b_reg[q * EPV + j];
                if constexpr (EPV == 8) transpose8x8_b16(blk); else transpose4x4_b32(blk);
                if (kq < BK / EPV) {
#pragma unroll
                    for (int j = 0; j < EPV; ++j)
                        *(uint4 *)(bs + ((t % RVB) * EPV + j) * LDB + kq * EPV) = blk[j];
                }
            }
        }
    };

    // ---- main loop -----------------------------------------------------------------
    floatx16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    if (nk > 0) {
        fill_ktab(0);
        lds_barrier();
#pragma unroll
        for (int j = 0; j < PF; ++j)
            if (j < nk) fetch(j, a_regs[j], b_regs[j]);
        stash(0, a_regs[0], b_regs[0]);
        lds_barrier();
        for (int ks0 = 0; ks0 < nk; ks0 += PF) {
#pragma unroll
            for (int j = 0; j < PF; ++j) {
                const int ks = ks0 + j;
                if (ks >= nk) break;
                const int nf = ks + PF;            // its data goes into the register slot step ks just left
                if (nf < nk) {
                    if (nf % kKTab == 0) {         // next window of the K-step table
                        lds_barrier();
                        fill_ktab(nf);
                        lds_barrier();
                    }
                    fetch(nf, a_regs[j], b_regs[j]);
                }
                const E *as = As + (ks & 1) * BM * LDA + (wm * WTM + (lane & 31)) * LDA + (lane >> 5) * EPV;
                const E *bs = Bs + (ks & 1) * BN * LDB + (wn * WTN + (lane & 31)) * LDB + (lane >> 5) * EPV;
#pragma unroll
                for (int kc = 0; kc < BK / KC; ++kc) {
                    uint4 af[TM], bf[TN];
#pragma unroll
                    for (int i = 0; i < TM; ++i) af[i] = *(const uint4 *)(as + i * 32 * LDA + kc * KC);
#pragma unroll
                    for (int jn = 0; jn < TN; ++jn) bf[jn] = *(const uint4 *)(bs + jn * 32 * LDB + kc * KC);
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int jn = 0; jn < TN; ++jn) mma_tile(acc[i][jn], af[i], bf[jn], T{});
                }
                if (ks + 1 < nk) stash((ks + 1) & 1, a_regs[(j + 1) % PF], b_regs[(j + 1) % PF]);
                lds_barrier();
            }
        }
    }

    igemm_epilogue<BM, TM, TN, WTM, WTN>(p, acc, (void *)smem_u4, m0, n0, wm, wn, split, bz);
}

struct DconvParams;           // dconv.h

// Launch of one instantiation; defined in the igemm_*.hip and dconv_*.hip files.
struct IgemmLaunch {
    const char *name;
    int dtype, BM, BN, BK, amode, bmode;
    int prefetch;             // register pipeline: K steps of loads in flight; DMA pipeline: LDS stages - 1
    int dma;                  // 1 = operands go global -> LDS directly (igemm_dma.h)
    size_t lds_bytes;
    hipError_t (*launch)(const IgemmParams &p, dim3 grid, hipStream_t st);
    // set instead of `launch` for the patch-resident direct convolution (dconv.h),
    // which splits K over channel slices and reduces them inside the same launch
    hipError_t (*launch_direct)(const DconvParams &p, size_t lds_bytes, hipStream_t st) = nullptr;
    int wgm = 0, wgn = 0;     // wave grid of a direct kernel
    int kw = 1;               // its K groups (each a wave grid of its own over a share of the channels)
    int stream = 0;           // 1: both operands stream through LDS (dstream.h: 1x1 filters and GEMMs of any depth);
                              // 2: channel-planar operands converted on the way into LDS (dplanar.h)
    int bt = 0;               // streaming kernel: 1 = B stored [K][N] (row-major), read through LDS transpose reads
};

template <typename T, int BM, int BN, int BK, int WGM, int WGN, int AMODE, int BMODE, int PF>
hipError_t igemm_launch(const IgemmParams &p, dim3 grid, hipStream_t st)
{
    using TR = ElemTraits<T>;
    constexpr size_t lds = (size_t)2 * (BM + BN) * (BK + TR::EPV) * TR::SIZE + kKTab * sizeof(KEntry);
    auto kern = igemm_kernel<T, BM, BN, BK, WGM, WGN, AMODE, BMODE, PF>;
    static bool attr_set = false;
    if (!attr_set && lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, grid, dim3(kIgemmThreads), lds, st, p);
    return hipGetLastError();
}

template <typename T, int BM, int BN, int BK>
constexpr size_t igemm_lds_bytes()
{
    return (size_t)2 * (BM + BN) * (BK + ElemTraits<T>::EPV) * ElemTraits<T>::SIZE + kKTab * sizeof(KEntry);
}

const std::vector<IgemmLaunch> &igemm_table();
void igemm_register(const IgemmLaunch &l);

}  // namespace alt

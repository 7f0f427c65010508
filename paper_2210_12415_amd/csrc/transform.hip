// Layout conversion operator (Section 4.2 of the paper): an element copy
// under two index maps.  Both maps are split+reorder sequences, so after
// cutting every logical dimension at the union of both layouts' block
// boundaries the conversion is a strided permutation of a small number of
// "pieces", each with a source and a destination stride.  Three kernels:
//   rows      – the memory-contiguous piece is the same on both sides:
//               contiguous runs are copied with vector loads and stores;
//   transpose – it differs: a 2-D tile (source-contiguous piece x
//               destination-contiguous piece) goes through LDS so that both
//               the global reads and the global writes are coalesced;
//   general   – anything else (blocks that do not nest, sequences with a
//               non-separable fuse): one thread per logical element.
#include <algorithm>
#include <functional>

#include "common.h"
#include "layout_eval.h"

namespace alt {

namespace {

constexpr int kThreads = 256;
constexpr int kMaxOuter = 7;

struct Piece {
    int64_t ext, ss, ds;
};

struct PermuteParams {
    const void *src;
    void *dst;
    int32_t n_outer;
    int32_t TA, TB, LD;
    int64_t outer_ext[kMaxOuter], outer_ss[kMaxOuter], outer_ds[kMaxOuter];
    int64_t ext_a, ext_b;     // extents of the two tile pieces
    int64_t ss_b, ds_b;       // strides of piece b (ds_b = 1 in the transpose kernel)
    int64_t ss_a, ds_a;       // strides of piece a (ss_a = 1 always; ds_a = 1 in the rows kernel)
    int64_t tiles_a, tiles_b;
};

template <int BYTES> struct Word;
template <> struct Word<2> { using type = uint16_t; };
template <> struct Word<4> { using type = uint32_t; };
template <> struct Word<8> { using type = uint2; };
template <> struct Word<16> { using type = uint4; };

// Block -> (outer indices, tile origin).  Uniform per block.  The block count and
// every extent fit 32 bits (checked by the host): 32-bit divisions, which cost a
// fraction of 64-bit ones, and these few dozen instructions are on every block's
// critical path before its first load.
__device__ inline void locate_tile(const PermuteParams &p, int64_t &src_base, int64_t &dst_base,
                                   int64_t &a0, int64_t &b0)
{
    uint32_t t = blockIdx.x;
    const uint32_t tiles_a = (uint32_t)p.tiles_a, tiles_b = (uint32_t)p.tiles_b;
    uint32_t q = t / tiles_a;
    const uint32_t ta = t - q * tiles_a;
    t = q;
    q = t / tiles_b;
    const uint32_t tb = t - q * tiles_b;
    t = q;
    a0 = (int64_t)ta * p.TA;
    b0 = (int64_t)tb * p.TB;
    src_base = a0 * p.ss_a + b0 * p.ss_b;
    dst_base = a0 * p.ds_a + b0 * p.ds_b;
    for (int d = p.n_outer - 1; d >= 0; --d) {
        const uint32_t e = (uint32_t)p.outer_ext[d];
        q = t / e;
        const uint32_t i = t - q * e;
        t = q;
        src_base += (int64_t)i * p.outer_ss[d];
        dst_base += (int64_t)i * p.outer_ds[d];
    }
}

// Two access policies.  Streaming (NT = true): a conversion reads every source element once and
// writes every destination element once, so both sides carry the non-temporal hint and the lines
// do not displace data somebody will read again; on tensors that exceed the caches this measured
// +25 % (12.8 MB tensor, cold) and +10 % (205 MB) against the other policy.  Cached (NT = false):
// plain loads, stores that go through to memory as they are written (sc0 sc1) but stay in the L2:
// a tensor that an operator has just produced is read from the cache, and the converted tensor is
// there for the operator that consumes it (7.2 -> 5.5 us for a 12.8 MB tensor between two layers).
// The host takes the cached policy for tensors of up to kStreamingBytes.
constexpr size_t kStreamingBytes = (size_t)16 << 20;

template <bool NT, typename V>
__device__ __forceinline__ void store_vec(char *addr, const V &w)
{
    typedef uint32_t n4_t __attribute__((ext_vector_type(4)));
    typedef uint32_t n2_t __attribute__((ext_vector_type(2)));
    if constexpr (NT) {
        if constexpr (sizeof(V) == 16) __builtin_nontemporal_store(__builtin_bit_cast(n4_t, w), (n4_t *)addr);
        else if constexpr (sizeof(V) == 8) __builtin_nontemporal_store(__builtin_bit_cast(n2_t, w), (n2_t *)addr);
        else if constexpr (sizeof(V) == 4) __builtin_nontemporal_store(__builtin_bit_cast(uint32_t, w), (uint32_t *)addr);
        else __builtin_nontemporal_store(__builtin_bit_cast(uint16_t, w), (uint16_t *)addr);
    } else if constexpr (sizeof(V) == 16) {
        // (a store of more than 64 bits reads its data registers up to two cycles after it issues, and
        // the compiler, which keeps VALU writes to them away from its own stores, does not look inside
        // an asm statement: the wait states stand here)
        const n4_t v = __builtin_bit_cast(n4_t, w);
        asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1\n\ts_nop 1" : : "v"(addr), "v"(v) : "memory");
    } else if constexpr (sizeof(V) == 8) {
        const n2_t v = __builtin_bit_cast(n2_t, w);
        asm volatile("global_store_dwordx2 %0, %1, off sc0 sc1" : : "v"(addr), "v"(v) : "memory");
    } else if constexpr (sizeof(V) == 4) {
        const uint32_t v = __builtin_bit_cast(uint32_t, w);
        asm volatile("global_store_dword %0, %1, off sc0 sc1" : : "v"(addr), "v"(v) : "memory");
    } else {
        *(V *)addr = w;
    }
}

template <bool NT, typename V>
__device__ __forceinline__ V load_vec(const char *addr)
{
    typedef uint32_t n4_t __attribute__((ext_vector_type(4)));
    typedef uint32_t n2_t __attribute__((ext_vector_type(2)));
    if constexpr (!NT) return *(const V *)addr;
    else if constexpr (sizeof(V) == 16) return __builtin_bit_cast(V, __builtin_nontemporal_load((const n4_t *)addr));
    else if constexpr (sizeof(V) == 8) return __builtin_bit_cast(V, __builtin_nontemporal_load((const n2_t *)addr));
    else if constexpr (sizeof(V) == 4) return __builtin_bit_cast(V, __builtin_nontemporal_load((const uint32_t *)addr));
    else return __builtin_bit_cast(V, __builtin_nontemporal_load((const uint16_t *)addr));
}

// Piece a is contiguous on both sides: copy TB runs of TA elements.
template <int ELSZ, int VBYTES, bool NT>
__global__ __launch_bounds__(kThreads) void permute_rows_kernel(PermuteParams p)
{
    using V = typename Word<VBYTES>::type;
    constexpr int VL = VBYTES / ELSZ;
    int64_t sb, db, a0, b0;
    locate_tile(p, sb, db, a0, b0);
    const int ta = (int)min((int64_t)p.TA, p.ext_a - a0);
    const int tb = (int)min((int64_t)p.TB, p.ext_b - b0);
    const int ra = ta / VL;                         // vectors per run (host guarantees divisibility)
    const char *src = (const char *)p.src;
    char *dst = (char *)p.dst;
    for (int v = threadIdx.x; v < ra * tb; v += kThreads) {
        int ib = v / ra, ia = (v - ib * ra) * VL;
        V w = load_vec<NT, V>(src + (sb + ib * p.ss_b + ia) * ELSZ);
        store_vec<NT>(dst + (db + ib * p.ds_b + ia) * ELSZ, w);
    }
}

// ---- tile kernel: piece a is contiguous in the source, piece b in the destination --------------
//
// A workgroup moves a tile of TG x TB x TA elements (g: an outer piece, b, a) through LDS.  The
// tile sits in LDS in source order; the load side copies 16-byte (or narrower) vectors along a,
// the store side gathers its vectors along b element by element.  All global loads of a trip
// (four vectors per thread) are issued before the first LDS write, so a workgroup has its whole
// tile in flight at once, and no thread divides: a vector's place in the tile comes from
// multiplications by reciprocals of the tile's (launch-wide) extents; threads whose place falls
// outside a ragged edge tile sit the trip out.
//
// "Flat" sides.  When the tile takes piece a whole and rows follow one another without a gap in
// the source (stride of b = extent of a), the tile's source is one contiguous run whatever the
// row length, and is loaded as such: 16-byte vectors even where a row is 49 elements long.
// Likewise the destination when the tile takes piece b whole and the stride of a there is the
// extent of b.  A g piece whose stride equals extent(a) * extent(b) on a flat side keeps it flat.
struct TileParams {
    const void *src;
    void *dst;
    int32_t n_outer;
    int32_t TA, TB, TG;                 // tile extents (full tiles)
    int32_t ext_a, ext_b, ext_g;        // piece extents
    int32_t LD, GS;                     // LDS: element (g, b, a) at g * GS + b * LD + a
    uint32_t tiles_a, tiles_b, tiles_g;
    uint32_t outer_ext[kMaxOuter];
    int64_t outer_ss[kMaxOuter], outer_ds[kMaxOuter];
    int64_t ss_b, ss_g;                 // source strides in elements (a: 1)
    int64_t ds_a, ds_g;                 // destination strides in elements (b: 1)
    FastDiv d_ra, d_tb;                 // load side: vectors per row (TA / VL), rows per g (TB)
    FastDiv d_rb, d_ta;                 // store side: vectors per row (TB / VS), rows per g (TA)
    FastDiv d_tiles_a, d_tiles_b, d_tiles_g;
};

// Where a tile starts: tile extents clipped at the pieces' ends, element offsets of its origin.
struct TileOrigin {
    int ta, tb, tg;
    int64_t sb, db;
};

__host__ __device__ inline TileOrigin tile_origin(const TileParams &p, uint32_t block)
{
    uint32_t t = block;
    uint32_t q = fast_div(t, p.d_tiles_a);
    const uint32_t ia = t - q * p.tiles_a;
    t = q;
    q = fast_div(t, p.d_tiles_b);
    const uint32_t ib = t - q * p.tiles_b;
    t = q;
    q = fast_div(t, p.d_tiles_g);
    const uint32_t ig = t - q * p.tiles_g;
    t = q;
    TileOrigin o;
    const int a0 = (int)ia * p.TA, b0 = (int)ib * p.TB, g0 = (int)ig * p.TG;
    o.ta = p.ext_a - a0 < p.TA ? p.ext_a - a0 : p.TA;
    o.tb = p.ext_b - b0 < p.TB ? p.ext_b - b0 : p.TB;
    o.tg = p.ext_g - g0 < p.TG ? p.ext_g - g0 : p.TG;
    o.sb = (int64_t)a0 + (int64_t)b0 * p.ss_b + (int64_t)g0 * p.ss_g;
    o.db = (int64_t)a0 * p.ds_a + (int64_t)b0 + (int64_t)g0 * p.ds_g;
    for (int d = p.n_outer - 1; d >= 0; --d) {
        const uint32_t e = p.outer_ext[d];
        q = t / e;
        const uint32_t i = t - q * e;
        t = q;
        o.sb += (int64_t)i * p.outer_ss[d];
        o.db += (int64_t)i * p.outer_ds[d];
    }
    return o;
}

// Load side, vector v of the tile: source offset (elements, relative to the tile's origin) and
// LDS index of its first element; false if the vector lies outside this (ragged) tile.
template <int VL, bool SF>
__host__ __device__ inline bool tile_load_slot(const TileParams &p, const TileOrigin &o, uint32_t v, int64_t *src_off,
                                               uint32_t *lds_idx)
{
    if constexpr (SF) {
        // one contiguous run of tg * tb * ta elements, copied as it is
        *src_off = (int64_t)v * VL;
        *lds_idx = v * VL;
        return v * VL < (uint32_t)(o.tg * o.tb * o.ta);
    } else {
        const uint32_t r = fast_div(v, p.d_ra), iav = v - r * (uint32_t)(p.TA / VL);
        const uint32_t ig = fast_div(r, p.d_tb), ib = r - ig * (uint32_t)p.TB;
        *src_off = (int64_t)ig * p.ss_g + (int64_t)ib * p.ss_b + iav * VL;
        *lds_idx = ig * p.GS + ib * p.LD + iav * VL;
        return iav * VL < (uint32_t)o.ta && ib < (uint32_t)o.tb && ig < (uint32_t)o.tg;
    }
}

// Store side, vector u of the tile: destination offset (elements, relative to the tile's origin)
// and, per element j of the vector, the LDS index it comes from.
template <int VS, bool DF>
__host__ __device__ inline bool tile_store_slot(const TileParams &p, const TileOrigin &o, uint32_t u, int64_t *dst_off,
                                                uint32_t (&lds_idx)[VS])
{
    if constexpr (DF) {
        // one contiguous run of tg * ta * tb elements (tb = the whole piece b); element f of it is
        // (g, a, b) = (f / (TA * tb), (f / tb) % TA, f % tb), and a vector may straddle rows
        *dst_off = (int64_t)u * VS;
#pragma unroll
        for (int j = 0; j < VS; ++j) {
            const uint32_t f = u * VS + j;
            const uint32_t r = fast_div(f, p.d_rb), ib = f - r * (uint32_t)p.TB;       // d_rb divides by TB here
            const uint32_t ig = fast_div(r, p.d_ta), ia = r - ig * (uint32_t)p.TA;
            lds_idx[j] = ig * p.GS + ib * p.LD + ia;
        }
        return u * VS < (uint32_t)(o.tg * o.ta * o.tb);
    } else {
        const uint32_t r = fast_div(u, p.d_rb), ibv = u - r * (uint32_t)(p.TB / VS);
        const uint32_t ig = fast_div(r, p.d_ta), ia = r - ig * (uint32_t)p.TA;
        *dst_off = (int64_t)ig * p.ds_g + (int64_t)ia * p.ds_a + ibv * VS;
        const uint32_t base = ig * p.GS + ibv * VS * p.LD + ia;
#pragma unroll
        for (int j = 0; j < VS; ++j) lds_idx[j] = base + j * p.LD;
        return ibv * VS < (uint32_t)o.tb && ia < (uint32_t)o.ta && ig < (uint32_t)o.tg;
    }
}

constexpr int kTrip = 4;                   // vectors a thread has in flight per trip

template <int ELSZ, int LBYTES, int SBYTES, bool SF, bool DF, bool NT>
__global__ __launch_bounds__(kThreads) void permute_tile_kernel(TileParams p)
{
    using E = typename Word<ELSZ>::type;
    using VLd = typename Word<LBYTES>::type;
    using VSt = typename Word<SBYTES>::type;
    constexpr int VL = LBYTES / ELSZ, VS = SBYTES / ELSZ;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    E *tile = (E *)smem_raw;
    const TileOrigin o = tile_origin(p, blockIdx.x);
    const char *src = (const char *)p.src + o.sb * ELSZ;
    char *dst = (char *)p.dst + o.db * ELSZ;
    const uint32_t nvl = SF ? (uint32_t)(p.TG * p.TB * p.TA) / VL : (uint32_t)(p.TG * p.TB) * (uint32_t)(p.TA / VL);
    const uint32_t nvs = DF ? (uint32_t)(p.TG * p.TA * p.TB) / VS : (uint32_t)(p.TG * p.TA) * (uint32_t)(p.TB / VS);
    for (uint32_t base = 0; base < nvl; base += kTrip * kThreads) {
        VLd w[kTrip];
        uint32_t li[kTrip];
        bool ok[kTrip];
#pragma unroll
        for (int k = 0; k < kTrip; ++k) {
            const uint32_t v = base + k * kThreads + threadIdx.x;
            int64_t so;
            ok[k] = tile_load_slot<VL, SF>(p, o, v, &so, &li[k]) && v < nvl;
            // (a vector outside the tile reads the tile's first vector instead: always in bounds, never stored)
            w[k] = load_vec<NT, VLd>(src + (ok[k] ? so : 0) * ELSZ);
        }
#pragma unroll
        for (int k = 0; k < kTrip; ++k) {
            if (!ok[k]) continue;
            if constexpr (SF) {
                *(VLd *)(tile + li[k]) = w[k];                  // the tile is a plain copy of the run
            } else {
                const E *e = (const E *)&w[k];
#pragma unroll
                for (int j = 0; j < VL; ++j) tile[li[k] + j] = e[j];
            }
        }
    }
    __syncthreads();
    for (uint32_t base = 0; base < nvs; base += kTrip * kThreads) {
#pragma unroll
        for (int k = 0; k < kTrip; ++k) {
            const uint32_t u = base + k * kThreads + threadIdx.x;
            int64_t dof;
            uint32_t li[VS];
            if (!(tile_store_slot<VS, DF>(p, o, u, &dof, li) && u < nvs)) continue;
            VSt w;
            E *e = (E *)&w;
#pragma unroll
            for (int j = 0; j < VS; ++j) e[j] = tile[li[j]];
            store_vec<NT>(dst + dof * ELSZ, w);
        }
    }
}

// One thread per logical index of the box `it_shape` (the tensor's shape; for the pad form the
// part of the index space both tensors have): each layout is evaluated under its own shape.
struct GeneralParams {
    const void *src;
    void *dst;
    BoundLayout ls, ld;
    int64_t it_shape[ALT_MAX_RANK], it_numel;
};

template <int ELSZ>
__global__ __launch_bounds__(kThreads) void permute_general_kernel(GeneralParams p)
{
    using E = typename Word<ELSZ>::type;
    const int64_t n = p.it_numel;
    for (int64_t e = blockIdx.x * (int64_t)kThreads + threadIdx.x; e < n; e += (int64_t)gridDim.x * kThreads) {
        int64_t idx[ALT_MAX_RANK];
        int64_t r = e;
        for (int d = p.ls.ndim - 1; d >= 0; --d) { idx[d] = r % p.it_shape[d]; r /= p.it_shape[d]; }
        ((E *)p.dst)[eval_offset(p.ld, idx)] = ((const E *)p.src)[eval_offset(p.ls, idx)];
    }
}

// Zeros over `bytes` bytes (a multiple of 2) at a 2-byte-aligned address: 16-byte stores over the
// aligned middle, 2-byte stores at the ends.  (A kernel, not a memset: callers may be under graph capture.)
__global__ __launch_bounds__(kThreads) void fill_zero_kernel(char *dst, int64_t bytes)
{
    const int64_t head = std::min<int64_t>(bytes, (16 - ((uintptr_t)dst & 15)) & 15);
    const int64_t nvec = (bytes - head) / 16, tail0 = head + nvec * 16;
    const int64_t tid = blockIdx.x * (int64_t)kThreads + threadIdx.x, nth = (int64_t)gridDim.x * kThreads;
    for (int64_t v = tid; v < nvec; v += nth) *(uint4 *)(dst + head + v * 16) = make_uint4(0, 0, 0, 0);
    for (int64_t b = tid * 2; b < head; b += nth * 2) *(uint16_t *)(dst + b) = 0;
    for (int64_t b = tail0 + tid * 2; b < bytes; b += nth * 2) *(uint16_t *)(dst + b) = 0;
}

// The unfold primitive on one dimension of a row-major tensor seen as [outer][D][inner]:
// dst[o][t][b][i] = src[o][t*S + b][i], zero where t*S + b >= D.  One thread per VB-byte
// piece of the inner run (VB = 16 when the run allows, else the element size).
template <int VB>
__global__ __launch_bounds__(kThreads) void unfold_kernel(const char *src, char *dst, int64_t total, uint32_t vec_inner,
                                                          uint32_t B, uint32_t T, int64_t D, int64_t S)
{
    using V = typename Word<VB>::type;
    for (int64_t v = blockIdx.x * (int64_t)kThreads + threadIdx.x; v < total; v += (int64_t)gridDim.x * kThreads) {
        const int64_t q = v / vec_inner;
        const uint32_t i = (uint32_t)(v - q * vec_inner);
        const int64_t q2 = q / B;
        const uint32_t b = (uint32_t)(q - q2 * B);
        const int64_t o = q2 / T;
        const uint32_t t = (uint32_t)(q2 - o * T);
        const int64_t e = (int64_t)t * S + b;
        V w;
        std::memset(&w, 0, sizeof w);
        if (e < D) w = *(const V *)(src + ((o * D + e) * vec_inner + i) * VB);
        store_vec<false>(dst + v * VB, w);
    }
}

// Cuts every logical dimension at the union of both layouts' boundaries.
// Returns false when the boundaries do not nest (e.g. blocks of 12 and 8).
bool refine(const BoundLayout &s, const BoundLayout &d, std::vector<Piece> *out)
{
    for (int dim = 0; dim < s.ndim; ++dim) {
        std::vector<int64_t> cuts;
        for (int j = 0; j < s.nsub; ++j) if (s.atom[j].dim == dim) cuts.push_back(s.atom[j].div);
        for (int j = 0; j < d.nsub; ++j) if (d.atom[j].dim == dim) cuts.push_back(d.atom[j].div);
        cuts.push_back(s.shape[dim]);
        std::sort(cuts.begin(), cuts.end());
        cuts.erase(std::unique(cuts.begin(), cuts.end()), cuts.end());
        for (size_t c = 0; c + 1 < cuts.size(); ++c) {
            int64_t lo = cuts[c], hi = cuts[c + 1];
            if (hi % lo != 0) return false;
            Piece pc{hi / lo, -1, -1};
            for (int j = 0; j < s.nsub; ++j) {
                const Atom &a = s.atom[j];
                if (a.dim == dim && a.div <= lo && lo < a.div * a.ext) {
                    if (lo % a.div != 0 || (a.div * a.ext) % hi != 0) return false;
                    pc.ss = a.stride * (lo / a.div);
                }
            }
            for (int j = 0; j < d.nsub; ++j) {
                const Atom &a = d.atom[j];
                if (a.dim == dim && a.div <= lo && lo < a.div * a.ext) {
                    if (lo % a.div != 0 || (a.div * a.ext) % hi != 0) return false;
                    pc.ds = a.stride * (lo / a.div);
                }
            }
            if (pc.ss < 0 || pc.ds < 0) return false;
            if (pc.ext > 1) out->push_back(pc);
        }
    }
    // destination order, then merge neighbours that are contiguous on both sides
    std::sort(out->begin(), out->end(), [](const Piece &x, const Piece &y) { return x.ds > y.ds; });
    std::vector<Piece> m;
    for (const Piece &pc : *out) {
        if (!m.empty() && m.back().ds == pc.ds * pc.ext && m.back().ss == pc.ss * pc.ext) {
            m.back().ext *= pc.ext;
            m.back().ss = pc.ss;
            m.back().ds = pc.ds;
        } else {
            m.push_back(pc);
        }
    }
    out->swap(m);
    return true;
}

int pick_vector_bytes(int elsz, int64_t run, const std::vector<int64_t> &strides, const void *ptr)
{
    for (int vb : {16, 8}) {
        if (vb <= elsz) break;
        int vl = vb / elsz;
        bool ok = run % vl == 0 && ((uintptr_t)ptr % vb) == 0;
        for (int64_t st : strides) ok = ok && (st % vl == 0);
        if (ok) return vb;
    }
    return elsz;
}

template <int ELSZ, bool NT>
void launch_rows_nt(int vb, const PermuteParams &p, dim3 grid, hipStream_t st)
{
    if (vb == 16) hipLaunchKernelGGL((permute_rows_kernel<ELSZ, 16, NT>), grid, dim3(kThreads), 0, st, p);
    else if (vb == 8) hipLaunchKernelGGL((permute_rows_kernel<ELSZ, 8, NT>), grid, dim3(kThreads), 0, st, p);
    else hipLaunchKernelGGL((permute_rows_kernel<ELSZ, ELSZ, NT>), grid, dim3(kThreads), 0, st, p);
}

template <int ELSZ>
void launch_rows(int vb, bool nt, const PermuteParams &p, dim3 grid, hipStream_t st)
{
    if (nt) launch_rows_nt<ELSZ, true>(vb, p, grid, st);
    else launch_rows_nt<ELSZ, false>(vb, p, grid, st);
}

template <int ELSZ, int LB, int SB, bool SF, bool DF>
void launch_tile_k(bool nt, const TileParams &p, dim3 grid, size_t lds, hipStream_t st)
{
    if (nt) hipLaunchKernelGGL((permute_tile_kernel<ELSZ, LB, SB, SF, DF, true>), grid, dim3(kThreads), lds, st, p);
    else hipLaunchKernelGGL((permute_tile_kernel<ELSZ, LB, SB, SF, DF, false>), grid, dim3(kThreads), lds, st, p);
}

template <int ELSZ, int LB, bool SF>
void launch_tile_s(int sb, bool df, bool nt, const TileParams &p, dim3 grid, size_t lds, hipStream_t st)
{
    if (df) launch_tile_k<ELSZ, LB, 16, SF, true>(nt, p, grid, lds, st);      // a flat side moves 16-byte vectors
    else if (sb == 16) launch_tile_k<ELSZ, LB, 16, SF, false>(nt, p, grid, lds, st);
    else if (sb == 8) launch_tile_k<ELSZ, LB, 8, SF, false>(nt, p, grid, lds, st);
    else launch_tile_k<ELSZ, LB, ELSZ, SF, false>(nt, p, grid, lds, st);
}

template <int ELSZ>
void launch_tile(int lb, int sb, bool sf, bool df, bool nt, const TileParams &p, dim3 grid, size_t lds, hipStream_t st)
{
    if (sf) launch_tile_s<ELSZ, 16, true>(sb, df, nt, p, grid, lds, st);
    else if (lb == 16) launch_tile_s<ELSZ, 16, false>(sb, df, nt, p, grid, lds, st);
    else if (lb == 8) launch_tile_s<ELSZ, 8, false>(sb, df, nt, p, grid, lds, st);
    else launch_tile_s<ELSZ, ELSZ, false>(sb, df, nt, p, grid, lds, st);
}

// Host replay of the tile kernel's index arithmetic for one workgroup: calls visit(src element
// offset, destination element offset) for every element the workgroup moves and vec(is_store,
// first element, elements) for every global vector access, and returns false if an LDS index
// falls outside the tile's allocation or an element read from LDS was never written.
template <int VL, int VS, bool SF, bool DF, typename F, typename G>
bool replay_tile(const TileParams &p, uint32_t block, size_t lds_elems, F &&visit, G &&vec)
{
    const TileOrigin o = tile_origin(p, block);
    const uint32_t nvl = SF ? (uint32_t)(p.TG * p.TB * p.TA) / VL : (uint32_t)(p.TG * p.TB) * (uint32_t)(p.TA / VL);
    const uint32_t nvs = DF ? (uint32_t)(p.TG * p.TA * p.TB) / VS : (uint32_t)(p.TG * p.TA) * (uint32_t)(p.TB / VS);
    std::vector<int64_t> from(lds_elems, -1);                    // LDS element -> source offset it holds
    for (uint32_t v = 0; v < nvl; ++v) {
        int64_t so;
        uint32_t li;
        if (!tile_load_slot<VL, SF>(p, o, v, &so, &li)) continue;
        vec(false, o.sb + so, VL);                               // the global vector access, for range and alignment
        for (int j = 0; j < VL; ++j) {
            if (li + j >= lds_elems) return false;
            from[li + j] = o.sb + so + j;
        }
    }
    for (uint32_t u = 0; u < nvs; ++u) {
        int64_t dof;
        uint32_t li[VS];
        if (!tile_store_slot<VS, DF>(p, o, u, &dof, li)) continue;
        vec(true, o.db + dof, VS);
        for (int j = 0; j < VS; ++j) {
            if (li[j] >= lds_elems || from[li[j]] < 0) return false;
            visit(from[li[j]], o.db + dof + j);
        }
    }
    return true;
}

// What one conversion launches: the kernel, its parameters and its grid.  Depends on the
// two bound layouts, the element size and the 16-byte alignment of the two buffers only.
struct TransformPlan {
    enum Kind { COPY, GENERAL, ROWS, TRANSPOSE } kind;
    int elsz, vb, lb, sb;
    unsigned blocks;
    size_t lds, bytes;
    bool sf, df;               // TRANSPOSE: flat source / destination side
    PermuteParams p;
    TileParams tp;
    GeneralParams gp;
};

static int64_t gcd64(int64_t a, int64_t b) { while (b) { const int64_t t = a % b; a = b; b = t; } return a; }

// Largest multiple of `unit` that is <= want (at least `unit`), preferring one that divides `ext`
// when such a multiple exists at no less than half of `want`.
static int64_t pick_extent(int64_t ext, int64_t want, int64_t unit)
{
    if (want >= ext) return ext;
    int64_t best = std::max<int64_t>(unit, want - want % unit);
    for (int64_t c = best; c >= unit && c * 2 >= want; c -= unit)
        if (ext % c == 0) return c;
    return best;
}

// Tile shape, flat sides and vector widths of the tile kernel for pieces A = pcs[ia] (contiguous in the
// source) and B = pcs[ib] (contiguous in the destination).
alt_status_t plan_tile(alt_handle_t h, int elsz, const std::vector<Piece> &pcs, int ia, int ib, const void *src, void *dst,
                       int64_t numel, TransformPlan *out)
{
    TransformPlan &t = *out;
    TileParams &p = t.tp;
    std::memset(&p, 0, sizeof p);
    p.src = src; p.dst = dst;
    const Piece A = pcs[ia], B = pcs[ib];
    if (A.ext > 0x3fffffff || B.ext > 0x3fffffff) return fail(h, ALT_UNSUPPORTED, "tensor too large for one launch");
    const int np = (int)pcs.size();
    std::vector<int64_t> sstr, dstr;
    for (int j = 0; j < np; ++j) {
        if (j != ia) sstr.push_back(pcs[j].ss);
        if (j != ib) dstr.push_back(pcs[j].ds);
    }
    t.lb = pick_vector_bytes(elsz, A.ext, sstr, src);
    t.sb = pick_vector_bytes(elsz, B.ext, dstr, dst);
    const int v16 = 16 / elsz;
    const int64_t block = A.ext * B.ext;
    // A side can be flat when the other piece follows without a gap there and every other piece starts
    // on a 16-byte boundary on that side.  It is taken flat where rows alone do not take 16-byte
    // vectors, and where the piece is short and no multiple of the square tile's edge (196 or 49
    // elements: cut into 64s it would leave narrow remainders, whole it gives one unbroken run).
    auto others_aligned = [&](bool source) {
        for (int j = 0; j < np; ++j)
            if (j != ia && j != ib && (source ? pcs[j].ss : pcs[j].ds) % v16) return false;
        return true;
    };
    // Tile budget: 16 KB (a 64 x 64 square of either element size where both sides are rows), less for
    // small tensors so that the launch still has several workgroups per compute unit, each with its
    // whole tile in flight; a flat side may take up to 32 KB to leave the other side runs of 128 bytes.
    int64_t budget = 16384;
    while (budget > 4096 && numel * elsz / budget < 768) budget /= 2;
    const int64_t E = budget / elsz;
    constexpr int64_t kEdge = 64;                             // edge of the square tile, elements
    const int64_t run = std::max<int64_t>(budget / 128 / elsz, 1);      // elements in 128 bytes (in 32 for the smallest tiles)
    auto awkward = [&](int64_t ext) { return budget == 16384 && ext > kEdge && ext <= 512 && ext % kEdge != 0; };
    const bool can_sf = (uintptr_t)src % 16 == 0 && B.ss == A.ext && block % v16 == 0 && others_aligned(true);
    const bool can_df = (uintptr_t)dst % 16 == 0 && A.ds == B.ext && block % v16 == 0 && others_aligned(false);
    t.sf = can_sf && (t.lb < 16 || awkward(A.ext));
    t.df = can_df && (t.sb < 16 || awkward(B.ext));
    int64_t TA = 0, TB = 0;
    int vl = 1, vs = 1;
    // Tile extents for a choice of flat sides; false when whole rows make the tile too large.
    auto shape = [&](bool sf, bool df) {
        vl = (sf ? 16 : t.lb) / elsz;
        vs = (df ? 16 : t.sb) / elsz;
        if (sf && df) {
            TA = A.ext; TB = B.ext;
        } else if (sf) {
            // whole rows of a; the tile's run of TB rows must be a whole number of 16-byte vectors
            TA = A.ext;
            TB = pick_extent(B.ext, std::max<int64_t>(E / TA, run), std::max<int64_t>(v16 / gcd64(v16, A.ext), vs));
        } else if (df) {
            TB = B.ext;
            TA = pick_extent(A.ext, std::max<int64_t>(E / TB, run), std::max<int64_t>(v16 / gcd64(v16, B.ext), vl));
        } else {
            // rows on both sides: a square of kEdge elements (fewer for small tensors), the other side
            // grown where a piece is shorter than the edge
            const int64_t esq = std::min<int64_t>(E, kEdge * kEdge);
            int64_t edge = kEdge;
            while (edge > 16 && edge * edge > esq) edge /= 2;
            TB = pick_extent(B.ext, std::max<int64_t>(edge, vs), vs);
            TA = pick_extent(A.ext, std::max<int64_t>(esq / TB, vl), vl);
            TB = pick_extent(B.ext, std::max<int64_t>(esq / TA, TB), vs);
        }
        return TA * TB * elsz <= 32768;
    };
    const bool want_sf = t.sf, want_df = t.df;
    if (!shape(want_sf, want_df)) {
        if (want_sf && want_df && shape(true, false)) t.df = false;
        else if (want_sf && want_df && shape(false, true)) t.sf = false;
        else {
            t.sf = t.df = false;
            if (!shape(false, false)) return fail(h, ALT_UNSUPPORTED, "internal: conversion tile too large");
        }
    }
    // A third tile dimension over an outer piece when the two pieces are taken whole and leave room
    int ig = -1;
    int64_t TG = 1;
    if (TA == A.ext && TB == B.ext && block * 2 <= E) {
        for (int j = np - 1; j >= 0 && ig < 0; --j) {
            if (j == ia || j == ib) continue;
            if (t.sf && pcs[j].ss != block) continue;
            if (t.df && pcs[j].ds != block) continue;
            ig = j;
        }
        if (ig >= 0) TG = pick_extent(pcs[ig].ext, E / block, 1);
    }
    p.TA = (int32_t)TA; p.TB = (int32_t)TB; p.TG = (int32_t)TG;
    p.ext_a = (int32_t)A.ext; p.ext_b = (int32_t)B.ext; p.ext_g = ig >= 0 ? (int32_t)pcs[ig].ext : 1;
    if (ig >= 0 && pcs[ig].ext > 0x3fffffff) return fail(h, ALT_UNSUPPORTED, "tensor too large for one launch");
    p.ss_b = B.ss; p.ds_a = A.ds;
    p.ss_g = ig >= 0 ? pcs[ig].ss : 0; p.ds_g = ig >= 0 ? pcs[ig].ds : 0;
    p.LD = t.sf ? (int32_t)TA : (int32_t)(TA | 1);            // flat: a plain copy of the run; else an odd pitch
    p.GS = p.LD * (int32_t)TB;
    t.lds = (size_t)p.GS * TG * elsz;
    if (t.lds > 64 * 1024) return fail(h, ALT_UNSUPPORTED, "internal: conversion tile exceeds LDS");
    p.tiles_a = (uint32_t)((A.ext + TA - 1) / TA);
    p.tiles_b = (uint32_t)((B.ext + TB - 1) / TB);
    p.tiles_g = (uint32_t)((p.ext_g + TG - 1) / TG);
    int64_t blocks = (int64_t)p.tiles_a * p.tiles_b * p.tiles_g;
    for (int j = 0; j < np; ++j) {
        if (j == ia || j == ib || j == ig) continue;
        if (pcs[j].ext > 0x7fffffff) return fail(h, ALT_UNSUPPORTED, "tensor too large for one launch");
        p.outer_ext[p.n_outer] = (uint32_t)pcs[j].ext;
        p.outer_ss[p.n_outer] = pcs[j].ss;
        p.outer_ds[p.n_outer] = pcs[j].ds;
        ++p.n_outer;
        blocks *= pcs[j].ext;
        if (blocks > 0x7fffffff) return fail(h, ALT_UNSUPPORTED, "tensor too large for one launch");
    }
    p.d_ra = make_fastdiv((uint32_t)(TA / vl));
    p.d_tb = make_fastdiv((uint32_t)TB);
    p.d_rb = make_fastdiv((uint32_t)(t.df ? TB : TB / vs));
    p.d_ta = make_fastdiv((uint32_t)TA);
    p.d_tiles_a = make_fastdiv(p.tiles_a);
    p.d_tiles_b = make_fastdiv(p.tiles_b);
    p.d_tiles_g = make_fastdiv(p.tiles_g);
    t.blocks = (unsigned)blocks;
    return ALT_OK;
}

alt_status_t plan_transform(alt_handle_t h, int elsz, const BoundLayout &ls, const void *src, const BoundLayout &ld,
                            void *dst, TransformPlan *out)
{
    TransformPlan &t = *out;
    t.elsz = elsz;
    const int64_t numel = ls.numel;
    t.bytes = (size_t)numel * elsz;
    std::vector<Piece> pcs;
    bool permutable = ls.separable && ld.separable && refine(ls, ld, &pcs) && (int)pcs.size() <= kMaxOuter + 2;
    if (permutable && numel >= ((int64_t)1 << 40)) permutable = false;
    if (!permutable) {
        t.kind = TransformPlan::GENERAL;
        t.gp.src = src; t.gp.dst = dst; t.gp.ls = ls; t.gp.ld = ld;
        for (int d = 0; d < ls.ndim; ++d) t.gp.it_shape[d] = ls.shape[d];
        t.gp.it_numel = numel;
        t.blocks = (unsigned)std::min<int64_t>((numel + kThreads - 1) / kThreads, 256 * 32);
        return ALT_OK;
    }
    if (pcs.size() <= 1) {                       // same placement: plain copy
        t.kind = TransformPlan::COPY;
        return ALT_OK;
    }
    // pieces are in destination order: the last one has ds = 1
    int ib = (int)pcs.size() - 1, ia = -1;
    for (int j = 0; j < (int)pcs.size(); ++j) if (pcs[j].ss == 1) ia = j;
    if (ia < 0 || pcs[ib].ds != 1) return fail(h, ALT_UNSUPPORTED, "internal: no unit-stride piece");

    PermuteParams &p = t.p;
    std::memset(&p, 0, sizeof p);
    p.src = src; p.dst = dst;
    const bool rows = ia == ib;
    if (rows) ib = (int)pcs.size() - 2;          // tile over the run and the next destination piece
    const Piece A = pcs[ia], B = pcs[ib];
    p.ext_a = A.ext; p.ext_b = B.ext;
    p.ss_a = A.ss; p.ds_a = A.ds; p.ss_b = B.ss; p.ds_b = B.ds;
    for (int j = 0; j < (int)pcs.size(); ++j) {
        if (j == ia || j == ib) continue;
        p.outer_ext[p.n_outer] = pcs[j].ext;
        p.outer_ss[p.n_outer] = pcs[j].ss;
        p.outer_ds[p.n_outer] = pcs[j].ds;
        ++p.n_outer;
    }
    std::vector<int64_t> sstr, dstr;
    for (int j = 0; j < (int)pcs.size(); ++j) {
        if (j != ia) sstr.push_back(pcs[j].ss);
        if (j != (rows ? ia : ib)) dstr.push_back(pcs[j].ds);
    }
    constexpr int64_t kTileElems = 4096;
    int64_t blocks = 0;
    if (rows) {
        t.kind = TransformPlan::ROWS;
        t.vb = std::min(pick_vector_bytes(elsz, A.ext, sstr, src), pick_vector_bytes(elsz, A.ext, dstr, dst));
        int vl = t.vb / elsz;
        int64_t TA = std::min<int64_t>(A.ext, kTileElems);
        TA -= TA % vl;
        if (TA == 0) TA = vl;
        int64_t TB = std::max<int64_t>(1, std::min<int64_t>(B.ext, kTileElems / TA));
        p.TA = (int)TA; p.TB = (int)TB;
        p.tiles_a = (A.ext + TA - 1) / TA;
        p.tiles_b = (B.ext + TB - 1) / TB;
        blocks = p.tiles_a * p.tiles_b;
        t.lds = 0;
    } else {
        t.kind = TransformPlan::TRANSPOSE;
        return plan_tile(h, elsz, pcs, ia, ib, src, dst, numel, &t);
    }
    for (int d = 0; d < p.n_outer; ++d) blocks *= p.outer_ext[d];
    if (blocks > 0x7fffffff) return fail(h, ALT_UNSUPPORTED, "tensor too large for one launch");
    t.blocks = (unsigned)blocks;
    return ALT_OK;
}

alt_status_t run_transform(alt_handle_t h, TransformPlan &t, const void *src, void *dst, hipStream_t st)
{
    if (!h->has_gpu) return fail(h, ALT_HIP_ERROR, "no GPU device available");
    switch (t.kind) {
        case TransformPlan::COPY:
            ALT_CHECK_HIP(h, hipMemcpyAsync(dst, src, t.bytes, hipMemcpyDeviceToDevice, st));
            return ALT_OK;
        case TransformPlan::GENERAL:
            t.gp.src = src; t.gp.dst = dst;
            if (t.elsz == 2) hipLaunchKernelGGL(permute_general_kernel<2>, dim3(t.blocks), dim3(kThreads), 0, st, t.gp);
            else hipLaunchKernelGGL(permute_general_kernel<4>, dim3(t.blocks), dim3(kThreads), 0, st, t.gp);
            break;
        case TransformPlan::ROWS:
            t.p.src = src; t.p.dst = dst;
            if (t.elsz == 2) launch_rows<2>(t.vb, t.bytes > kStreamingBytes, t.p, dim3(t.blocks), st);
            else launch_rows<4>(t.vb, t.bytes > kStreamingBytes, t.p, dim3(t.blocks), st);
            break;
        case TransformPlan::TRANSPOSE:
            t.tp.src = src; t.tp.dst = dst;
            if (t.elsz == 2) launch_tile<2>(t.lb, t.sb, t.sf, t.df, t.bytes > kStreamingBytes, t.tp, dim3(t.blocks), t.lds, st);
            else launch_tile<4>(t.lb, t.sb, t.sf, t.df, t.bytes > kStreamingBytes, t.tp, dim3(t.blocks), t.lds, st);
            break;
    }
    ALT_CHECK_HIP(h, hipGetLastError());
    return ALT_OK;
}

}  // namespace

// Shared with ops.hip (weight packing) and the tuner.
alt_status_t transform_bound(alt_handle_t h, int elsz, const BoundLayout &ls, const void *src,
                             const BoundLayout &ld, void *dst, hipStream_t st)
{
    if (!h->has_gpu) return fail(h, ALT_HIP_ERROR, "no GPU device available");
    TransformPlan t;
    alt_status_t s = plan_transform(h, elsz, ls, src, ld, dst, &t);
    if (s != ALT_OK) return s;
    return run_transform(h, t, src, dst, st);
}

}  // namespace alt

// Recent alt_layout_transform calls reduced to launch plans (the planning costs several
// microseconds of host time, more than most of these conversions take on the device).
struct alt_transform_memo {
    struct Entry {
        int dtype, ndim;
        unsigned sig;
        int64_t shape[ALT_MAX_RANK];
        alt_layout_t src, dst;
        alt::TransformPlan plan;
    };
    std::vector<Entry> entries;
    size_t next = 0;
};

namespace alt {
void transform_memo_free(alt_handle_t h)
{
    delete h->tmemo;
    h->tmemo = nullptr;
}
}  // namespace alt

using namespace alt;

extern "C" alt_status_t alt_layout_transform(alt_handle_t h, alt_dtype_t dtype, int ndim, const int64_t *shape,
                                             const alt_layout_t *src_layout, const void *src,
                                             const alt_layout_t *dst_layout, void *dst, void *stream)
{
    if (!h) return ALT_INVALID_ARG;
    if (!shape || !src_layout || !dst_layout || !src || !dst)
        return fail(h, ALT_INVALID_ARG, "alt_layout_transform: null argument");
    if (dtype != ALT_F32 && dtype != ALT_BF16) return fail(h, ALT_INVALID_ARG, "alt_layout_transform: bad dtype");
    if (src == dst) return fail(h, ALT_INVALID_ARG, "alt_layout_transform: src and dst must not overlap");
    if (ndim < 1 || ndim > ALT_MAX_RANK) return fail(h, ALT_INVALID_ARG, "alt_layout_transform: bad rank");
    if (!h->has_gpu) return fail(h, ALT_HIP_ERROR, "no GPU device available");
    const unsigned sig = (unsigned)(((uintptr_t)src & 15) | (((uintptr_t)dst & 15) << 4));
    if (h->tmemo) {
        for (auto &e : h->tmemo->entries)
            if (e.dtype == (int)dtype && e.ndim == ndim && e.sig == sig &&
                std::memcmp(e.shape, shape, sizeof(int64_t) * ndim) == 0 &&
                std::memcmp(&e.src, src_layout, sizeof(alt_layout_t)) == 0 &&
                std::memcmp(&e.dst, dst_layout, sizeof(alt_layout_t)) == 0) {
                const char *a = (const char *)src, *b = (const char *)dst;
                if ((a < b + e.plan.bytes) && (b < a + e.plan.bytes))
                    return fail(h, ALT_INVALID_ARG, "alt_layout_transform: src and dst must not overlap");
                return run_transform(h, e.plan, src, dst, (hipStream_t)stream);
            }
    }
    BoundLayout ls, ld;
    std::string err;
    alt_status_t s = bind_layout(src_layout, ndim, shape, &ls, &err);
    if (s != ALT_OK) return fail(h, s, "source layout: %s", err.c_str());
    s = bind_layout(dst_layout, ndim, shape, &ld, &err);
    if (s != ALT_OK) return fail(h, s, "destination layout: %s", err.c_str());
    const size_t bytes = (size_t)ls.numel * dtype_size(dtype);
    const char *a = (const char *)src, *b = (const char *)dst;
    if ((a < b + bytes) && (b < a + bytes))
        return fail(h, ALT_INVALID_ARG, "alt_layout_transform: src and dst must not overlap");
    alt_transform_memo::Entry e;
    e.dtype = (int)dtype; e.ndim = ndim; e.sig = sig;
    std::memset(e.shape, 0, sizeof e.shape);
    std::memcpy(e.shape, shape, sizeof(int64_t) * ndim);
    e.src = *src_layout; e.dst = *dst_layout;
    s = plan_transform(h, (int)dtype_size(dtype), ls, src, ld, dst, &e.plan);
    if (s != ALT_OK) return s;
    s = run_transform(h, e.plan, src, dst, (hipStream_t)stream);
    if (s != ALT_OK) return s;
    constexpr size_t kEntries = 32;
    if (!h->tmemo) h->tmemo = new alt_transform_memo();
    auto &v = h->tmemo->entries;
    if (v.size() < kEntries) v.push_back(e);
    else { v[h->tmemo->next] = e; h->tmemo->next = (h->tmemo->next + 1) % kEntries; }
    return ALT_OK;
}

namespace alt {
namespace {

template <int VL, int VS>
bool replay_flags(bool sf, bool df, const TileParams &p, uint32_t block, size_t lds_elems,
                  const std::function<void(int64_t, int64_t)> &visit, const std::function<void(bool, int64_t, int)> &vec)
{
    if (sf && df) return replay_tile<VL, VS, true, true>(p, block, lds_elems, visit, vec);
    if (sf) return replay_tile<VL, VS, true, false>(p, block, lds_elems, visit, vec);
    if (df) return replay_tile<VL, VS, false, true>(p, block, lds_elems, visit, vec);
    return replay_tile<VL, VS, false, false>(p, block, lds_elems, visit, vec);
}

template <int VL>
bool replay_vs(int vs, bool sf, bool df, const TileParams &p, uint32_t block, size_t lds_elems,
               const std::function<void(int64_t, int64_t)> &visit, const std::function<void(bool, int64_t, int)> &vec)
{
    switch (vs) {
        case 1: return replay_flags<VL, 1>(sf, df, p, block, lds_elems, visit, vec);
        case 2: return replay_flags<VL, 2>(sf, df, p, block, lds_elems, visit, vec);
        case 4: return replay_flags<VL, 4>(sf, df, p, block, lds_elems, visit, vec);
        case 8: return replay_flags<VL, 8>(sf, df, p, block, lds_elems, visit, vec);
    }
    return false;
}

bool replay_any(int vl, int vs, bool sf, bool df, const TileParams &p, uint32_t block, size_t lds_elems,
                const std::function<void(int64_t, int64_t)> &visit, const std::function<void(bool, int64_t, int)> &vec)
{
    switch (vl) {
        case 1: return replay_vs<1>(vs, sf, df, p, block, lds_elems, visit, vec);
        case 2: return replay_vs<2>(vs, sf, df, p, block, lds_elems, visit, vec);
        case 4: return replay_vs<4>(vs, sf, df, p, block, lds_elems, visit, vec);
        case 8: return replay_vs<8>(vs, sf, df, p, block, lds_elems, visit, vec);
    }
    return false;
}

}  // namespace
}  // namespace alt

extern "C" alt_status_t alt_layout_transform_pad(alt_handle_t h, alt_dtype_t dtype, int ndim, const int64_t *src_shape,
                                                 const alt_layout_t *src_layout, const void *src,
                                                 const int64_t *dst_shape, const alt_layout_t *dst_layout, void *dst,
                                                 void *stream)
{
    if (!h) return ALT_INVALID_ARG;
    if (!src_shape || !dst_shape || !src_layout || !dst_layout || !src || !dst)
        return fail(h, ALT_INVALID_ARG, "alt_layout_transform_pad: null argument");
    if (dtype != ALT_F32 && dtype != ALT_BF16) return fail(h, ALT_INVALID_ARG, "alt_layout_transform_pad: bad dtype");
    if (ndim < 1 || ndim > ALT_MAX_RANK) return fail(h, ALT_INVALID_ARG, "alt_layout_transform_pad: bad rank");
    BoundLayout ls, ld;
    std::string err;
    alt_status_t s = bind_layout(src_layout, ndim, src_shape, &ls, &err);
    if (s != ALT_OK) return fail(h, s, "source layout: %s", err.c_str());
    s = bind_layout(dst_layout, ndim, dst_shape, &ld, &err);
    if (s != ALT_OK) return fail(h, s, "destination layout: %s", err.c_str());
    const size_t elsz = dtype_size(dtype);
    const char *a = (const char *)src, *b = (const char *)dst;
    if ((a < b + (size_t)ld.numel * elsz) && (b < a + (size_t)ls.numel * elsz))
        return fail(h, ALT_INVALID_ARG, "alt_layout_transform_pad: src and dst must not overlap");
    if ((uintptr_t)src % elsz || (uintptr_t)dst % elsz)
        return fail(h, ALT_INVALID_ARG, "alt_layout_transform_pad: buffers are not aligned to the element size");
    if (!h->has_gpu) return fail(h, ALT_HIP_ERROR, "no GPU device available");
    GeneralParams gp;
    gp.src = src; gp.dst = dst; gp.ls = ls; gp.ld = ld;
    gp.it_numel = 1;
    bool grows = false;
    for (int d = 0; d < ndim; ++d) {
        gp.it_shape[d] = std::min(src_shape[d], dst_shape[d]);
        gp.it_numel *= gp.it_shape[d];
        grows |= dst_shape[d] > src_shape[d];
    }
    hipStream_t st = (hipStream_t)stream;
    if (grows) {
        const int64_t bytes = ld.numel * (int64_t)elsz;
        const unsigned blocks = (unsigned)std::min<int64_t>((bytes / 16 + kThreads) / kThreads, 256 * 16);
        hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(kThreads), 0, st, (char *)dst, bytes);
        ALT_CHECK_HIP(h, hipGetLastError());
    }
    const unsigned blocks = (unsigned)std::min<int64_t>((gp.it_numel + kThreads - 1) / kThreads, 256 * 32);
    if (elsz == 2) hipLaunchKernelGGL(permute_general_kernel<2>, dim3(blocks), dim3(kThreads), 0, st, gp);
    else hipLaunchKernelGGL(permute_general_kernel<4>, dim3(blocks), dim3(kThreads), 0, st, gp);
    ALT_CHECK_HIP(h, hipGetLastError());
    return ALT_OK;
}

extern "C" alt_status_t alt_layout_transform_plan(alt_handle_t h, alt_dtype_t dtype, int ndim, const int64_t *shape,
                                                  const alt_layout_t *src_layout, int src_misalign,
                                                  const alt_layout_t *dst_layout, int dst_misalign, int replay,
                                                  alt_transform_plan_t *out)
{
    if (!h) return ALT_INVALID_ARG;
    if (!shape || !src_layout || !dst_layout || !out) return fail(h, ALT_INVALID_ARG, "alt_layout_transform_plan: null argument");
    if (dtype != ALT_F32 && dtype != ALT_BF16) return fail(h, ALT_INVALID_ARG, "alt_layout_transform_plan: bad dtype");
    if (ndim < 1 || ndim > ALT_MAX_RANK) return fail(h, ALT_INVALID_ARG, "alt_layout_transform_plan: bad rank");
    const int elsz = (int)dtype_size(dtype);
    if (src_misalign < 0 || src_misalign > 15 || dst_misalign < 0 || dst_misalign > 15 || src_misalign % elsz || dst_misalign % elsz)
        return fail(h, ALT_INVALID_ARG, "alt_layout_transform_plan: misalignment must be a multiple of the element size below 16");
    BoundLayout ls, ld;
    std::string err;
    alt_status_t s = bind_layout(src_layout, ndim, shape, &ls, &err);
    if (s != ALT_OK) return fail(h, s, "source layout: %s", err.c_str());
    s = bind_layout(dst_layout, ndim, shape, &ld, &err);
    if (s != ALT_OK) return fail(h, s, "destination layout: %s", err.c_str());
    TransformPlan t;
    std::memset(&t, 0, sizeof t);
    // (only the addresses' low four bits enter the plan)
    s = plan_transform(h, elsz, ls, (const void *)(uintptr_t)(4096 + src_misalign), ld, (void *)(uintptr_t)(8192 + dst_misalign), &t);
    if (s != ALT_OK) return s;
    std::memset(out, 0, sizeof *out);
    out->kind = (int32_t)t.kind;
    out->mismatches = -1;
    out->workgroups = t.kind == TransformPlan::COPY ? 0 : (int64_t)t.blocks;
    if (t.kind == TransformPlan::ROWS) { out->load_bytes = out->store_bytes = t.vb; out->tile_a = t.p.TA; out->tile_b = t.p.TB; out->tile_g = 1; }
    if (t.kind != TransformPlan::TRANSPOSE) return ALT_OK;
    out->src_flat = t.sf; out->dst_flat = t.df;
    out->load_bytes = t.sf ? 16 : t.lb; out->store_bytes = t.df ? 16 : t.sb;
    out->tile_a = t.tp.TA; out->tile_b = t.tp.TB; out->tile_g = t.tp.TG;
    out->lds_bytes = (int64_t)t.lds;
    if (!replay) return ALT_OK;
    const int64_t numel = ls.numel;
    if (numel > ((int64_t)1 << 27)) return fail(h, ALT_UNSUPPORTED, "alt_layout_transform_plan: too many elements to replay on the host");
    // Every workgroup's moves, replayed: each destination element must be written exactly once, from
    // the source element the two layouts' index maps name.
    std::vector<int64_t> from((size_t)numel, -1);
    int64_t bad = 0;
    const std::function<void(int64_t, int64_t)> visit = [&](int64_t so, int64_t dof) {
        if (so < 0 || so >= numel || dof < 0 || dof >= numel || from[(size_t)dof] >= 0) { ++bad; return; }
        from[(size_t)dof] = so;
    };
    // every global vector access inside its buffer and aligned to its own size
    const std::function<void(bool, int64_t, int)> vec = [&](bool store, int64_t first, int n) {
        const int64_t addr = first * elsz + (store ? dst_misalign : src_misalign);
        if (first < 0 || first + n > numel || addr % ((int64_t)n * elsz)) ++bad;
    };
    const int vl = out->load_bytes / elsz, vs = out->store_bytes / elsz;
    for (uint32_t b = 0; b < t.blocks; ++b)
        if (!replay_any(vl, vs, t.sf, t.df, t.tp, b, t.lds / elsz, visit, vec)) ++bad;
    int64_t idx[ALT_MAX_RANK] = {0};
    for (int64_t e = 0; e < numel; ++e) {
        int64_t r = e;
        for (int d = ndim - 1; d >= 0; --d) { idx[d] = r % shape[d]; r /= shape[d]; }
        if (from[(size_t)eval_offset(ld, idx)] != eval_offset(ls, idx)) ++bad;
    }
    out->mismatches = bad;
    return ALT_OK;
}

extern "C" alt_status_t alt_unfold_shape(int ndim, const int64_t *shape, int dim, int64_t B, int64_t S, int64_t *out_shape)
{
    if (!shape || !out_shape || ndim < 1 || ndim >= ALT_MAX_RANK || dim < 0 || dim >= ndim || B < 1 || S < 1) return ALT_INVALID_ARG;
    for (int d = 0; d < ndim; ++d)
        if (shape[d] < 1) return ALT_INVALID_ARG;
    const int64_t D = shape[dim], num = D - B;
    const int64_t T = (num <= 0 ? 0 : (num + S - 1) / S) + 1;
    for (int d = 0, o = 0; d < ndim; ++d) {
        if (d == dim) { out_shape[o++] = T; out_shape[o++] = B; }
        else out_shape[o++] = shape[d];
    }
    return ALT_OK;
}

extern "C" alt_status_t alt_unfold(alt_handle_t h, alt_dtype_t dtype, int ndim, const int64_t *shape, int dim, int64_t B,
                                   int64_t S, const void *src, void *dst, void *stream)
{
    if (!h) return ALT_INVALID_ARG;
    if (dtype != ALT_F32 && dtype != ALT_BF16) return fail(h, ALT_INVALID_ARG, "alt_unfold: bad dtype");
    int64_t os[ALT_MAX_RANK];
    if (alt_unfold_shape(ndim, shape, dim, B, S, os) != ALT_OK) return fail(h, ALT_INVALID_ARG, "alt_unfold: bad shape, dimension, tile size or stride");
    if (!src || !dst) return fail(h, ALT_INVALID_ARG, "alt_unfold: null buffer");
    if (!h->has_gpu) return fail(h, ALT_HIP_ERROR, "no GPU device available");
    const int64_t esz = (int64_t)dtype_size(dtype);
    int64_t outer = 1, inner = 1;
    for (int d = 0; d < dim; ++d) outer *= shape[d];
    for (int d = dim + 1; d < ndim; ++d) inner *= shape[d];
    const int64_t D = shape[dim], T = os[dim];
    if (B > 0x7fffffff || T > 0x7fffffff || inner * esz > 0x7fffffff) return fail(h, ALT_UNSUPPORTED, "alt_unfold: extent too large");
    const int64_t out_bytes = outer * T * B * inner * esz, in_bytes = outer * D * inner * esz;
    const char *a = (const char *)src;
    char *b = (char *)dst;
    if (a < b + out_bytes && b < a + in_bytes) return fail(h, ALT_INVALID_ARG, "alt_unfold: src and dst must not overlap");
    const bool wide = (inner * esz) % 16 == 0 && (uintptr_t)src % 16 == 0 && (uintptr_t)dst % 16 == 0;
    const int vb = wide ? 16 : (int)esz;
    const uint32_t vec_inner = (uint32_t)(inner * esz / vb);
    const int64_t total = outer * T * B * vec_inner;
    const unsigned blocks = (unsigned)std::min<int64_t>((total + kThreads - 1) / kThreads, 256 * 32);
    hipStream_t st = (hipStream_t)stream;
    if (vb == 16) hipLaunchKernelGGL(unfold_kernel<16>, dim3(blocks), dim3(kThreads), 0, st, a, b, total, vec_inner, (uint32_t)B, (uint32_t)T, D, S);
    else if (vb == 4) hipLaunchKernelGGL(unfold_kernel<4>, dim3(blocks), dim3(kThreads), 0, st, a, b, total, vec_inner, (uint32_t)B, (uint32_t)T, D, S);
    else hipLaunchKernelGGL(unfold_kernel<2>, dim3(blocks), dim3(kThreads), 0, st, a, b, total, vec_inner, (uint32_t)B, (uint32_t)T, D, S);
    ALT_CHECK_HIP(h, hipGetLastError());
    return ALT_OK;
}

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

// Store that goes through to memory as it is written (sc0 + sc1) instead of leaving a dirty
// line in the XCD's L2 for the write-back at the end of the kernel: the output of a
// conversion is not read again by this kernel, and the shorter kernel end is what counts
// for these few-microsecond launches.
template <typename V>
__device__ __forceinline__ void store_through(char *addr, const V &w)
{
    typedef uint32_t w4_t __attribute__((ext_vector_type(4)));
    typedef uint32_t w2_t __attribute__((ext_vector_type(2)));
    if constexpr (sizeof(V) == 16) {
        const w4_t v = __builtin_bit_cast(w4_t, w);
        asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" : : "v"(addr), "v"(v) : "memory");
    } else if constexpr (sizeof(V) == 8) {
        const w2_t v = __builtin_bit_cast(w2_t, w);
        asm volatile("global_store_dwordx2 %0, %1, off sc0 sc1" : : "v"(addr), "v"(v) : "memory");
    } else if constexpr (sizeof(V) == 4) {
        const uint32_t v = __builtin_bit_cast(uint32_t, w);
        asm volatile("global_store_dword %0, %1, off sc0 sc1" : : "v"(addr), "v"(v) : "memory");
    } else {
        *(V *)addr = w;
    }
}

// Piece a is contiguous on both sides: copy TB runs of TA elements.
template <int ELSZ, int VBYTES>
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
        V w = *(const V *)(src + (sb + ib * p.ss_b + ia) * ELSZ);
        store_through(dst + (db + ib * p.ds_b + ia) * ELSZ, w);
    }
}

// Piece a is contiguous in the source, piece b in the destination.
template <int ELSZ, int LBYTES, int SBYTES>
__global__ __launch_bounds__(kThreads) void permute_transpose_kernel(PermuteParams p)
{
    using E = typename Word<ELSZ>::type;
    using VLd = typename Word<LBYTES>::type;
    using VSt = typename Word<SBYTES>::type;
    constexpr int VL = LBYTES / ELSZ, VS = SBYTES / ELSZ;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    E *tile = (E *)smem_raw;                        // [TB][LD], element (ib, ia) at ib*LD + ia
    int64_t sb, db, a0, b0;
    locate_tile(p, sb, db, a0, b0);
    const int ta = (int)min((int64_t)p.TA, p.ext_a - a0);
    const int tb = (int)min((int64_t)p.TB, p.ext_b - b0);
    const int LD = p.LD;
    const char *src = (const char *)p.src;
    char *dst = (char *)p.dst;
    {
        const int ra = ta / VL;
        for (int v = threadIdx.x; v < ra * tb; v += kThreads) {
            int ib = v / ra, ia = (v - ib * ra) * VL;
            VLd w = *(const VLd *)(src + (sb + ib * p.ss_b + ia) * ELSZ);
            const E *e = (const E *)&w;
#pragma unroll
            for (int j = 0; j < VL; ++j) tile[ib * LD + ia + j] = e[j];
        }
    }
    __syncthreads();
    {
        const int rb = tb / VS;
        for (int v = threadIdx.x; v < rb * ta; v += kThreads) {
            int ia = v / rb, ib = (v - ia * rb) * VS;
            VSt w;
            E *e = (E *)&w;
#pragma unroll
            for (int j = 0; j < VS; ++j) e[j] = tile[(ib + j) * LD + ia];
            store_through(dst + (db + ia * p.ds_a + ib) * ELSZ, w);
        }
    }
}

struct GeneralParams {
    const void *src;
    void *dst;
    BoundLayout ls, ld;
};

template <int ELSZ>
__global__ __launch_bounds__(kThreads) void permute_general_kernel(GeneralParams p)
{
    using E = typename Word<ELSZ>::type;
    const int64_t n = p.ls.numel;
    for (int64_t e = blockIdx.x * (int64_t)kThreads + threadIdx.x; e < n; e += (int64_t)gridDim.x * kThreads) {
        int64_t idx[ALT_MAX_RANK];
        int64_t r = e;
        for (int d = p.ls.ndim - 1; d >= 0; --d) { idx[d] = r % p.ls.shape[d]; r /= p.ls.shape[d]; }
        ((E *)p.dst)[eval_offset(p.ld, idx)] = ((const E *)p.src)[eval_offset(p.ls, idx)];
    }
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
        store_through(dst + v * VB, w);
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

template <int ELSZ>
void launch_rows(int vb, const PermuteParams &p, dim3 grid, hipStream_t st)
{
    if (vb == 16) hipLaunchKernelGGL((permute_rows_kernel<ELSZ, 16>), grid, dim3(kThreads), 0, st, p);
    else if (vb == 8) hipLaunchKernelGGL((permute_rows_kernel<ELSZ, 8>), grid, dim3(kThreads), 0, st, p);
    else hipLaunchKernelGGL((permute_rows_kernel<ELSZ, ELSZ>), grid, dim3(kThreads), 0, st, p);
}

template <int ELSZ, int LB>
void launch_transpose_s(int sb, const PermuteParams &p, dim3 grid, size_t lds, hipStream_t st)
{
    if (sb == 16) hipLaunchKernelGGL((permute_transpose_kernel<ELSZ, LB, 16>), grid, dim3(kThreads), lds, st, p);
    else if (sb == 8) hipLaunchKernelGGL((permute_transpose_kernel<ELSZ, LB, 8>), grid, dim3(kThreads), lds, st, p);
    else hipLaunchKernelGGL((permute_transpose_kernel<ELSZ, LB, ELSZ>), grid, dim3(kThreads), lds, st, p);
}

template <int ELSZ>
void launch_transpose(int lb, int sb, const PermuteParams &p, dim3 grid, size_t lds, hipStream_t st)
{
    if (lb == 16) launch_transpose_s<ELSZ, 16>(sb, p, grid, lds, st);
    else if (lb == 8) launch_transpose_s<ELSZ, 8>(sb, p, grid, lds, st);
    else launch_transpose_s<ELSZ, ELSZ>(sb, p, grid, lds, st);
}


// What one conversion launches: the kernel, its parameters and its grid.  Depends on the
// two bound layouts, the element size and the 16-byte alignment of the two buffers only.
struct TransformPlan {
    enum Kind { COPY, GENERAL, ROWS, TRANSPOSE } kind;
    int elsz, vb, lb, sb;
    unsigned blocks;
    size_t lds, bytes;
    PermuteParams p;
    GeneralParams gp;
};

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
        t.lb = pick_vector_bytes(elsz, A.ext, sstr, src);
        t.sb = pick_vector_bytes(elsz, B.ext, dstr, dst);
        int vl = t.lb / elsz, vs = t.sb / elsz;
        int64_t TA = std::min<int64_t>(A.ext, 64), TB = std::min<int64_t>(B.ext, 64);
        if (TA < 64) TB = std::min<int64_t>(B.ext, kTileElems / TA);
        else if (TB < 64) TA = std::min<int64_t>(A.ext, kTileElems / TB);
        TA -= TA % vl; if (TA == 0) TA = vl;
        TB -= TB % vs; if (TB == 0) TB = vs;
        p.TA = (int)TA; p.TB = (int)TB;
        p.LD = (int)TA | 1;                      // odd row pitch: conflict-free column reads
        p.tiles_a = (A.ext + TA - 1) / TA;
        p.tiles_b = (B.ext + TB - 1) / TB;
        blocks = p.tiles_a * p.tiles_b;
        t.lds = (size_t)p.LD * p.TB * elsz;
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
            if (t.elsz == 2) launch_rows<2>(t.vb, t.p, dim3(t.blocks), st);
            else launch_rows<4>(t.vb, t.p, dim3(t.blocks), st);
            break;
        case TransformPlan::TRANSPOSE:
            t.p.src = src; t.p.dst = dst;
            if (t.elsz == 2) launch_transpose<2>(t.lb, t.sb, t.p, dim3(t.blocks), t.lds, st);
            else launch_transpose<4>(t.lb, t.sb, t.p, dim3(t.blocks), t.lds, st);
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

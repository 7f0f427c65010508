// Internal declarations shared by the library's translation units.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <map>
#include <string>
#include <vector>

#include "../../include/alt.h"

namespace alt {

// ---- bound layouts ---------------------------------------------------------

// One piece of a physical dimension: digit (i[dim] / div) % ext, weighted by
// `stride` elements in memory.
struct Atom {
    int32_t dim;
    int32_t group;
    int64_t div;
    int64_t ext;
    int64_t stride;
};

// A layout bound to a concrete logical shape.  POD so that it can be passed to
// kernels by value.
struct BoundLayout {
    int32_t ndim;
    int32_t nsub;
    int32_t separable;
    int32_t nprims;
    int64_t shape[ALT_MAX_RANK];
    int64_t numel;
    Atom atom[ALT_MAX_RANK];            // outermost first (separable form)
    alt_prim_t prims[ALT_MAX_PRIMS];    // general form
};

alt_status_t bind_layout(const alt_layout_t *l, int ndim, const int64_t *shape, BoundLayout *out,
                         std::string *err);

// Two-level strided addressing of one logical dimension:
// off(i) = (i / f) * so + (i % f) * si.  An unsplit dimension has f = extent
// (so unused).  Everything conv/gemm kernels need to know about a layout.
// Division by a runtime constant without a divide: for 0 <= n < 2^31 and
// d >= 2, n / d == umulhi(n, mul) >> shift with mul = ceil(2^(32+shift) / d),
// shift = ceil(log2 d) - 1 (the rounding error n * (mul*d - 2^(32+shift)) stays
// below 2^(32+shift)); d == 1 is passed through.
struct FastDiv {
    uint32_t d, mul, shift, pad_;
};

inline FastDiv make_fastdiv(uint32_t d)
{
    FastDiv f{d, 0, 0, 0};
    if (d <= 1) return f;
    uint32_t l = 0;
    while (((uint64_t)1 << l) < d) ++l;                       // ceil(log2 d)
    const unsigned p = 31 + l;
    f.mul = (uint32_t)((((uint64_t)1 << p) + d - 1) / d);     // < 2^32
    f.shift = p - 32;
    return f;
}

__host__ __device__ inline uint32_t fast_div(uint32_t n, const FastDiv &f)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return f.d <= 1 ? n : (__umulhi(n, f.mul) >> f.shift);
#else
    return f.d <= 1 ? n : (uint32_t)(((uint64_t)n * f.mul) >> 32) >> f.shift;
#endif
}

struct Dim2 {
    int32_t f;
    int32_t pad_;
    int64_t so;
    int64_t si;
    FastDiv fd;        // of f
};

// Reduces a bound separable layout to one Dim2 per logical dimension; fails if
// a dimension is cut into more than two pieces.
bool layout_to_dim2(const BoundLayout &b, Dim2 *out /*[ndim]*/);

// ---- handle ------------------------------------------------------------------

struct TuneEntry {
    int variant;
    float us;
};

}  // namespace alt

struct alt_context {
    int device = -1;
    bool has_gpu = false;
    int compute_units = 0;
    int clock_mhz = 0;
    std::string arch;
    std::string last_error;
    std::map<std::string, alt::TuneEntry> cache;   // key -> tuned variant
    unsigned cache_gen = 0;                        // bumped whenever `cache` changes
    struct alt_launch_memo *memo = nullptr;        // ops.hip: recent descriptors reduced to launch parameters
    struct alt_transform_memo *tmemo = nullptr;    // transform.hip: recent conversions reduced to launch plans
};

namespace alt {

alt_status_t fail(alt_handle_t h, alt_status_t s, const char *fmt, ...);

#define ALT_CHECK_HIP(h, expr)                                                              \
    do {                                                                                    \
        hipError_t e_ = (expr);                                                             \
        if (e_ != hipSuccess)                                                               \
            return alt::fail((h), ALT_HIP_ERROR, "%s: %s", #expr, hipGetErrorString(e_));   \
    } while (0)

inline size_t dtype_size(int dt) { return dt == ALT_BF16 ? 2 : 4; }

void launch_memo_free(alt_handle_t h);       // ops.hip
void transform_memo_free(alt_handle_t h);    // transform.hip

// Cache keys (tune.cpp)
std::string conv_key(alt_handle_t h, const alt_conv_desc_t *d);
std::string gemm_key(alt_handle_t h, const alt_gemm_desc_t *d);
std::string layout_text(const alt_layout_t *l);

}  // namespace alt

// Separable layouts of four-dimensional tensors with fewer than 2^31 elements in a form
// kernels can walk with 32-bit arithmetic and divisions by multiplication: used by the
// kernels that prepare the operands of the transposed and the 3-D convolution.
#pragma once

#include "common.h"

namespace alt {

struct FastAtom {
    uint32_t dim, div, ext, stride;
    FastDiv by_div, by_ext, by_stride;
};
struct FastLayout {
    int32_t n, pad_;
    FastAtom a[ALT_MAX_RANK];
};
__device__ __forceinline__ uint32_t fast_mod(uint32_t n, const FastDiv &f) { return n - fast_div(n, f) * f.d; }

inline bool fast_layout(const BoundLayout &b, FastLayout *out)
{
    if (!b.separable || b.ndim != 4 || b.numel >= ((int64_t)1 << 31) || b.nsub > ALT_MAX_RANK) return false;
    out->n = b.nsub;
    out->pad_ = 0;
    for (int j = 0; j < b.nsub; ++j) {
        const Atom &a = b.atom[j];
        if (a.div >= ((int64_t)1 << 31) || a.ext >= ((int64_t)1 << 31) || a.stride >= ((int64_t)1 << 31) || a.stride < 1) return false;
        FastAtom &f = out->a[j];
        f.dim = (uint32_t)a.dim; f.div = (uint32_t)a.div; f.ext = (uint32_t)a.ext; f.stride = (uint32_t)a.stride;
        f.by_div = make_fastdiv(f.div); f.by_ext = make_fastdiv(f.ext); f.by_stride = make_fastdiv(f.stride);
    }
    return true;
}

// The piece of a bound layout that is contiguous in memory (stride 1), or null.
inline const Atom *unit_stride_atom(const BoundLayout &b)
{
    const Atom *r = nullptr;
    for (int j = 0; j < b.nsub; ++j) if (b.atom[j].stride == 1) r = &b.atom[j];
    return r;
}

}  // namespace alt

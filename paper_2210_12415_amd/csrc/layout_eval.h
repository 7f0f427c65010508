// Offset of a logical index under a bound layout, usable on host and device.
// Separable layouts sum one digit per piece; general layouts replay the
// primitive sequence on the index vector (Table 1 of the paper: split takes
// mixed-radix digits of one index, reorder permutes, fuse linearises).
#pragma once

#include "common.h"

namespace alt {

__host__ __device__ inline int64_t eval_separable(const BoundLayout &b, const int64_t *idx)
{
    int64_t off = 0;
    for (int j = 0; j < b.nsub; ++j) {
        const Atom &a = b.atom[j];
        off += ((idx[a.dim] / a.div) % a.ext) * a.stride;
    }
    return off;
}

// Replays b.prims on (shape, idx); returns the row-major offset under the
// transformed shape.  The caller guarantees the sequence was validated.
__host__ __device__ inline int64_t eval_general(const BoundLayout &b, const int64_t *idx_in)
{
    int64_t sh[ALT_MAX_RANK + 4], ix[ALT_MAX_RANK + 4], sh2[ALT_MAX_RANK + 4], ix2[ALT_MAX_RANK + 4];
    int rank = b.ndim;
    for (int d = 0; d < rank; ++d) { sh[d] = b.shape[d]; ix[d] = idx_in[d]; }
    for (int q = 0; q < b.nprims; ++q) {
        const alt_prim_t &p = b.prims[q];
        int r = 0;
        if (p.kind == ALT_PRIM_SPLIT) {
            for (int d = 0; d < p.dim; ++d) { sh2[r] = sh[d]; ix2[r] = ix[d]; ++r; }
            int64_t rem = ix[p.dim];
            int64_t below = sh[p.dim];
            for (int j = 0; j < p.count; ++j) {
                below /= p.v[j];                 // product of the factors after j
                sh2[r] = p.v[j];
                ix2[r] = rem / below;
                rem -= ix2[r] * below;
                ++r;
            }
            for (int d = p.dim + 1; d < rank; ++d) { sh2[r] = sh[d]; ix2[r] = ix[d]; ++r; }
        } else if (p.kind == ALT_PRIM_REORDER) {
            for (int j = 0; j < rank; ++j) { sh2[j] = sh[p.v[j]]; ix2[j] = ix[p.v[j]]; }
            r = rank;
        } else {
            for (int d = 0; d < p.dim; ++d) { sh2[r] = sh[d]; ix2[r] = ix[d]; ++r; }
            int64_t e = 1, lin = 0;
            for (int d = p.dim; d < p.dim + p.count; ++d) { lin = lin * sh[d] + ix[d]; e *= sh[d]; }
            sh2[r] = e; ix2[r] = lin; ++r;
            for (int d = p.dim + p.count; d < rank; ++d) { sh2[r] = sh[d]; ix2[r] = ix[d]; ++r; }
        }
        rank = r;
        for (int d = 0; d < rank; ++d) { sh[d] = sh2[d]; ix[d] = ix2[d]; }
    }
    int64_t off = 0;
    for (int d = 0; d < rank; ++d) off = off * sh[d] + ix[d];
    return off;
}

__host__ __device__ inline int64_t eval_offset(const BoundLayout &b, const int64_t *idx)
{
    return b.separable ? eval_separable(b, idx) : eval_general(b, idx);
}

}  // namespace alt

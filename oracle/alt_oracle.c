/*
 * CPU oracle for layout index maps, the layout conversion operator, 2-D
 * convolution and matrix multiplication.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is the slow, plain definition that the
 * GPU library is checked against; only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it.  It shares no code with the GPU
 * library and includes none of its headers.
 *
 * What it follows (paper: "ALT: Breaking the Wall between Graph and Operator
 * Level Optimizations for Deep Learning Compilation"):
 *   - basic layout primitives split / reorder / fuse: Table 1 and the worked
 *     sequences of Section 4.1.1;
 *   - unfold (overlapped tiling): Section 4.1.2 and Eq. 1;
 *   - the layout conversion operator: Section 4.2 (an element copy under two
 *     index maps);
 *   - C2D: the multiply-accumulate of the program in Fig. 3 (cross-correlation,
 *     no kernel flip) with zero padding as in Section 4.2;
 *   - GMM: C = A B, Section 5.1.
 * Layouts never change a mathematical result (Section 4.1.1: the basic
 * primitives are one-to-one), so conv and gemm are the textbook definitions on
 * logical NCHW / OIHW / row-major tensors, accumulated in double precision and
 * rounded once; other layouts are reached by composing with the conversion
 * operator below.
 *
 * Parity pins (tests/test_oracle_*.py): printed examples of Section 4.1.1 and
 * 4.1.2, closed forms, bijection checks, numpy transposes, delta-kernel and
 * all-ones convolutions, an independently written im2col product, library
 * matmul.  Nothing here is "parity unpinned" except the paper's speedup
 * figures, which are not computed at all.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_MAX_RANK 12

/* One layout primitive (Table 1).
 *   kind 0  split  : dimension k is replaced by m dimensions with extents
 *                    v[0..m-1] (outermost first); their product must equal the
 *                    extent of k.
 *   kind 1  reorder: new dimension j is old dimension v[j], j = 0..m-1.
 *   kind 2  fuse   : dimensions k .. k+m-1 become one dimension.
 * Dimension numbers are 0-based here; the paper's examples are 1-based. */
typedef struct {
    int32_t kind;
    int32_t k;
    int32_t m;
    int32_t pad_;
    int64_t v[8];
} orc_prim_t;

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Apply a primitive sequence to (shape, idx) in place.  Returns the new rank,
 * or -1 for a malformed primitive.  idx may be NULL to transform only the
 * shape. */
static int apply_prims(int rank, int64_t *shape, int64_t *idx,
                       const orc_prim_t *p, int np)
{
    int64_t s2[ORC_MAX_RANK], i2[ORC_MAX_RANK];
    for (int q = 0; q < np; ++q) {
        const orc_prim_t *pr = &p[q];
        if (pr->kind == 0) {                       /* split */
            int k = pr->k, m = pr->m;
            if (k < 0 || k >= rank || m < 1 || m > 8 || rank + m - 1 > ORC_MAX_RANK) return -1;
            int64_t prod = 1;
            for (int j = 0; j < m; ++j) { if (pr->v[j] < 1) return -1; prod *= pr->v[j]; }
            if (prod != shape[k]) return -1;
            int r = 0;
            for (int d = 0; d < k; ++d) { s2[r] = shape[d]; if (idx) i2[r] = idx[d]; ++r; }
            for (int j = 0; j < m; ++j) {
                /* i_k / (F_{j+1} ... F_m)  mod  F_j */
                int64_t below = 1;
                for (int t = j + 1; t < m; ++t) below *= pr->v[t];
                s2[r] = pr->v[j];
                if (idx) i2[r] = (idx[k] / below) % pr->v[j];
                ++r;
            }
            for (int d = k + 1; d < rank; ++d) { s2[r] = shape[d]; if (idx) i2[r] = idx[d]; ++r; }
            rank = r;
        } else if (pr->kind == 1) {                /* reorder */
            if (pr->m != rank) return -1;
            int seen[ORC_MAX_RANK] = {0};
            for (int j = 0; j < rank; ++j) {
                int64_t o = pr->v[j];
                if (o < 0 || o >= rank || seen[o]) return -1;
                seen[o] = 1;
                s2[j] = shape[o];
                if (idx) i2[j] = idx[o];
            }
        } else if (pr->kind == 2) {                /* fuse */
            int k = pr->k, m = pr->m;
            if (k < 0 || m < 1 || k + m > rank) return -1;
            int r = 0;
            for (int d = 0; d < k; ++d) { s2[r] = shape[d]; if (idx) i2[r] = idx[d]; ++r; }
            int64_t ext = 1, lin = 0;
            for (int d = k; d < k + m; ++d) {
                ext *= shape[d];
                if (idx) lin = lin * shape[d] + idx[d];   /* row-major over the fused dims */
            }
            s2[r] = ext; if (idx) i2[r] = lin; ++r;
            for (int d = k + m; d < rank; ++d) { s2[r] = shape[d]; if (idx) i2[r] = idx[d]; ++r; }
            rank = r;
        } else {
            return -1;
        }
        memcpy(shape, s2, sizeof(int64_t) * rank);
        if (idx) memcpy(idx, i2, sizeof(int64_t) * rank);
    }
    return rank;
}

/* Physical shape of a tensor of logical `shape` after the sequence.  Returns
 * the physical rank or -1. */
int orc_layout_shape(int rank, const int64_t *shape, const orc_prim_t *p, int np,
                     int64_t *out_shape)
{
    int64_t s[ORC_MAX_RANK];
    if (rank < 1 || rank > 8) return -1;
    memcpy(s, shape, sizeof(int64_t) * rank);
    int r = apply_prims(rank, s, NULL, p, np);
    if (r < 0) return -1;
    memcpy(out_shape, s, sizeof(int64_t) * r);
    return r;
}

/* Transformed index of one logical index (the "accessing expression" column of
 * Table 1) and its row-major offset under the transformed shape.  Returns the
 * offset or -1. */
int64_t orc_layout_offset(int rank, const int64_t *shape, const orc_prim_t *p, int np,
                          const int64_t *idx, int64_t *out_idx)
{
    int64_t s[ORC_MAX_RANK], i[ORC_MAX_RANK];
    if (rank < 1 || rank > 8) return -1;
    for (int d = 0; d < rank; ++d)
        if (idx[d] < 0 || idx[d] >= shape[d]) return -1;
    memcpy(s, shape, sizeof(int64_t) * rank);
    memcpy(i, idx, sizeof(int64_t) * rank);
    int r = apply_prims(rank, s, i, p, np);
    if (r < 0) return -1;
    int64_t off = 0;
    for (int d = 0; d < r; ++d) off = off * s[d] + i[d];
    if (out_idx) memcpy(out_idx, i, sizeof(int64_t) * r);
    return off;
}

/* Offsets of every logical index, in logical row-major order. */
int orc_layout_offsets_all(int rank, const int64_t *shape, const orc_prim_t *p, int np,
                           int64_t *out)
{
    int64_t idx[ORC_MAX_RANK] = {0};
    int64_t n = 1;
    for (int d = 0; d < rank; ++d) n *= shape[d];
    for (int64_t e = 0; e < n; ++e) {
        int64_t off = orc_layout_offset(rank, shape, p, np, idx, NULL);
        if (off < 0) return -1;
        out[e] = off;
        for (int d = rank - 1; d >= 0; --d) { if (++idx[d] < shape[d]) break; idx[d] = 0; }
    }
    return 0;
}

/* Layout conversion operator: dst[off_dst(i)] = src[off_src(i)] for every
 * logical index i.  Words of elsize 2 or 4 bytes are moved as integers. */
int orc_layout_transform(int elsize, int rank, const int64_t *shape,
                         const orc_prim_t *ps, int nps, const void *src,
                         const orc_prim_t *pd, int npd, void *dst)
{
    if (elsize != 2 && elsize != 4) return -1;
    int64_t outer = shape[0], inner = 1;
    for (int d = 1; d < rank; ++d) inner *= shape[d];
    int bad = 0;
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < outer; ++o) {
        int64_t idx[ORC_MAX_RANK] = {0};
        idx[0] = o;
        for (int64_t e = 0; e < inner; ++e) {
            int64_t a = orc_layout_offset(rank, shape, ps, nps, idx, NULL);
            int64_t b = orc_layout_offset(rank, shape, pd, npd, idx, NULL);
            if (a < 0 || b < 0) { bad = 1; break; }
            if (elsize == 2) ((uint16_t *)dst)[b] = ((const uint16_t *)src)[a];
            else             ((uint32_t *)dst)[b] = ((const uint32_t *)src)[a];
            for (int d = rank - 1; d >= 1; --d) { if (++idx[d] < shape[d]) break; idx[d] = 0; }
        }
    }
    return bad ? -1 : 0;
}

/* ---- unfold: overlapped tiling of one dimension (Section 4.1.2) -------- */

/* Number of tiles for extent D, tile size B, stride S: ceil((D-B)/S) + 1. */
int64_t orc_unfold_tiles(int64_t D, int64_t B, int64_t S)
{
    int64_t num = D - B;
    int64_t q = num <= 0 ? 0 : (num + S - 1) / S;
    return q + 1;
}

/* 1-D unfold: dst[t][b] = src[t*S + b], zero where t*S + b >= D. */
void orc_unfold_1d(const double *src, int64_t D, int64_t B, int64_t S, double *dst)
{
    int64_t T = orc_unfold_tiles(D, B, S);
    for (int64_t t = 0; t < T; ++t)
        for (int64_t b = 0; b < B; ++b) {
            int64_t e = t * S + b;
            dst[t * B + b] = e < D ? src[e] : 0.0;
        }
}

/* Eq. 1: the access T[V*i + r] (window i, in-window offset r, window size M)
 * becomes T'[tile][within] on the unfolded dimension. */
void orc_unfold_access(int64_t V, int64_t i, int64_t r, int64_t B, int64_t S, int64_t M,
                       int64_t *tile, int64_t *within)
{
    int64_t per_tile = (B - M) / V + 1;       /* windows that fit in one tile */
    *tile = i / per_tile;
    *within = V * i + r - S * (*tile);
}

/* ---- bf16 ---------------------------------------------------------------- */

static inline float bf16_to_f32(uint16_t u)
{
    uint32_t w = (uint32_t)u << 16;
    float f;
    memcpy(&f, &w, 4);
    return f;
}

uint16_t orc_f32_to_bf16(float f)
{
    uint32_t w;
    memcpy(&w, &f, 4);
    if ((w & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((w >> 16) | 0x40u);   /* NaN */
    uint32_t keep = w >> 16, rest = w & 0xFFFFu;
    if (rest > 0x8000u || (rest == 0x8000u && (keep & 1u))) keep += 1;           /* ties to even */
    return (uint16_t)keep;
}

static inline double load_el(const void *p, int64_t i, int is_bf16)
{
    return is_bf16 ? (double)bf16_to_f32(((const uint16_t *)p)[i])
                   : (double)((const float *)p)[i];
}

static inline void store_el(void *p, int64_t i, int is_bf16, double acc)
{
    float f = (float)acc;                              /* one rounding to fp32 */
    if (is_bf16) ((uint16_t *)p)[i] = orc_f32_to_bf16(f);
    else         ((float *)p)[i] = f;
}

/* ---- C2D ----------------------------------------------------------------- */

typedef struct {
    int64_t N, C, H, W, K, R, S;
    int64_t stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
    int32_t in_bf16;      /* x and w element type: 0 = fp32, 1 = bf16 bits */
    int32_t out_bf16;     /* y element type */
    int32_t has_bias;     /* bias is fp32[K] */
    int32_t relu;
} orc_conv_t;

int64_t orc_conv_out_h(const orc_conv_t *c)
{
    return (c->H + 2 * c->pad_h - c->dil_h * (c->R - 1) - 1) / c->stride_h + 1;
}
int64_t orc_conv_out_w(const orc_conv_t *c)
{
    return (c->W + 2 * c->pad_w - c->dil_w * (c->S - 1) - 1) / c->stride_w + 1;
}

/* One output element: sum over (c, r, s) of x[n,c,ih,iw] * w[k,c,r,s] with
 * zeros outside the input; then bias and ReLU. */
static double conv_point(const orc_conv_t *c, const void *x, const void *w, const float *bias,
                         int64_t n, int64_t k, int64_t oh, int64_t ow)
{
    double acc = 0.0;
    for (int64_t ci = 0; ci < c->C; ++ci)
        for (int64_t r = 0; r < c->R; ++r) {
            int64_t ih = oh * c->stride_h - c->pad_h + r * c->dil_h;
            if (ih < 0 || ih >= c->H) continue;
            for (int64_t s = 0; s < c->S; ++s) {
                int64_t iw = ow * c->stride_w - c->pad_w + s * c->dil_w;
                if (iw < 0 || iw >= c->W) continue;
                double xv = load_el(x, ((n * c->C + ci) * c->H + ih) * c->W + iw, c->in_bf16);
                double wv = load_el(w, ((k * c->C + ci) * c->R + r) * c->S + s, c->in_bf16);
                acc += xv * wv;
            }
        }
    if (c->has_bias) acc += (double)bias[k];
    if (c->relu && acc < 0.0) acc = 0.0;
    return acc;
}

/* x: NCHW, w: OIHW (= K C R S), y: N K OH OW, all dense row-major. */
int orc_conv2d(const orc_conv_t *c, const void *x, const void *w, const float *bias, void *y)
{
    int64_t OH = orc_conv_out_h(c), OW = orc_conv_out_w(c);
    if (OH < 1 || OW < 1) return -1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < c->N; ++n)
        for (int64_t k = 0; k < c->K; ++k)
            for (int64_t oh = 0; oh < OH; ++oh)
                for (int64_t ow = 0; ow < OW; ++ow) {
                    double acc = conv_point(c, x, w, bias, n, k, oh, ow);
                    store_el(y, ((n * c->K + k) * OH + oh) * OW + ow, c->out_bf16, acc);
                }
    return 0;
}

/* Selected outputs only: flat[i] indexes y as N K OH OW row-major; out[i] gets
 * the double-precision value before the final rounding. */
int orc_conv2d_at(const orc_conv_t *c, const void *x, const void *w, const float *bias,
                  const int64_t *flat, int64_t count, double *out)
{
    int64_t OH = orc_conv_out_h(c), OW = orc_conv_out_w(c);
    if (OH < 1 || OW < 1) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        int64_t e = flat[i];
        int64_t ow = e % OW; e /= OW;
        int64_t oh = e % OH; e /= OH;
        int64_t k = e % c->K; e /= c->K;
        out[i] = conv_point(c, x, w, bias, e, k, oh, ow);
    }
    return 0;
}

/* ---- GMM ----------------------------------------------------------------- */

/* A: [batch][M][K], B: [batch][K][N], C: [batch][M][N], dense row-major. */
int orc_gemm(int64_t batch, int64_t M, int64_t N, int64_t K, int in_bf16, int out_bf16,
             const void *A, const void *B, void *C)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t b = 0; b < batch; ++b)
        for (int64_t m = 0; m < M; ++m)
            for (int64_t n = 0; n < N; ++n) {
                double acc = 0.0;
                for (int64_t k = 0; k < K; ++k)
                    acc += load_el(A, (b * M + m) * K + k, in_bf16) *
                           load_el(B, (b * K + k) * N + n, in_bf16);
                store_el(C, (b * M + m) * N + n, out_bf16, acc);
            }
    return 0;
}

/* Selected outputs of the product, double precision, flat index over
 * [batch][M][N]. */
int orc_gemm_at(int64_t batch, int64_t M, int64_t N, int64_t K, int in_bf16,
                const void *A, const void *B, const int64_t *flat, int64_t count, double *out)
{
    (void)batch;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        int64_t e = flat[i];
        int64_t n = e % N; e /= N;
        int64_t m = e % M; e /= M;
        double acc = 0.0;
        for (int64_t k = 0; k < K; ++k)
            acc += load_el(A, (e * M + m) * K + k, in_bf16) *
                   load_el(B, (e * K + k) * N + n, in_bf16);
        out[i] = acc;
    }
    return 0;
}

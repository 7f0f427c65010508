/*
 * alt.h — C ABI of the MI355X (gfx950) tensor-operator library: 2-D
 * convolution and matrix multiplication executed under explicit tensor data
 * layouts, the layout conversion operator, and an on-device tuner over
 * {layout, kernel tile configuration}.
 *
 * The operations follow "ALT: Breaking the Wall between Graph and Operator
 * Level Optimizations for Deep Learning Compilation" (arXiv 2210.12415);
 * every entry point cites the passage that defines what it computes.
 *
 * Conventions
 *  - Plain C.  Every call returns alt_status_t; 0 is success.  No exception
 *    crosses the boundary.  alt_last_error(h) returns a string owned by the
 *    handle, valid until the next call on that handle.
 *  - "device pointer" = memory of the GPU that was current when the handle was
 *    created.  The caller owns every tensor buffer, the workspace and the
 *    stream.  `stream` is a hipStream_t passed as void* (NULL = default
 *    stream).  Calls that take a stream only enqueue work on it and return;
 *    the alt_tune_* calls synchronise.
 *  - The library never allocates device memory: split-K partial sums live in
 *    the caller's workspace, the tuner's scratch tensors in the caller's arena.
 *  - Tensors are addressed through a *logical* index and a layout.  Logical
 *    dimension order is fixed per operand: activations (N, C, H, W), weights
 *    (O, I, H, W) = (K, C, R, S), outputs (N, K, OH, OW); matrices A (M, K),
 *    B (K, N), C (M, N), with an optional dense outermost batch.
 *  - Element types: ALT_F32 (IEEE binary32) and ALT_BF16 (bfloat16 bit
 *    patterns in 16-bit words).  Products are accumulated in fp32.
 *  - Kernel arguments: these kernels run for a few microseconds, and with the
 *    HIP runtime's default (kernel arguments in host memory) every workgroup's
 *    first loads cross the host link, which costs each launch 2-5 us.  Set
 *    HIP_FORCE_DEV_KERNARG=1 in the environment before the process makes its
 *    first HIP call; the library cannot do it (the runtime reads the variable
 *    once, when it starts).  The Python binding sets it on import if unset.
 */
#ifndef ALT_H_
#define ALT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif
#if defined(__GNUC__)
#pragma GCC visibility push(default)   /* the entry points below are the library's only exports */
#endif

typedef enum {
    ALT_OK = 0,
    ALT_INVALID_ARG = 1,          /* null pointer, bad enum, non-positive size */
    ALT_INVALID_LAYOUT = 2,       /* unparsable string / malformed primitive */
    ALT_SHAPE_MISMATCH = 3,       /* layout does not tile the given shape exactly */
    ALT_UNSUPPORTED = 4,          /* valid request no kernel covers */
    ALT_WORKSPACE_TOO_SMALL = 5,
    ALT_HIP_ERROR = 6,            /* a HIP runtime call failed; see alt_last_error */
    ALT_NOT_TUNED = 7             /* cache lookup found no entry */
} alt_status_t;

typedef enum { ALT_F32 = 0, ALT_BF16 = 1 } alt_dtype_t;

typedef struct alt_context *alt_handle_t;

#define ALT_MAX_RANK 8            /* most logical or physical dimensions */
#define ALT_MAX_PRIMS 8           /* longest primitive sequence kept */

/* ---- layout primitives (Table 1 of the paper) --------------------------- */

typedef enum { ALT_PRIM_SPLIT = 0, ALT_PRIM_REORDER = 1, ALT_PRIM_FUSE = 2 } alt_prim_kind_t;

/* One primitive.  Dimension numbers are 0-based (the paper's examples count
 * from 1).
 *   SPLIT  : dimension `dim` becomes `count` dimensions with extents
 *            v[0..count-1], outermost first; their product must equal the
 *            extent being split.
 *   REORDER: count = current rank; new dimension j is old dimension v[j].
 *   FUSE   : dimensions dim .. dim+count-1 become one (row-major). */
typedef struct {
    int32_t kind;
    int32_t dim;
    int32_t count;
    int32_t reserved;
    int64_t v[ALT_MAX_RANK];
} alt_prim_t;

/* A layout: where each logical index lives in memory.  Plain data, copied by
 * value, no pointers.
 *
 * Separable form (separable = 1): the physical dimensions, outermost first,
 * are `nsub` pieces; piece j takes digit (i[sub_dim[j]] / sub_div[j]) mod
 * sub_extent[j] of one logical index.  sub_extent = 0 means "the rest": the
 * logical extent divided by sub_div (the outermost piece of that dimension).
 * Pieces with the same sub_group were fused into one physical dimension.
 * Every layout that alt_layout_parse accepts, and every split/reorder
 * sequence, has this form.
 *
 * General form (separable = 0): a sequence containing a fuse that is later
 * split across the old dimension boundaries (the N(O/4)(HW)4 example of
 * Section 4.1.1).  Only `prims`/`shape` describe it; it is bound to that
 * shape.  Index math and the conversion operator accept it; conv and gemm do
 * not. */
typedef struct {
    int32_t ndim;                         /* logical rank */
    int32_t nsub;                         /* number of pieces (separable form) */
    int32_t separable;
    int32_t nprims;                       /* > 0 only when built from primitives */
    int32_t sub_dim[ALT_MAX_RANK];
    int32_t sub_group[ALT_MAX_RANK];
    int64_t sub_div[ALT_MAX_RANK];
    int64_t sub_extent[ALT_MAX_RANK];
    int64_t shape[ALT_MAX_RANK];          /* logical shape the primitives were given for */
    alt_prim_t prims[ALT_MAX_PRIMS];
} alt_layout_t;

/* ---- lifecycle ----------------------------------------------------------- */

/* Creates a handle bound to the current HIP device.  With no usable GPU the
 * handle is still created (layout index math and argument checking work) and
 * every call that would launch a kernel returns ALT_HIP_ERROR. */
alt_status_t alt_create(alt_handle_t *out);
alt_status_t alt_destroy(alt_handle_t h);
const char *alt_last_error(alt_handle_t h);
const char *alt_status_string(alt_status_t s);
/* Library version, "major.minor". */
const char *alt_version(void);

/* ---- layouts: index math (Table 1; worked sequences of Section 4.1.1) ---- */

/* Parses "LOGICAL->PHYSICAL", e.g. "NCHW->NHWC", "NCHW->NCHW16c",
 * "OIHW->OIHW16i32o", "OIHW->OHWI", "MK->KM", "KN->KN64k32n".  Upper-case
 * letters name logical dimensions; in PHYSICAL an upper-case letter is the
 * outermost piece of that dimension and <factor><lower-case letter> an inner
 * block of that extent, exactly the N(O/o_t)HWo_t notation of the paper.  The
 * result is shape-independent. */
alt_status_t alt_layout_parse(const char *text, alt_layout_t *out);

/* Builds a layout from a primitive sequence applied to a tensor of logical
 * `shape` (host pointers).  At most ALT_MAX_PRIMS primitives and ALT_MAX_RANK
 * dimensions at any point of the sequence. */
alt_status_t alt_layout_from_prims(int ndim, const int64_t *shape, const alt_prim_t *seq,
                                   int nseq, alt_layout_t *out);

/* Physical shape of a tensor of logical `shape` under `l`; out_shape must
 * hold ALT_MAX_RANK entries.  ALT_SHAPE_MISMATCH if a block factor does not
 * divide its dimension. */
alt_status_t alt_layout_physical_shape(const alt_layout_t *l, const int64_t *shape,
                                       int64_t *out_shape, int *out_rank);

/* Element offset (row-major under the physical shape) of logical index `idx`. */
alt_status_t alt_layout_offset(const alt_layout_t *l, const int64_t *shape, const int64_t *idx,
                               int64_t *out_offset);

/* Inverse map: logical index stored at physical element offset `offset`. */
alt_status_t alt_layout_index_of(const alt_layout_t *l, const int64_t *shape, int64_t offset,
                                 int64_t *out_idx);

/* ---- layout conversion operator (Section 4.2, first way of Fig. 5) ------ */

/* dst[off_dst(i)] = src[off_src(i)] for every logical index i of a tensor of
 * logical `shape` (host pointer, `ndim` entries).  src and dst are device
 * pointers to numel elements each and must not overlap.  Bits are moved
 * unchanged.  Asynchronous on `stream`. */
alt_status_t alt_layout_transform(alt_handle_t h, alt_dtype_t dtype, int ndim, const int64_t *shape,
                                  const alt_layout_t *src_layout, const void *src,
                                  const alt_layout_t *dst_layout, void *dst, void *stream);

/* The pad primitive and its inverse (Section 4.1.2: zeros appended to selected dimensions) carried by the
 * conversion operator (Section 4.2: a padding operator with a propagated layout pads and converts in one
 * pass).  src holds a tensor of logical `src_shape` under `src_layout`, dst receives the tensor of logical
 * `dst_shape` under `dst_layout` (each layout is bound to its own shape; this is how a channel count that a
 * block factor does not divide reaches a blocked layout: pad it to the next multiple).  dst's element at
 * index i is src's where i lies inside both shapes and zero (all bits clear) elsewhere: extents may grow
 * (pad), shrink (unpad) or both.  Device pointers to numel(src_shape) and numel(dst_shape) elements, no
 * overlap.  One thread per element (this form is for operands prepared once, not for the hot path).
 * Asynchronous on `stream`; launches kernels only (safe under stream capture). */
alt_status_t alt_layout_transform_pad(alt_handle_t h, alt_dtype_t dtype, int ndim, const int64_t *src_shape,
                                      const alt_layout_t *src_layout, const void *src,
                                      const int64_t *dst_shape, const alt_layout_t *dst_layout, void *dst,
                                      void *stream);

/* What alt_layout_transform would launch for a conversion, without launching it (host only: works
 * without a GPU).  src_misalign / dst_misalign: the buffers' addresses modulo 16, which decide the
 * vector widths.  kind: 0 plain copy, 1 one thread per element (layouts whose blocks do not nest,
 * non-separable fuse sequences), 2 contiguous runs copied as they are, 3 tiles through LDS (the
 * contiguous piece differs between the two layouts).  With replay != 0 and kind = 3 the call also
 * replays every workgroup's index arithmetic on the host and counts, in `mismatches`, destination
 * elements not written exactly once from the source element that the two layouts' index maps
 * (Table 1) name, plus LDS indices out of range: 0 means the plan is the conversion operator of
 * Section 4.2; -1 means not replayed. */
typedef struct {
    int32_t kind;
    int32_t src_flat, dst_flat;   /* kind 3: that side of a tile is one contiguous run, moved in 16-byte vectors */
    int32_t load_bytes, store_bytes;
    int32_t tile_a, tile_b, tile_g;
    int64_t workgroups;
    int64_t lds_bytes;
    int64_t mismatches;
} alt_transform_plan_t;
alt_status_t alt_layout_transform_plan(alt_handle_t h, alt_dtype_t dtype, int ndim, const int64_t *shape,
                                       const alt_layout_t *src_layout, int src_misalign,
                                       const alt_layout_t *dst_layout, int dst_misalign, int replay,
                                       alt_transform_plan_t *out);

/* ---- C2D (program of Fig. 3; zero padding as in Section 4.2; fused bias and
 *      ReLU as in Fig. 6; producer writes the consumer's layout, Section 4.2) */

#define ALT_EPI_BIAS 1            /* y += bias[k], bias is fp32[K] on the device */
#define ALT_EPI_RELU 2            /* y = max(y, 0) after the bias */

typedef struct {
    int64_t N, C, H, W;           /* input activations */
    int64_t K, R, S;              /* output channels, kernel height, width */
    int32_t stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
    int32_t in_dtype;             /* alt_dtype_t of x and w */
    int32_t out_dtype;            /* alt_dtype_t of y (bf16 = fp32 sum rounded to nearest even) */
    int32_t epilogue;             /* ALT_EPI_* flags */
    int32_t variant;              /* kernel variant; -1 = cached tuned one, else the default */
    alt_layout_t x_layout;        /* of logical (N, C, H, W) */
    alt_layout_t w_layout;        /* of logical (K, C, R, S) */
    alt_layout_t y_layout;        /* of logical (N, K, OH, OW) */
    int32_t groups;               /* 0 or 1: ordinary; g > 1: output channel k reads only the C/g input channels of
                                     group k / (K/g) (C and K multiples of g), w is logical (K, C/g, R, S);
                                     g = C = K is the depth-wise convolution */
    int32_t reserved;             /* 0 */
} alt_conv_desc_t;

/* y[n,k,oh,ow] = sum_{c,r,s} x[n,c,oh*stride-pad+r*dil, ow*stride-pad+s*dil] * w[k,c,r,s]
 * (cross-correlation, zeros outside the input), OH = floor((H+2pad-dil(R-1)-1)/stride)+1.
 * With groups = g > 1 (the group-wise and depth-wise C2D of Section 6.1) c runs over the
 * C/g channels of k's group: x channel (k / (K/g)) * (C/g) + c.  Grouped problems run on
 * the implicit-GEMM kernels with one group per grid plane (channel blocks of a blocked
 * layout must not straddle groups); depth-wise ones on kernels of their own, which have no
 * variants: the tuner and alt_conv2d_variant_* do not take them.
 * x, w, y are device pointers holding the tensors under the descriptor's
 * layouts; `w` is what alt_pack_weights wrote (or any buffer already in
 * w_layout).  bias may be NULL without ALT_EPI_BIAS.  `workspace` (device,
 * ws_bytes) holds split-K partial sums.  With variant = -1 the library only
 * picks variants whose partial sums fit the workspace given (none is needed
 * without split-K, so NULL/0 always works); alt_conv2d_workspace_size reports
 * what the preferred variant would like.  An explicitly requested variant
 * whose needs exceed ws_bytes fails with ALT_WORKSPACE_TOO_SMALL.
 * Asynchronous on `stream`. */
alt_status_t alt_conv2d(alt_handle_t h, const alt_conv_desc_t *d, const void *x, const void *w,
                        const float *bias, void *y, void *workspace, size_t ws_bytes, void *stream);
alt_status_t alt_conv2d_workspace_size(alt_handle_t h, const alt_conv_desc_t *d, size_t *bytes);

/* alt_conv2d for callers that cannot bring a workspace or allocate one: code under HIP
 * graph capture, serving loops and harnesses where hipMalloc is forbidden.  Same operation,
 * same kernels and same variant choice as alt_conv2d, but the split-K partial tiles go to a
 * static device array of ALT_STATIC_WORKSPACE_BYTES that the library's code object holds on
 * every device it is loaded on, from load to process end.  The call allocates and frees no
 * device memory.  With variant = -1 only variants whose partial tiles fit the array are
 * picked (none are needed without split-K); an explicit split-K variant that needs more
 * fails with ALT_WORKSPACE_TOO_SMALL and a message giving both sizes.  Nothing in the array
 * has to be zero between calls (every partial tile is written before it is read; the
 * arrival counters reset themselves).  All calls on one device share the one array: two
 * calls that may run at the same time (different streams, or a replayed graph beside eager
 * calls) race on it and must be ordered by the caller; calls on one stream are ordered. */
#define ALT_STATIC_WORKSPACE_BYTES (32u << 20)
alt_status_t alt_conv2d_static(alt_handle_t h, const alt_conv_desc_t *d, const void *x, const void *w,
                               const float *bias, void *y, void *stream);

/* Split-K variants of the tile kernels (names ending _k2, _k4, ...: the reduction over input
 * channels of the Fig. 3 program cut into slices that run as separate workgroups) sum their
 * slices inside the one launch: every slice writes its partial tile to `workspace`, the last
 * slice to arrive at the tile's counter adds them in slice order.  The counters live in a
 * static device array of ALT_SPLITK_MAX_STREAMS sets; a set is bound to the stream that first
 * launches a split-K variant and serves that stream from then on, so launches on different
 * streams never share one.  Limits that follow:
 *  - when more than ALT_SPLITK_MAX_STREAMS streams have launched split-K variants on a device,
 *    the next new stream makes the library wait for the device to go idle and release the
 *    sets (those that a graph capture has seen stay bound for good); while a stream is being
 *    captured that wait is not possible and the call returns ALT_UNSUPPORTED;
 *  - a captured graph carries the set of the stream it was captured on: do not replay it
 *    while other split-K launches issued or captured on that same stream are in flight;
 *  - partial tiles and counters are exchanged with device scope (written through to the
 *    memory all XCDs share): the result does not depend on where workgroups run. */
#define ALT_SPLITK_MAX_STREAMS 64
typedef struct {
    int32_t streams_bound;        /* counter sets bound to a stream */
    int32_t max_streams;          /* ALT_SPLITK_MAX_STREAMS */
    int32_t counters_nonzero;     /* arrival counters that are not zero with the device idle (always 0 unless a launch failed) */
} alt_splitk_status_t;
/* Waits for the device to go idle, then reports the above. */
alt_status_t alt_splitk_status(alt_handle_t h, alt_splitk_status_t *out);

/* alt_conv2d with a sum fused into its epilogue (the fused loop nest of Fig. 6; a residual
 * join whose other operand is already in the convolution's output layout):
 *   y = act(conv(x, w) + bias + addend),
 * the sum in fp32 before the one rounding of the output.  `addend` (device, 16-byte aligned)
 * has y's layout and element type and may not alias y.  Built into the tile kernels (dense
 * NHWC activations and output, OHWI weights, bf16 inputs: the direct and streaming kernels);
 * descriptors only the implicit-GEMM kernels cover, grouped and depth-wise ones fail with
 * ALT_UNSUPPORTED (run alt_conv2d and alt_eltwise_add instead).  Everything else as alt_conv2d. */
alt_status_t alt_conv2d_add(alt_handle_t h, const alt_conv_desc_t *d, const void *x, const void *w,
                            const float *bias, const void *addend, void *y, void *workspace, size_t ws_bytes,
                            void *stream);

/* One alt_conv2d call's arguments, for alt_conv2d_multi. */
typedef struct {
    const alt_conv_desc_t *d;
    const void *x, *w;
    const float *bias;
    void *y;
    void *workspace;
    size_t ws_bytes;
    void *stream;
} alt_conv_call_t;

/* Issues n convolutions that do not depend on one another (operators of a computational
 * graph with no path between them, Section 2.2's graph view; e.g. a residual block's
 * projection shortcut beside its main branch), the i-th exactly as
 * alt_conv2d(h, calls[i].d, ...) on calls[i].stream.  Calls given different streams may
 * run on the GPU at the same time, so a kernel that cannot fill the chip alone shares it
 * and one call's start-up overlaps another's tail; ordering between the streams is the
 * caller's (events or stream synchronisation).  The outputs and workspaces must not
 * overlap.  Stops at the first call that fails and returns its status; the calls before
 * it stay issued. */
alt_status_t alt_conv2d_multi(alt_handle_t h, const alt_conv_call_t *calls, int32_t n);
alt_status_t alt_conv2d_output_shape(const alt_conv_desc_t *d, int64_t *out_nkhw);

/* Offline weight transformation (Section 4.2: the weight tensor is a constant,
 * so its layout is changed once, outside the timed path): dense OIHW ->
 * d->w_layout.  Device pointers, asynchronous on `stream`. */
alt_status_t alt_pack_weights(alt_handle_t h, const alt_conv_desc_t *d, const void *w_oihw,
                              void *w_packed, void *stream);

/* Transposed 2-D convolution (T2D in the operator list of Section 6.1), the adjoint of the
 * C2D that maps K channels to C with the same filter:
 *   y[n,k,ih*stride-pad+r*dil, iw*stride-pad+s*dil] += x[n,c,ih,iw] * w[c,k,r,s],
 *   OH = (H-1)*stride - 2*pad + dil*(R-1) + 1 (likewise OW); needs pad <= dil*(R-1), groups = 1.
 * The descriptor's N,C,H,W describe x, K the output channels, R,S,stride,pad,dil the
 * transposed operator; x_layout and y_layout are the layouts of x and y, w_layout the layout
 * of the equivalent forward filter w'[k,c,r,s] = w[c,k,R-1-r,S-1-s] (logical (K,C,R,S)), which
 * alt_pack_weights_transpose writes once, offline, from the dense (C,K,R,S) filter.
 * It runs as the equivalent forward convolution: x with stride-1 zeros between its pixels
 * (written into the workspace under x_layout by a kernel of its own; skipped for stride 1)
 * convolved with w' at stride 1 and padding dil*(R-1)-pad by alt_conv2d's kernels (variant,
 * epilogue, dtypes and tuning cache as for alt_conv2d).
 * Sub-pixel form: where both output extents are multiples of the strides and the taps of the
 * stride_h*stride_w output phases fit one symmetric window (4x4 at stride 2 with padding 1, 2x2
 * at stride 2, 6x6 at stride 2 with padding 2, 8x8 at stride 4 with padding 2, ...) the library
 * instead runs ONE stride-1 convolution of x itself with stride_h*stride_w*K output channels,
 *   y'[n, (ph*stride_w + pw)*K + k, q, p] = y[n, k, q*stride_h + ph, p*stride_w + pw],
 * into the workspace (no inserted zeros are multiplied) and moves y' into place under y_layout
 * with a kernel of its own; the packed filter is then the merged one, logical
 * (stride_h*stride_w*K, C, R', S') under w_layout with R', S' the common window of the phases.
 * Which form a descriptor takes depends on the descriptor alone;
 * alt_conv2d_transpose_weight_shape reports the logical shape of the packed filter (so its
 * size), alt_pack_weights_transpose writes it, alt_conv2d_transpose_workspace_size counts the
 * form's needs.  `workspace` (device, 16-byte aligned) holds the expanded input (or y' and a
 * bias vector) followed by what alt_conv2d wants; less than the first part fails with
 * ALT_WORKSPACE_TOO_SMALL.  Asynchronous on `stream`. */
alt_status_t alt_conv2d_transpose(alt_handle_t h, const alt_conv_desc_t *d, const void *x, const void *w_packed,
                                  const float *bias, void *y, void *workspace, size_t ws_bytes, void *stream);
alt_status_t alt_conv2d_transpose_workspace_size(alt_handle_t h, const alt_conv_desc_t *d, size_t *bytes);
alt_status_t alt_conv2d_transpose_output_shape(const alt_conv_desc_t *d, int64_t *out_nkhw);
alt_status_t alt_conv2d_transpose_weight_shape(const alt_conv_desc_t *d, int64_t *out_kcrs);
/* The 2-D forward problem alt_conv2d_transpose hands to alt_conv2d's kernels for this descriptor
 * (extents, padding and layouts of the form it takes; epilogue, dtypes and variant as given):
 * tune(op, shape) for the transposed operator is alt_tune_conv2d on it, after which the call
 * finds the winning variant in the cache. */
alt_status_t alt_conv2d_transpose_problem(alt_handle_t h, const alt_conv_desc_t *d, alt_conv_desc_t *out);
alt_status_t alt_pack_weights_transpose(alt_handle_t h, const alt_conv_desc_t *d, const void *w_ckrs,
                                        void *w_packed, void *stream);

/* 3-D convolution (C3D in the operator list of Section 6.1):
 *   y[n,k,od,oh,ow] = sum_{c,t,r,s} x[n,c,od*stride_d-pad_d+t*dil_d, oh*stride_h-pad_h+r*dil_h, ow*stride_w-pad_w+s*dil_w] * w[k,c,t,r,s],
 *   zeros outside the input, OD = floor((D+2pad_d-dil_d(T-1)-1)/stride_d)+1 (OH, OW as for alt_conv2d).
 * `plane` is the 2-D part of the problem: N, C, H, W, K, R, S, the strides, padding and dilation
 * of the two directions of a depth slice, dtypes, epilogue, variant, and the layouts of ONE depth
 * slice; D, T and the *_d fields are the depth part.  Tensors are stacks of depth slices, batch
 * index outermost (every layout alt_layout_parse accepts keeps it there):
 *   x is logical (N*D,  C, H,  W)  under plane.x_layout, slice (n, d)  at batch index n*D  + d,
 *   y is logical (N*OD, K, OH, OW) under plane.y_layout, slice (n, od) at batch index n*OD + od,
 * so "NCHW->NHWC" here is the NDHWC tensor and "NCHW->NCHW" the NDCHW one (a tensor with the
 * channels outside the depth is brought there by alt_layout_transform on its five dimensions).
 * It runs as a 2-D convolution: unfolding the depth (Section 4.1.2, Eq. 1) into tiles of T slices
 * every stride_d and placing the tile index beside the channels gives
 *   x'[(n,od), t*C + c, h, w] = x[(n, od*stride_d - pad_d + t*dil_d), c, h, w]   (zero outside the depth),
 * logical (N*OD, T*C, H, W) under plane.x_layout, which a kernel of its own writes into the
 * workspace per call; alt_conv2d's kernels (variants, tuning cache, epilogue as there) convolve it
 * with w'[k, t*C + c, r, s] = w[k,c,t,r,s], logical (K, T*C, R, S) under plane.w_layout, which
 * alt_pack_weights3d writes once, offline, from the dense (K,C,T,R,S) filter.  Blocked layouts
 * must divide T*C as they would C.  T = 1 with stride_d = 1 and pad_d = 0 is alt_conv2d on x itself.
 * `workspace` (device, 16-byte aligned) holds x' followed by what alt_conv2d wants;
 * alt_conv3d_workspace_size reports the sum, less than x' fails with ALT_WORKSPACE_TOO_SMALL.
 * groups > 1 is ALT_UNSUPPORTED.  alt_conv3d_output_shape writes (N, K, OD, OH, OW).
 * Asynchronous on `stream`. */
typedef struct {
    alt_conv_desc_t plane;
    int64_t D, T;                 /* input depth, filter depth */
    int32_t stride_d, pad_d, dil_d;
    int32_t reserved;             /* 0 */
} alt_conv3d_desc_t;

alt_status_t alt_conv3d(alt_handle_t h, const alt_conv3d_desc_t *d, const void *x, const void *w_packed,
                        const float *bias, void *y, void *workspace, size_t ws_bytes, void *stream);
alt_status_t alt_conv3d_workspace_size(alt_handle_t h, const alt_conv3d_desc_t *d, size_t *bytes);
alt_status_t alt_conv3d_output_shape(const alt_conv3d_desc_t *d, int64_t *out_nkdhw);
alt_status_t alt_pack_weights3d(alt_handle_t h, const alt_conv3d_desc_t *d, const void *w_kctrs,
                                void *w_packed, void *stream);
/* The 2-D problem (batch N*OD, T*C channels) that alt_conv3d hands to alt_conv2d's kernels: tune(op, shape)
 * for the 3-D operator is alt_tune_conv2d on it. */
alt_status_t alt_conv3d_problem(alt_handle_t h, const alt_conv3d_desc_t *d, alt_conv_desc_t *out);

/* Transposed 3-D convolution (T3D in the operator list of Section 6.1), the adjoint of the C3D
 * that maps K channels to C with the same filter:
 *   y[n,k, id*stride_d-pad_d+t*dil_d, ih*stride_h-pad_h+r*dil_h, iw*stride_w-pad_w+s*dil_w] += x[n,c,id,ih,iw] * w[c,k,t,r,s],
 *   OD = (D-1)*stride_d - 2*pad_d + dil_d*(T-1) + 1 (likewise OH, OW); needs pad <= dil*(taps-1) in
 *   each direction, groups = 1.
 * The descriptor reads as for alt_conv3d with N, C, D, H, W describing x, K the output channels and
 * the strides, padding and dilation those of the transposed operator; tensors are stacks of depth
 * slices as there.  It runs as the forward operator at stride 1 and padding dil*(taps-1)-pad over x
 * with stride-1 zeros between its elements in all three directions, with the mirrored,
 * channel-swapped filter: the depth-unfolding kernel of alt_conv3d reads x where all three
 * indices are multiples of the strides and writes zeros elsewhere (one pass, into the workspace),
 * alt_pack_weights3d_transpose writes w'[k, t*C + c, r, s] = w[c, k, T-1-t, R-1-r, S-1-s], logical
 * (K, T*C, R, S) under plane.w_layout, once from the dense (C,K,T,R,S) filter, and alt_conv2d's
 * kernels do the rest.
 * Sub-pixel form, as for alt_conv2d_transpose: where the output extents are multiples of the strides
 * and the taps of the stride_d*stride_h*stride_w output phases fit one symmetric window per direction
 * (4x4x4 at stride 2 with padding 1, 2x2x2 at stride 2, ...), the library instead runs one forward
 * 3-D convolution of x itself (stride 1) with that many times K output channels into the workspace
 * and moves the phases into place with a kernel of its own; the packed filter is then the merged
 * one.  alt_conv3d_transpose_weight_shape reports the logical shape (K', T'*C, R', S') of the packed
 * filter of the form the descriptor takes (so its size).
 * Workspace and errors as for alt_conv3d.  Asynchronous on `stream`. */
alt_status_t alt_conv3d_transpose(alt_handle_t h, const alt_conv3d_desc_t *d, const void *x, const void *w_packed,
                                  const float *bias, void *y, void *workspace, size_t ws_bytes, void *stream);
alt_status_t alt_conv3d_transpose_workspace_size(alt_handle_t h, const alt_conv3d_desc_t *d, size_t *bytes);
alt_status_t alt_conv3d_transpose_output_shape(const alt_conv3d_desc_t *d, int64_t *out_nkdhw);
alt_status_t alt_pack_weights3d_transpose(alt_handle_t h, const alt_conv3d_desc_t *d, const void *w_cktrs,
                                          void *w_packed, void *stream);
alt_status_t alt_conv3d_transpose_problem(alt_handle_t h, const alt_conv3d_desc_t *d, alt_conv_desc_t *out);
alt_status_t alt_conv3d_transpose_weight_shape(alt_handle_t h, const alt_conv3d_desc_t *d, int64_t *out_kcrs);

/* Kernel variants applicable to a descriptor (loop-tuning space of Section
 * 4.3 realised as tile shapes, K-depth per LDS stage, split-K factor and
 * operand loader).  Variant numbers are stable within one library build.
 * alt_conv2d_variant_name with variant = -1 names the variant alt_conv2d picks for
 * the descriptor when it is left to choose (the tuned one if the cache has it, else
 * the best by the library's cost estimate); ALT_UNSUPPORTED if `variant` does not
 * apply to the descriptor. */
alt_status_t alt_conv2d_variant_count(alt_handle_t h, const alt_conv_desc_t *d, int *count);
alt_status_t alt_conv2d_variant_name(alt_handle_t h, const alt_conv_desc_t *d, int variant,
                                     char *buf, size_t buflen);

/* ---- GMM (Section 5.1: C = A B with per-operand layouts) ----------------- */

typedef struct {
    int64_t batch, M, N, K;       /* batch >= 1; operands of one batch entry are dense, batch outermost */
    int32_t in_dtype, out_dtype;
    int32_t variant;              /* -1 = cached tuned one, else the default */
    int32_t reserved;
    alt_layout_t a_layout;        /* of logical (M, K) */
    alt_layout_t b_layout;        /* of logical (K, N); "KN->NK" is a transposed operand */
    alt_layout_t c_layout;        /* of logical (M, N) */
} alt_gemm_desc_t;

/* C[b,m,n] = sum_k A[b,m,k] * B[b,k,n].  Device pointers; asynchronous. */
alt_status_t alt_gemm(alt_handle_t h, const alt_gemm_desc_t *d, const void *A, const void *B,
                      void *C, void *workspace, size_t ws_bytes, void *stream);
alt_status_t alt_gemm_workspace_size(alt_handle_t h, const alt_gemm_desc_t *d, size_t *bytes);
alt_status_t alt_gemm_variant_count(alt_handle_t h, const alt_gemm_desc_t *d, int *count);
/* (variant = -1 names the variant alt_gemm picks for the descriptor, as alt_conv2d_variant_name does) */
alt_status_t alt_gemm_variant_name(alt_handle_t h, const alt_gemm_desc_t *d, int variant,
                                   char *buf, size_t buflen);

/* ---- joint tuning (Section 5.2: cross exploration — pick a layout, tune the
 *      loops under it, feed the best latency back; budget counted in on-device
 *      measurements as in Section 6) --------------------------------------- */

typedef struct {
    int32_t max_trials;           /* measurement budget; <= 0 = unlimited */
    int32_t warmup;               /* untimed launches per measurement (default 3) */
    int32_t reps;                 /* timed launches per measurement (default 20) */
    int32_t layout_mask;          /* bit i enables layout candidate i; 0 = all */
    void *arena;                  /* device scratch for the tuner's tensors */
    size_t arena_bytes;
    void *stream;
} alt_tune_opts_t;

#define ALT_MAX_CANDIDATES 16

typedef struct {
    int32_t trials;               /* measurements actually run */
    int32_t n_layouts;            /* layout candidates explored */
    float best_us;                /* latency of the winner */
    float default_us;             /* best latency under the default layouts (NCHW/OIHW, row-major) */
    float layout_best_us[ALT_MAX_CANDIDATES];   /* the reward of each layout: its best latency */
    int32_t layout_best_variant[ALT_MAX_CANDIDATES];
    char layout_name[ALT_MAX_CANDIDATES][48];
} alt_tune_report_t;

/* Required arena size for the tune calls below. */
alt_status_t alt_tune_conv2d_arena_size(alt_handle_t h, const alt_conv_desc_t *shape, size_t *bytes);
alt_status_t alt_tune_gemm_arena_size(alt_handle_t h, const alt_gemm_desc_t *shape, size_t *bytes);

/* Explores layout candidates x kernel variants for the problem in `shape`
 * (its layouts and variant are ignored), writes the winner (layouts + variant
 * filled in) to best_out, remembers it in the handle's cache so that later
 * alt_conv2d / alt_gemm calls with variant = -1 on the same problem and
 * layouts use the tuned variant.  Synchronises. */
alt_status_t alt_tune_conv2d(alt_handle_t h, const alt_conv_desc_t *shape, const alt_tune_opts_t *opts,
                             alt_conv_desc_t *best_out, alt_tune_report_t *report);
alt_status_t alt_tune_gemm(alt_handle_t h, const alt_gemm_desc_t *shape, const alt_tune_opts_t *opts,
                           alt_gemm_desc_t *best_out, alt_tune_report_t *report);

/* Loop-only stage (Section 5.2): layouts in `d` are kept, only the kernel
 * variant is searched; the winner is written to d->variant and cached. */
alt_status_t alt_tune_conv2d_variants(alt_handle_t h, alt_conv_desc_t *d, const alt_tune_opts_t *opts,
                                      float *best_us, int *trials);

/* Loop-only stage for n independent convolutions that alt_conv2d_multi launches together
 * (n <= ALT_MAX_MULTI).  Tuned one at a time each problem gets the variant that is fastest
 * alone on an idle chip; launched together they share compute units, LDS and L2, and a
 * variant that leaves room for a neighbour's workgroups can make the whole launch faster
 * though it is slower alone.  So the cost here is the measured time of one alt_conv2d_multi
 * step (Section 5.2's cross exploration with the launch as the unit): every problem's
 * variants are first timed alone on its stream (at most opts->max_trials each when > 0; those
 * within 2x of its best stay candidates, split-K ones only if calls[i].workspace holds their
 * partial sums), then rounds of coordinate descent replace one problem's variant at a time
 * while the step gets faster, and last the order in which the step issues the calls is chosen
 * the same way (all orders for n <= 5).  The layouts in calls[i].d are kept.  Writes the chosen
 * variant of call i to variants[i], the issue order (indices into calls) to order[0..n), the
 * step time to *step_us and the number of step measurements to *measurements (either may be
 * NULL).  Uses the callers' buffers and streams: the outputs are overwritten.  Depth-wise
 * problems have no variants and are refused.  opts->arena is not used.  Synchronises. */
#define ALT_MAX_MULTI 8
alt_status_t alt_tune_conv2d_multi(alt_handle_t h, const alt_conv_call_t *calls, int32_t n,
                                   const alt_tune_opts_t *opts, int32_t *variants, int32_t *order,
                                   float *step_us, int32_t *measurements);

#define ALT_MAX_CHAIN 8

typedef struct {
    int32_t nops;
    int32_t trials;
    alt_conv_desc_t op[ALT_MAX_CHAIN];        /* chosen layouts and variant per operator */
    int32_t transform_before[ALT_MAX_CHAIN];  /* 1: a conversion operator feeds op i's input */
    alt_layout_t edge_layout[ALT_MAX_CHAIN + 1]; /* layout the producer writes on edge i (edge 0 = chain input) */
    float op_us[ALT_MAX_CHAIN];
    float transform_us[ALT_MAX_CHAIN];
    float total_us;                           /* planned end-to-end latency */
    float default_total_us;                   /* same chain with NCHW on every edge */
} alt_chain_plan_t;

/* Graph-level choice for a chain of convolutions (Section 4.2, third
 * constraint: each complex operator is tuned on its own and a conversion
 * operator is inserted between two of them only where their layouts differ).
 * ops[i+1] consumes ops[i]'s output; the chain input arrives in `in_layout`
 * and the last output leaves in the layout the last operator prefers.
 * Measures every operator under every (input, output) layout pair and every
 * conversion, then takes the cheapest path.  Synchronises. */
alt_status_t alt_tune_chain(alt_handle_t h, const alt_conv_desc_t *ops, int nops,
                            const alt_layout_t *in_layout, const alt_tune_opts_t *opts,
                            alt_chain_plan_t *plan);

/* Pure planner behind alt_tune_chain (host only, no device work): given
 * op_cost[i][a][b] = latency of operator i reading layout a and writing layout
 * b (row-major [nops][nl][nl]), conv_cost[i][a][b] = latency of converting
 * edge i from a to b ([nops][nl][nl], zero on the diagonal) and the layout
 * index the chain input arrives in, returns per operator the (input, output)
 * layout indices of the cheapest plan and its total cost. */
alt_status_t alt_plan_chain(int nops, int nl, const float *op_cost, const float *conv_cost,
                            int in_layout, int *out_in_idx, int *out_out_idx, float *out_total);

/* ---- unfold primitive: overlapped tiling (Section 4.1.2, Eq. 1) ---------- */

/* Shape after unfolding dimension `dim` of `shape` (ndim entries, ndim <
 * ALT_MAX_RANK) into tiles of B elements every S elements: the dimension is
 * replaced by (T, B) with T = ceil((D - B) / S) + 1 (1 if D <= B); out_shape
 * gets ndim + 1 entries.  Host only. */
alt_status_t alt_unfold_shape(int ndim, const int64_t *shape, int dim, int64_t B, int64_t S, int64_t *out_shape);

/* dst[..., t, b, ...] = src[..., t*S + b, ...] over a row-major tensor of
 * `shape`, zero bits where t*S + b runs past the dimension (the last tile of a
 * non-dividing tiling).  This is the conversion that materialises the
 * overlapped-tile layout of a convolution input: it expands the data by about
 * B / S.  src and dst are device buffers that do not overlap; bits are moved
 * unchanged.  Asynchronous on `stream`. */
alt_status_t alt_unfold(alt_handle_t h, alt_dtype_t dtype, int ndim, const int64_t *shape, int dim, int64_t B,
                        int64_t S, const void *src, void *dst, void *stream);

/* ---- graphs of operators: layout propagation (Section 4.2) ---------------- */

/* y[i] = a[i] + b[i] (b may be null: y = a), then max(., 0) if relu != 0, for
 * numel elements of `dtype`.  bf16: the exact sum rounded once to nearest even.
 * An element-wise operator takes the layout of its producer (Section 4.2), so
 * the three device buffers are flat and share one layout; y may alias a or b.
 * 16-byte aligned buffers.  Asynchronous on `stream`. */
alt_status_t alt_eltwise_add(alt_handle_t h, alt_dtype_t dtype, int64_t numel, const void *a, const void *b,
                             void *y, int relu, void *stream);

#define ALT_MAX_GRAPH 8
#define ALT_NODE_CONV 0
#define ALT_NODE_ADD 1

typedef struct {
    int32_t kind;             /* ALT_NODE_CONV or ALT_NODE_ADD */
    int32_t in0, in1;         /* tensors read: 0 = the graph input, i + 1 = the output of node i (earlier nodes
                                 only); in1 is ignored for ALT_NODE_CONV */
    int32_t relu;             /* ALT_NODE_ADD: ReLU after the sum (a convolution's is in its epilogue flags) */
    alt_conv_desc_t conv;     /* ALT_NODE_CONV: shape, types, stride, padding, epilogue; layouts and variant ignored */
} alt_graph_node_t;

typedef struct {
    int32_t nnodes, trials;
    alt_conv_desc_t conv[ALT_MAX_GRAPH];            /* ALT_NODE_CONV nodes: chosen layouts and variant */
    alt_layout_t tensor_layout[ALT_MAX_GRAPH + 1];  /* layout tensor t is stored in (0 = the graph input) */
    alt_layout_t read_layout[ALT_MAX_GRAPH][2];     /* layout node i reads its input j in */
    int32_t convert[ALT_MAX_GRAPH][2];              /* 1: a conversion operator feeds input j of node i */
    float convert_us[ALT_MAX_GRAPH][2];
    float node_us[ALT_MAX_GRAPH];
    float total_us;                                 /* planned latency of the graph */
    float default_total_us;                         /* the same graph with NCHW on every tensor */
    int32_t fused_into[ALT_MAX_GRAPH];              /* ALT_NODE_ADD node i: index of the convolution node whose
                                                       epilogue computes it (alt_conv2d_add; conv[] of that node then
                                                       carries the sum's ReLU and node_us the fused time, node_us[i]
                                                       is 0), or -1: the sum runs as alt_eltwise_add */
} alt_graph_plan_t;

/* Layout choice for a small graph of convolutions and element-wise sums, e.g.
 * a residual block (Section 4.2: layouts propagate from the complex operators
 * through the simple ones; a tensor with several consumers is stored once, in
 * its producer's layout, and a conversion operator is inserted in front of the
 * consumers that read another layout, one per target layout: consumers that
 * read the same converted copy share it, and convert_us is zero for all but the
 * first of them).  An ALT_NODE_ADD reads both inputs and
 * writes its output in one layout.  nodes[i] may only read the graph input and
 * outputs of nodes before it; the last node's output is the graph's.  Measures
 * every convolution under every (input, output) layout pair, every conversion
 * of every consumed tensor and every sum, then takes the cheapest assignment.
 * Last, a sum one of whose operands is the output of a convolution without ReLU
 * that nothing else reads, read as stored, while the other operand (possibly a
 * converted copy) exists before that convolution runs, is measured
 * fused into that convolution's epilogue (alt_conv2d_add) and fused in the plan
 * if that is faster than the two launches.  Synchronises. */
alt_status_t alt_tune_graph(alt_handle_t h, const alt_graph_node_t *nodes, int nnodes,
                            const alt_layout_t *in_layout, const alt_tune_opts_t *opts,
                            alt_graph_plan_t *plan);

/* Pure planner behind alt_tune_graph (host only).  kind/in0/in1: as in
 * alt_graph_node_t, per node.  op_cost[i][a][b] ([nnodes][nl][nl], convolutions
 * only): latency reading layout a, writing layout b.  conv_cost[t][a][b]
 * ([nnodes + 1][nl][nl]): latency of converting tensor t from a to b (the
 * diagonal is taken as zero; a tensor converted to one layout for several
 * consumers is charged once).  add_cost[i]: latency of sum node i.  Infinite
 * entries mark impossible combinations.  Returns the stored layout index of
 * every tensor ([nnodes + 1], entry 0 = in_layout), the layout index every
 * node reads each input in ([nnodes][2], -1 for unused) and the total. */
alt_status_t alt_plan_graph(int nnodes, const int32_t *kind, const int32_t *in0, const int32_t *in1, int nl,
                            const float *op_cost, const float *conv_cost, const float *add_cost, int in_layout,
                            int32_t *tensor_layout, int32_t *read_layout, float *total);

/* Tune cache persistence: text file, one line per entry keyed by problem,
 * dtype, layouts and the device architecture name. */
alt_status_t alt_cache_save(alt_handle_t h, const char *path);
alt_status_t alt_cache_load(alt_handle_t h, const char *path);
alt_status_t alt_cache_clear(alt_handle_t h);

/* ---- introspection -------------------------------------------------------- */

typedef struct {
    float copy_gbps;              /* measured large streaming copy, read+write bytes per second / 1e9 */
    float mfma_bf16_tflops;       /* measured register-resident bf16 MFMA loop */
    float nominal_hbm_gbps;       /* 8000 */
    float nominal_bf16_tflops;    /* 2500 */
    int32_t compute_units;
    int32_t clock_mhz;
    char arch[32];
    float read_gbps;              /* measured read-only pass over the arena, bytes read per second / 1e9 */
    float write_gbps;             /* measured write-only pass over the arena, bytes written per second / 1e9 */
} alt_peaks_t;

/* Measures attainable peaks on the handle's device using `arena` (device,
 * >= 1 GiB recommended: the passes must not fit the 256 MiB last-level cache)
 * as copy buffer; the arena's contents are overwritten.  Synchronises. */
alt_status_t alt_get_peak(alt_handle_t h, void *arena, size_t arena_bytes, alt_peaks_t *out);

#if defined(__GNUC__)
#pragma GCC visibility pop
#endif
#ifdef __cplusplus
}
#endif
#endif /* ALT_H_ */

// Shared between ops.hip (conv/gemm entry points) and tune.cpp.
#pragma once

#include "dconv.h"

namespace alt {

// One conv/gemm call reduced to what the implicit-GEMM kernels need.
struct Problem {
    IgemmParams p;
    int dtype;
    bool a_vec, a_trans, b_vec, b_trans;   // loaders the operand layouts admit (gather always works)
    bool spatial_split, spatial_ok;
    int64_t x_elems, w_elems;              // elements of one batch entry of each operand
    int64_t groups;                        // convolution groups (1 for ordinary problems and products)
    bool depthwise;                        // groups = C = K: runs on dwconv.hip, p describes the whole tensors
};

extern const int kSplitFactors[];
int igemm_num_splits();
int igemm_variant_count();
std::string igemm_variant_name(int variant);
void igemm_analyse(Problem *pb);
bool igemm_applicable(const Problem &pb, const IgemmLaunch &k, int splitk, IgemmParams *out, std::string *why);
size_t igemm_workspace(const Problem &pb, int splitk);
double igemm_estimate(const Problem &pb, const IgemmLaunch &k, const IgemmParams &p);
int igemm_default_variant(const Problem &pb, size_t ws_limit);
alt_status_t igemm_run(alt_handle_t h, const Problem &pb, int variant, void *workspace, size_t ws_bytes,
                       hipStream_t st);

// dconv.hip
bool dconv_setup(const Problem &pb, const IgemmLaunch &k, int splitk, DconvParams *out, size_t *lds_bytes,
                 std::string *why);
void dconv_splitk_state(int *slots_bound, int *counters_nonzero);
hipError_t dconv_run(const IgemmLaunch &k, DconvParams d, size_t lds, float *partial, hipStream_t st);

// ops.hip: device address of alt_conv2d_static's workspace array on the current device
hipError_t static_scratch(void **out);

// dwconv.hip
alt_status_t depthwise_run(alt_handle_t h, const Problem &pb, int64_t N, int64_t C, hipStream_t st);

// eltwise.hip
alt_status_t eltwise_add(alt_handle_t h, int dtype, int64_t numel, const void *a, const void *b, void *y, int relu,
                         hipStream_t st);

alt_status_t conv_problem(alt_handle_t h, const alt_conv_desc_t *d, const void *x, const void *w,
                          const float *bias, void *y, Problem *pb);
alt_status_t gemm_problem(alt_handle_t h, const alt_gemm_desc_t *d, const void *A, const void *B, void *C,
                          Problem *pb);

// t2d.hip: the kernels that put the output phases of a sub-pixel transposed convolution into place
alt_status_t phase_shuffle(alt_handle_t h, const alt_layout_t *layout, int64_t N, int64_t K, int64_t ODq, int64_t OHq, int64_t OWq,
                           int sd, int sh, int sw, int elsz, const void *src, void *dst, hipStream_t st);
alt_status_t phase_bias(alt_handle_t h, const float *bias, float *out, int64_t K, int64_t n, hipStream_t st);

alt_status_t transform_bound(alt_handle_t h, int elsz, const BoundLayout &ls, const void *src,
                             const BoundLayout &ld, void *dst, hipStream_t st);

}  // namespace alt

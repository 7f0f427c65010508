// Host side of alt_conv2d / alt_gemm: descriptor checks, mapping of layouts to
// the implicit-GEMM kernel's addressing, variant table, split-K reduction,
// weight packing.
#include <algorithm>
#include <mutex>

#include "igemm.h"
#include "ops.h"

namespace alt {

// ---- kernel registry -----------------------------------------------------------

static std::vector<IgemmLaunch> &registry()
{
    static std::vector<IgemmLaunch> v;
    return v;
}

void igemm_register(const IgemmLaunch &l) { registry().push_back(l); }

const std::vector<IgemmLaunch> &igemm_table()
{
    static std::once_flag once;
    std::call_once(once, [] {
        auto &v = registry();
        std::sort(v.begin(), v.end(), [](const IgemmLaunch &a, const IgemmLaunch &b) {
            return std::strcmp(a.name, b.name) < 0;
        });
    });
    return registry();
}

const int kSplitFactors[] = {1, 2, 3, 4, 6, 8, 9, 12, 16, 18, 24, 36};
static const int *const kSplits = kSplitFactors;
constexpr int kNumSplits = 12;
int igemm_num_splits() { return kNumSplits; }

int igemm_variant_count() { return (int)igemm_table().size() * kNumSplits; }

// ---- split-K reduction + epilogue ----------------------------------------------

__global__ __launch_bounds__(256) void splitk_reduce_kernel(const IgemmParams p)
{
    const int64_t per_batch = (int64_t)p.M * p.Nc;
    const int64_t total = per_batch * p.batch;
    const int ohow = p.OH * p.OW;
    for (int64_t e = blockIdx.x * (int64_t)256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
        const int bz = p.batch == 1 ? 0 : (int)(e / per_batch);
        const int64_t r = e - bz * per_batch;
        const int m = (int)fast_div((uint32_t)r, p.fd_nc), n = (int)(r - (int64_t)m * p.Nc);
        float v = 0.f;
        for (int s = 0; s < p.splitk; ++s) v += p.partial[(int64_t)s * total + e];
        if (p.epilogue & ALT_EPI_BIAS) v += p.bias[bz * p.bias_bstride + n];
        if (p.epilogue & ALT_EPI_RELU) v = fmaxf(v, 0.f);
        const int img = (int)fast_div(m, p.fd_ohow), rem = m - img * ohow;
        const int oh = (int)fast_div(rem, p.fd_ow), ow = rem - oh * p.OW;
        const int64_t off = (int64_t)bz * p.y_bstride + dim2_off(p.yn, img) + dim2_off(p.yk, n) +
                            dim2_off(p.yh, oh) + dim2_off(p.yw, ow);
        if (p.out_bf16) ((uint16_t *)p.y)[off] = f32_to_bf16_rne(v);
        else ((float *)p.y)[off] = v;
    }
}

// ---- eligibility of loaders ------------------------------------------------------

static bool mult(int64_t v, int m) { return v % m == 0; }

void igemm_analyse(Problem *pb)
{
    const IgemmParams &p = pb->p;
    const int epv = pb->dtype == ALT_BF16 ? 8 : 4;
    const int es = pb->dtype == ALT_BF16 ? 2 : 4;
    const bool x_spatial_split = (p.xh.f < p.H) || (p.xw.f < p.W);
    pb->spatial_split = x_spatial_split;
    pb->spatial_ok = !x_spatial_split || (p.R == 1 && p.S == 1 && p.pad_h == 0 && p.pad_w == 0);
    // A: 16-byte loads along channels
    pb->a_vec = p.xc.si == 1 && mult(p.xc.f, epv) && (p.xc.f >= p.C || mult(p.xc.so, epv)) &&
                mult(p.xn.si, epv) && mult(p.xn.so, epv) && mult(p.xh.si, epv) && mult(p.xh.so, epv) &&
                mult(p.xw.si, epv) && mult(p.xw.so, epv) && mult(p.x_bstride, epv) &&
                ((uintptr_t)p.x % 16 == 0) && pb->spatial_ok && pb->x_elems * es < 0x7fffffff;
    // A: rows (GMM m) contiguous, no spatial structure
    pb->a_trans = p.H == 1 && p.R == 1 && p.S == 1 && p.pad_h == 0 && p.pad_w == 0 && p.stride_w == 1 &&
                  p.xw.si == 1 && p.xw.f >= p.W && mult(p.M, epv) && p.xc.f >= p.C && mult(p.xc.si, epv) &&
                  mult(p.x_bstride, epv) && ((uintptr_t)p.x % 16 == 0) && p.OW == p.M;
    pb->b_vec = p.wi.si == 1 && mult(p.wi.f, epv) && (p.wi.f >= p.C || mult(p.wi.so, epv)) &&
                mult(p.wo.si, epv) && mult(p.wo.so, epv) && mult(p.wr.si, epv) && mult(p.wr.so, epv) &&
                mult(p.ws.si, epv) && mult(p.ws.so, epv) && mult(p.w_bstride, epv) &&
                ((uintptr_t)p.w % 16 == 0) && pb->w_elems * es < 0x7fffffff;
    pb->b_trans = p.R == 1 && p.S == 1 && p.wo.si == 1 && mult(p.wo.f, epv) &&
                  (p.wo.f >= p.Nc || mult(p.wo.so, epv)) && mult(p.Nc, epv) && mult(p.wi.si, epv) &&
                  mult(p.wi.so, epv) && mult(p.w_bstride, epv) && ((uintptr_t)p.w % 16 == 0);
}

static bool nests(int64_t f, int64_t C, int bk) { return f >= C ? true : (f % bk == 0 || bk % f == 0); }

// Can kernel `k` with split factor `splitk` run this problem?  Fills the
// launch-dependent fields of a copy of the parameters.
bool igemm_applicable(const Problem &pb, const IgemmLaunch &k, int splitk, IgemmParams *out, std::string *why)
{
    auto no = [&](const char *m) { if (why) *why = m; return false; };
    const IgemmParams &p0 = pb.p;
    if (k.dtype != pb.dtype) return no("element type");
    if (p0.addend && !k.launch_direct) return no("the fused sum is built into the tile kernels only");
    if (k.launch_direct) {
        if (!dconv_setup(pb, k, splitk, nullptr, nullptr, why)) return false;
        if (out) {
            IgemmParams p = p0;
            p.splitk = splitk;
            p.ksteps_total = p.R * p.S * (p.C / 64);
            p.ksteps_per_split = p.ksteps_total / splitk;
            p.tiles_m = (p.M + k.BM - 1) / k.BM;
            p.tiles_n = (p.Nc + k.BN - 1) / k.BN;
            *out = p;
        }
        return true;
    }
    if (!pb.spatial_ok && (k.amode != LOAD_GATHER)) return no("blocked H/W needs R=S=1 without padding");
    const bool uniform = p0.C % k.BK == 0 && nests(p0.xc.f, p0.C, k.BK) && nests(p0.wi.f, p0.C, k.BK);
    if (k.amode == LOAD_VEC && !(pb.a_vec && uniform)) return no("A is not channel-contiguous in 16-byte blocks");
    if (k.bmode == LOAD_VEC && !(pb.b_vec && uniform)) return no("B is not channel-contiguous in 16-byte blocks");
    if (k.amode == LOAD_TRANS && !pb.a_trans) return no("A rows are not contiguous");
    if (k.bmode == LOAD_TRANS && !pb.b_trans) return no("B rows are not contiguous");
    if (pb.spatial_split && k.amode == LOAD_GATHER && !(p0.R == 1 && p0.S == 1 && p0.pad_h == 0 && p0.pad_w == 0))
        return no("blocked H/W with a sliding window");
    IgemmParams p = p0;
    p.fd_ohow = make_fastdiv((uint32_t)(p.OH * p.OW));
    p.fd_ow = make_fastdiv((uint32_t)p.OW);
    p.fd_c = make_fastdiv((uint32_t)p.C);
    p.fd_s = make_fastdiv((uint32_t)p.S);
    p.fd_nc = make_fastdiv((uint32_t)p.Nc);
    p.uniform_rs = uniform ? 1 : 0;
    p.spatial_split = pb.spatial_split ? 1 : 0;
    p.ksteps_total = (p.Kg + k.BK - 1) / k.BK;
    if (splitk < 1 || splitk > p.ksteps_total) return no("split-K factor exceeds the K steps");
    if (splitk > 1 && (int64_t)p.M * p.Nc * 4 >= 0x7fffffff) return no("output too large for the split-K reduction");
    p.splitk = splitk;
    p.ksteps_per_split = (p.ksteps_total + splitk - 1) / splitk;
    if ((int64_t)(splitk - 1) * p.ksteps_per_split >= p.ksteps_total) return no("split-K factor leaves an empty slice");
    p.tiles_m = (p.M + k.BM - 1) / k.BM;
    p.tiles_n = (p.Nc + k.BN - 1) / k.BN;
    if ((int64_t)p.batch * splitk > 65535) return no("batch x split-K exceeds the grid");
    if (out) *out = p;
    return true;
}

size_t igemm_workspace(const Problem &pb, int splitk)
{
    if (splitk <= 1) return 0;
    return (size_t)splitk * pb.p.batch * pb.p.M * pb.p.Nc * sizeof(float);
}

// Rough relative time of one variant: rounds of workgroups over the chip x
// (K steps x per-step cost), gather/transposing loaders penalised.  Only used
// to pick a default and to order the tuner's trials best-first.
double igemm_estimate(const Problem &pb, const IgemmLaunch &k, const IgemmParams &p)
{
    (void)pb;
    if (k.launch_direct && k.stream == 1) {
        // Streaming kernel: all K groups take one K step each in the larger of their matrix-core
        // time (at the efficiency these kernels reach: less with fewer than eight waves) and the
        // time to bring their operand tiles into LDS (about 45 bytes per clock per CU), plus a
        // fixed part; a workgroup adds a prologue and an epilogue; as many workgroups share a CU
        // as their LDS allows.  Clocks at 2.2 GHz, scaled to the unit of the estimate below
        // (about 45 per microsecond).
        const int waves = k.kw * k.wgm * k.wgn;
        const double lds = (double)k.kw * (k.prefetch + 1) * (k.BM + k.BN) * k.BK * 2;
        const double stage = (double)k.kw * k.BM * (k.BN + 8.0 * k.wgn) * 4;
        const int per_cu = std::max(1, (int)(160.0 * 1024 / std::max(lds, stage)));
        const double blocks = (double)p.tiles_m * p.tiles_n * p.splitk * p.batch;
        const double rounds = std::ceil(blocks / (256.0 * per_cu));
        const double steps = (double)p.C / p.splitk / k.kw / k.BK;
        const double mfma = (double)k.kw * k.BM * k.BN * k.BK / 16384.0 * 8.0 * (waves >= 8 ? 1.7 : 2.0);
        const double bytes = (double)k.kw * (k.BM + k.BN) * k.BK * 2 / 45.0;
        const double clk = rounds * (steps * (std::max(mfma, bytes) + 120.0) + 6000.0);
        // (halved like the direct kernels' estimate below: wherever one of these kernels applies it
        // has beaten the implicit-GEMM kernels, whose estimate is optimistic)
        return 0.5 * (clk / 2200.0 * 45.0 + (p.splitk > 1 ? 140.0 : 0.0));
    }
    if (k.launch_direct && k.stream == 2) {
        // Channel-planar kernel: a workgroup converts its patch on the way in (about 20 bytes per clock
        // after a start-up latency), then per 64 channels runs all taps out of LDS (matrix-core time of
        // the tile, or the time to bring the weights in) between two barriers and a weight scatter, then
        // stores its tile plane by plane.  As many workgroups share a CU as their LDS allows.
        const int taps = p.R * p.S, st = p.stride_h;
        const double halo = (double)(p.dil_h * (p.R - 1)) * p.W + p.dil_w * (p.S - 1);
        const double np = (double)k.BM * st * st + halo + 8;
        const double lds = std::max((double)taps * (k.BN * 144 + 16) + np * (p.C * 2 + 16), (double)k.kw * k.BN * (k.BM + 4) * 4);
        const int per_cu = std::max(1, (int)(160.0 * 1024 / lds));
        // (workgroups that share a CU overlap their latencies, not their traffic or their matrix-core time)
        const double blocks = (double)p.tiles_m * p.tiles_n;
        const double per_cu_work = std::ceil(blocks / 256.0), rounds = std::ceil(blocks / (256.0 * per_cu));
        const double wload = (double)k.BN * 64 * taps * 2 / 40.0;      // the super-step's weights through L2
        const double busy = np * p.C * 2 / 20.0 + (p.C / 64) * std::max(taps * (double)k.BM * k.BN / 32.0 * 1.2, wload) +
                            (double)k.BM * k.BN / 8.0;
        const double latency = 3000.0 + (p.C / 64) * 800.0 + 1500.0;
        const double clk = per_cu_work * busy + rounds * latency + 5000.0;
        return 0.5 * (clk / 2200.0 * 45.0);
    }
    double mode_cost = 1.0;
    if (k.amode == LOAD_GATHER) mode_cost *= 6.0;
    if (k.bmode == LOAD_GATHER) mode_cost *= 3.0;
    if (k.amode == LOAD_TRANS) mode_cost *= 1.5;
    if (k.bmode == LOAD_TRANS) mode_cost *= 1.5;
    if (k.prefetch > 1) mode_cost *= 0.8;
    if (k.launch_direct) mode_cost *= 0.5;
    // (a 1x1 filter leaves the patch-resident kernel nothing to reuse: the streaming kernel runs the same
    // problem without staging the patch first, and has measured faster wherever both apply)
    if (k.launch_direct && p.R == 1 && p.S == 1) mode_cost *= 1.5;
    const double blocks = (double)p.tiles_m * p.tiles_n * p.splitk * p.batch;
    const double rounds = std::ceil(blocks / 512.0);
    const double step = (double)k.BM * k.BN * k.BK / 16384.0 + 3.0 * (k.BM + k.BN) * k.BK / 8192.0 + 2.0;
    double est = rounds * (p.ksteps_per_split * step + 60.0) * mode_cost;
    if (p.splitk > 1) est += (k.launch_direct ? 5.0 : 30.0) + 0.00002 * p.splitk * (double)p.M * p.Nc * p.batch;
    return est;
}

int igemm_default_variant(const Problem &pb, size_t ws_limit)
{
    const auto &tab = igemm_table();
    double best = 1e300;
    int best_v = -1;
    for (int ki = 0; ki < (int)tab.size(); ++ki)
        for (int si = 0; si < kNumSplits; ++si) {
            IgemmParams p;
            if (!igemm_applicable(pb, tab[ki], kSplits[si], &p, nullptr)) continue;
            if (igemm_workspace(pb, kSplits[si]) > ws_limit) continue;
            const double est = igemm_estimate(pb, tab[ki], p);
            if (est < best) { best = est; best_v = ki * kNumSplits + si; }
        }
    return best_v;
}

alt_status_t igemm_run(alt_handle_t h, const Problem &pb, int variant, void *workspace, size_t ws_bytes,
                       hipStream_t st)
{
    if (!h->has_gpu) return fail(h, ALT_HIP_ERROR, "no GPU device available");
    const auto &tab = igemm_table();
    if (variant < 0 || variant >= (int)tab.size() * kNumSplits)
        return fail(h, ALT_INVALID_ARG, "variant %d out of range", variant);
    const IgemmLaunch &k = tab[variant / kNumSplits];
    const int splitk = kSplits[variant % kNumSplits];
    IgemmParams p;
    std::string why;
    if (!igemm_applicable(pb, k, splitk, &p, &why))
        return fail(h, ALT_UNSUPPORTED, "variant %s/splitk%d not applicable: %s", k.name, splitk, why.c_str());
    const size_t need = igemm_workspace(pb, splitk);
    if (k.launch_direct) {
        if (need > 0 && (!workspace || ws_bytes < need))
            return fail(h, ALT_WORKSPACE_TOO_SMALL, "split-K needs %zu workspace bytes, got %zu", need, ws_bytes);
        DconvParams dp;
        size_t lds = 0;
        if (!dconv_setup(pb, k, splitk, &dp, &lds, &why))
            return fail(h, ALT_UNSUPPORTED, "variant %s/splitk%d not applicable: %s", k.name, splitk, why.c_str());
        hipError_t e = dconv_run(k, dp, lds, (float *)workspace, st);
        if (e == hipErrorNotReady)
            return fail(h, ALT_UNSUPPORTED, "%s: no split-K counter set is free for this stream (%d streams hold one; sets "
                                            "that captured graphs use are never released)", k.name, kDconvSlots);
        if (e != hipSuccess) return fail(h, ALT_HIP_ERROR, "launch of %s failed: %s", k.name, hipGetErrorString(e));
        return ALT_OK;
    }
    if (need > 0) {
        if (!workspace || ws_bytes < need)
            return fail(h, ALT_WORKSPACE_TOO_SMALL, "split-K needs %zu workspace bytes, got %zu", need, ws_bytes);
        p.partial = (float *)workspace;
    }
    dim3 grid((unsigned)(p.tiles_m * p.tiles_n), (unsigned)(p.batch * p.splitk));
    hipError_t e = k.launch(p, grid, st);
    if (e != hipSuccess) return fail(h, ALT_HIP_ERROR, "launch of %s failed: %s", k.name, hipGetErrorString(e));
    if (splitk > 1) {
        const int64_t total = (int64_t)p.M * p.Nc * p.batch;
        unsigned blocks = (unsigned)std::min<int64_t>((total + 255) / 256, 256 * 16);
        hipLaunchKernelGGL(splitk_reduce_kernel, dim3(blocks), dim3(256), 0, st, p);
        ALT_CHECK_HIP(h, hipGetLastError());
    }
    return ALT_OK;
}

std::string igemm_variant_name(int variant)
{
    const auto &tab = igemm_table();
    if (variant < 0 || variant >= (int)tab.size() * kNumSplits) return "";
    char buf[96];
    std::snprintf(buf, sizeof buf, "%s_k%d", tab[variant / kNumSplits].name, kSplits[variant % kNumSplits]);
    return buf;
}

// ---- descriptor -> problem ------------------------------------------------------------

static bool fits32(int64_t v) { return v >= 0 && v <= 0x7fffffff; }

alt_status_t conv_problem(alt_handle_t h, const alt_conv_desc_t *d, const void *x, const void *w,
                          const float *bias, void *y, Problem *pb)
{
    if (!d) return fail(h, ALT_INVALID_ARG, "null descriptor");
    if (d->N < 1 || d->C < 1 || d->H < 1 || d->W < 1 || d->K < 1 || d->R < 1 || d->S < 1)
        return fail(h, ALT_INVALID_ARG, "conv2d: non-positive extent");
    if (d->stride_h < 1 || d->stride_w < 1 || d->pad_h < 0 || d->pad_w < 0 || d->dil_h < 1 || d->dil_w < 1)
        return fail(h, ALT_INVALID_ARG, "conv2d: bad stride/pad/dilation");
    if ((d->in_dtype != ALT_F32 && d->in_dtype != ALT_BF16) || (d->out_dtype != ALT_F32 && d->out_dtype != ALT_BF16))
        return fail(h, ALT_INVALID_ARG, "conv2d: bad dtype");
    if (d->epilogue & ~(ALT_EPI_BIAS | ALT_EPI_RELU)) return fail(h, ALT_INVALID_ARG, "conv2d: unknown epilogue flag");
    const int64_t OH = (d->H + 2 * d->pad_h - d->dil_h * (d->R - 1) - 1) / d->stride_h + 1;
    const int64_t OW = (d->W + 2 * d->pad_w - d->dil_w * (d->S - 1) - 1) / d->stride_w + 1;
    if (d->H + 2 * d->pad_h < d->dil_h * (d->R - 1) + 1 || d->W + 2 * d->pad_w < d->dil_w * (d->S - 1) + 1)
        return fail(h, ALT_INVALID_ARG, "conv2d: kernel larger than padded input");
    const int64_t G = d->groups > 1 ? d->groups : 1;
    if (d->groups < 0 || d->C % G || d->K % G) return fail(h, ALT_INVALID_ARG, "conv2d: groups must divide C and K");
    const int64_t Cg = d->C / G, Kg = d->K / G;
    const int64_t xs[4] = {d->N, d->C, d->H, d->W}, wsh[4] = {d->K, Cg, d->R, d->S}, ys[4] = {d->N, d->K, OH, OW};
    BoundLayout bx, bw, by;
    std::string err;
    alt_status_t s;
    if ((s = bind_layout(&d->x_layout, 4, xs, &bx, &err)) != ALT_OK) return fail(h, s, "x_layout: %s", err.c_str());
    if ((s = bind_layout(&d->w_layout, 4, wsh, &bw, &err)) != ALT_OK) return fail(h, s, "w_layout: %s", err.c_str());
    if ((s = bind_layout(&d->y_layout, 4, ys, &by, &err)) != ALT_OK) return fail(h, s, "y_layout: %s", err.c_str());
    Dim2 dx[4], dw[4], dy[4];
    if (!layout_to_dim2(bx, dx) || !layout_to_dim2(bw, dw) || !layout_to_dim2(by, dy))
        return fail(h, ALT_UNSUPPORTED, "conv2d: layouts must be separable with at most one block level per dimension");
    if (!fits32(d->N * OH * OW) || !fits32(d->C * d->R * d->S) || !fits32(d->K) || !fits32(bx.numel / d->N * 2))
        return fail(h, ALT_UNSUPPORTED, "conv2d: problem too large for 32-bit tile indices");
    std::memset(pb, 0, sizeof(*pb));
    pb->dtype = d->in_dtype;
    pb->groups = G;
    pb->depthwise = G > 1 && Cg == 1 && Kg == 1;
    IgemmParams &p = pb->p;
    p.x = x; p.w = w; p.bias = bias; p.y = y;
    p.M = (int32_t)(d->N * OH * OW); p.Nc = (int32_t)d->K; p.Kg = (int32_t)(d->C * d->R * d->S);
    p.C = (int32_t)d->C; p.H = (int32_t)d->H; p.W = (int32_t)d->W; p.R = (int32_t)d->R; p.S = (int32_t)d->S;
    p.OH = (int32_t)OH; p.OW = (int32_t)OW;
    p.stride_h = d->stride_h; p.stride_w = d->stride_w; p.pad_h = d->pad_h; p.pad_w = d->pad_w;
    p.dil_h = d->dil_h; p.dil_w = d->dil_w;
    p.batch = 1; p.splitk = 1;
    p.epilogue = d->epilogue; p.out_bf16 = d->out_dtype == ALT_BF16;
    p.xn = dx[0]; p.xc = dx[1]; p.xh = dx[2]; p.xw = dx[3];
    p.wo = dw[0]; p.wi = dw[1]; p.wr = dw[2]; p.ws = dw[3];
    p.yn = dy[0]; p.yk = dy[1]; p.yh = dy[2]; p.yw = dy[3];
    pb->x_elems = bx.numel;
    pb->w_elems = bw.numel;
    {
        const int64_t yb = by.numel * (int64_t)dtype_size(d->out_dtype);
        p.y_bytes = yb < 0x7fffffff ? (uint32_t)yb : 0;
    }
    p.x_bytes = (uint32_t)std::min<int64_t>(bx.numel * (int64_t)dtype_size(d->in_dtype), 0x7fffffff);
    p.w_bytes = (uint32_t)std::min<int64_t>(bw.numel * (int64_t)dtype_size(d->in_dtype), 0x7fffffff);
    if (G > 1 && !pb->depthwise) {
        // One group per batch entry of the implicit-GEMM kernels: the group's channels start a fixed
        // number of elements further on in each tensor, which needs whole channel blocks per group.
        auto group_step = [](const Dim2 &c, int64_t extent, int64_t per_group, int64_t *step) {
            if (c.f >= extent) { *step = per_group * c.si; return true; }
            if (per_group % c.f) return false;
            *step = per_group / c.f * c.so;
            return true;
        };
        int64_t sx, sw, sy;
        if (!group_step(p.xc, d->C, Cg, &sx) || !group_step(p.wo, d->K, Kg, &sw) || !group_step(p.yk, d->K, Kg, &sy))
            return fail(h, ALT_UNSUPPORTED, "conv2d: a channel block of a layout straddles two groups");
        p.C = (int32_t)Cg; p.Nc = (int32_t)Kg; p.Kg = (int32_t)(Cg * d->R * d->S);
        p.batch = (int32_t)G;
        p.x_bstride = sx; p.w_bstride = sw; p.y_bstride = sy;
        p.bias_bstride = (int32_t)Kg;
    }
    igemm_analyse(pb);
    return ALT_OK;
}

alt_status_t gemm_problem(alt_handle_t h, const alt_gemm_desc_t *d, const void *A, const void *B, void *C,
                          Problem *pb)
{
    if (!d) return fail(h, ALT_INVALID_ARG, "null descriptor");
    if (d->batch < 1 || d->M < 1 || d->N < 1 || d->K < 1) return fail(h, ALT_INVALID_ARG, "gemm: non-positive extent");
    if ((d->in_dtype != ALT_F32 && d->in_dtype != ALT_BF16) || (d->out_dtype != ALT_F32 && d->out_dtype != ALT_BF16))
        return fail(h, ALT_INVALID_ARG, "gemm: bad dtype");
    const int64_t as[2] = {d->M, d->K}, bs[2] = {d->K, d->N}, cs[2] = {d->M, d->N};
    BoundLayout ba, bb, bc;
    std::string err;
    alt_status_t s;
    if ((s = bind_layout(&d->a_layout, 2, as, &ba, &err)) != ALT_OK) return fail(h, s, "a_layout: %s", err.c_str());
    if ((s = bind_layout(&d->b_layout, 2, bs, &bb, &err)) != ALT_OK) return fail(h, s, "b_layout: %s", err.c_str());
    if ((s = bind_layout(&d->c_layout, 2, cs, &bc, &err)) != ALT_OK) return fail(h, s, "c_layout: %s", err.c_str());
    Dim2 da[2], db[2], dc[2];
    if (!layout_to_dim2(ba, da) || !layout_to_dim2(bb, db) || !layout_to_dim2(bc, dc))
        return fail(h, ALT_UNSUPPORTED, "gemm: layouts must be separable with at most one block level per dimension");
    if (!fits32(d->M) || !fits32(d->N) || !fits32(d->K))
        return fail(h, ALT_UNSUPPORTED, "gemm: problem too large for 32-bit tile indices");
    std::memset(pb, 0, sizeof(*pb));
    pb->dtype = d->in_dtype;
    IgemmParams &p = pb->p;
    const Dim2 one = {1, 0, 0, 0, make_fastdiv(1)};
    p.x = A; p.w = B; p.y = C; p.bias = nullptr;
    p.M = (int32_t)d->M; p.Nc = (int32_t)d->N; p.Kg = (int32_t)d->K;
    p.C = (int32_t)d->K; p.H = 1; p.W = (int32_t)d->M; p.R = 1; p.S = 1; p.OH = 1; p.OW = (int32_t)d->M;
    p.stride_h = p.stride_w = 1; p.dil_h = p.dil_w = 1;
    p.batch = (int32_t)d->batch; p.splitk = 1;
    p.out_bf16 = d->out_dtype == ALT_BF16;
    p.x_bstride = d->M * d->K; p.w_bstride = d->K * d->N; p.y_bstride = d->M * d->N;
    p.xn = one; p.xc = da[1]; p.xh = one; p.xw = da[0];
    p.wo = db[1]; p.wi = db[0]; p.wr = one; p.ws = one;
    p.yn = one; p.yk = dc[1]; p.yh = one; p.yw = dc[0];
    pb->x_elems = ba.numel;
    pb->w_elems = bb.numel;
    {
        const int64_t yb = bc.numel * (int64_t)dtype_size(d->out_dtype);
        p.y_bytes = yb < 0x7fffffff ? (uint32_t)yb : 0;
    }
    p.x_bytes = (uint32_t)std::min<int64_t>(ba.numel * (int64_t)dtype_size(d->in_dtype), 0x7fffffff);
    p.w_bytes = (uint32_t)std::min<int64_t>(bb.numel * (int64_t)dtype_size(d->in_dtype), 0x7fffffff);
    igemm_analyse(pb);
    return ALT_OK;
}

}  // namespace alt

using namespace alt;

extern "C" {

alt_status_t alt_conv2d_output_shape(const alt_conv_desc_t *d, int64_t *out)
{
    if (!d || !out) return ALT_INVALID_ARG;
    if (d->stride_h < 1 || d->stride_w < 1 || d->dil_h < 1 || d->dil_w < 1) return ALT_INVALID_ARG;
    out[0] = d->N;
    out[1] = d->K;
    out[2] = (d->H + 2 * d->pad_h - d->dil_h * (d->R - 1) - 1) / d->stride_h + 1;
    out[3] = (d->W + 2 * d->pad_w - d->dil_w * (d->S - 1) - 1) / d->stride_w + 1;
    return (out[2] < 1 || out[3] < 1) ? ALT_INVALID_ARG : ALT_OK;
}

// ---- launch memo -------------------------------------------------------------------
// Turning a descriptor into launch parameters (three layouts bound, loaders analysed,
// with variant = -1 every kernel estimated) costs far more host time than the launch
// itself, and callers repeat the same few descriptors.  The handle remembers the last
// descriptors byte for byte, with what else the result depends on: 16-byte alignment
// of the buffers, the workspace size, the tune cache's generation.

struct MemoEntry {
    std::vector<unsigned char> desc;
    unsigned sig, gen;
    size_t ws_limit;
    Problem pb;
    int variant;
};

}  // extern "C"

struct alt_launch_memo {
    std::vector<MemoEntry> entries;
    size_t next = 0;
};

namespace alt {
void launch_memo_free(alt_handle_t h)
{
    delete h->memo;
    h->memo = nullptr;
}
}  // namespace alt

extern "C" {

static unsigned align_sig(const void *a, const void *b, const void *c, const void *d)
{
    return (unsigned)(((uintptr_t)a & 15) | (((uintptr_t)b & 15) << 4) | (((uintptr_t)c & 15) << 8) |
                      (((uintptr_t)d & 15) << 12) | ((c ? 1u : 0u) << 16));
}

static MemoEntry *memo_find(alt_handle_t h, const void *desc, size_t bytes, unsigned sig, size_t ws_limit)
{
    if (!h->memo) return nullptr;
    for (MemoEntry &e : h->memo->entries)
        if (e.sig == sig && e.gen == h->cache_gen && e.ws_limit == ws_limit && e.desc.size() == bytes &&
            std::memcmp(e.desc.data(), desc, bytes) == 0)
            return &e;
    return nullptr;
}

static void memo_store(alt_handle_t h, const void *desc, size_t bytes, unsigned sig, size_t ws_limit, const Problem &pb,
                       int variant)
{
    constexpr size_t kMemoEntries = 32;
    if (!h->memo) h->memo = new alt_launch_memo();
    MemoEntry e;
    e.desc.assign((const unsigned char *)desc, (const unsigned char *)desc + bytes);
    e.sig = sig; e.gen = h->cache_gen; e.ws_limit = ws_limit; e.pb = pb; e.variant = variant;
    auto &v = h->memo->entries;
    if (v.size() < kMemoEntries) v.push_back(std::move(e));
    else { v[h->memo->next] = std::move(e); h->memo->next = (h->memo->next + 1) % kMemoEntries; }
}

// variant = -1: the cached tuned variant if it applies and its split-K partial
// sums fit the workspace the caller brought, else the best-estimate variant
// that fits.
static int pick_variant(alt_handle_t h, const Problem &pb, int requested, const std::string &key, size_t ws_limit)
{
    if (requested >= 0) return requested;
    auto it = h->cache.find(key);
    if (it != h->cache.end()) {
        // a cached entry is only trusted if it still applies (pointers may be aligned differently)
        const auto &tab = igemm_table();
        int v = it->second.variant;
        if (v >= 0 && v < (int)tab.size() * kNumSplits &&
            igemm_applicable(pb, tab[v / kNumSplits], kSplits[v % kNumSplits], nullptr, nullptr) &&
            igemm_workspace(pb, kSplits[v % kNumSplits]) <= ws_limit)
            return v;
    }
    return igemm_default_variant(pb, ws_limit);
}

static alt_status_t conv2d_impl(alt_handle_t h, const alt_conv_desc_t *d, const void *x, const void *w, const float *bias,
                                const void *addend, void *y, void *workspace, size_t ws_bytes, void *stream, const char *who)
{
    if (!h) return ALT_INVALID_ARG;
    if (!d || !x || !w || !y) return fail(h, ALT_INVALID_ARG, "%s: null argument", who);
    if ((d->epilogue & ALT_EPI_BIAS) && !bias) return fail(h, ALT_INVALID_ARG, "%s: bias flag without bias", who);
    const size_t ws_limit = workspace ? ws_bytes : 0;
    const unsigned sig = align_sig(x, w, bias, y) | (addend ? 1u << 17 : 0u) | ((unsigned)((uintptr_t)addend & 15) << 18);
    if (MemoEntry *m = memo_find(h, d, sizeof *d, sig, ws_limit)) {
        m->pb.p.x = x; m->pb.p.w = w; m->pb.p.bias = bias; m->pb.p.y = y; m->pb.p.addend = addend;
        return igemm_run(h, m->pb, m->variant, workspace, ws_bytes, (hipStream_t)stream);
    }
    Problem pb;
    alt_status_t s = conv_problem(h, d, x, w, bias, y, &pb);
    if (s != ALT_OK) return s;
    if (addend) {
        if (pb.depthwise || pb.groups > 1) return fail(h, ALT_UNSUPPORTED, "%s: no fused sum for grouped convolutions", who);
        if ((uintptr_t)addend % 16) return fail(h, ALT_INVALID_ARG, "%s: the addend must be 16-byte aligned", who);
        pb.p.addend = addend;
    }
    if (pb.depthwise) return depthwise_run(h, pb, d->N, d->C, (hipStream_t)stream);
    // (a tuned choice for the same problem without the sum is a good one with it, if it applies)
    int v = pick_variant(h, pb, d->variant, d->variant >= 0 ? std::string() : conv_key(h, d), ws_limit);
    if (v < 0) return fail(h, ALT_UNSUPPORTED, "%s: no kernel variant applies", who);
    memo_store(h, d, sizeof *d, sig, ws_limit, pb, v);
    return igemm_run(h, pb, v, workspace, ws_bytes, (hipStream_t)stream);
}

alt_status_t alt_conv2d(alt_handle_t h, const alt_conv_desc_t *d, const void *x, const void *w, const float *bias,
                        void *y, void *workspace, size_t ws_bytes, void *stream)
{
    return conv2d_impl(h, d, x, w, bias, nullptr, y, workspace, ws_bytes, stream, "alt_conv2d");
}

// ---- alt_conv2d without a caller's workspace ---------------------------------------------
// The split-K partial tiles of alt_conv2d_static live in this array instead of a workspace
// the caller brings.  The name below is a host-side stand-in: the array's device address is
// looked up once per device (static_scratch) and that pointer is what kernels get.
constexpr size_t kStaticScratchBytes = ALT_STATIC_WORKSPACE_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static void *g_scratch_ptr[16];
static std::mutex g_scratch_mutex;

}  // extern "C"

namespace alt {
// Device address of `scratch` on the current device; first use on a device asks the runtime.
hipError_t static_scratch(void **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 16) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}
}  // namespace alt

extern "C" {

alt_status_t alt_conv2d_static(alt_handle_t h, const alt_conv_desc_t *d, const void *x, const void *w, const float *bias,
                               void *y, void *stream)
{
    if (!h) return ALT_INVALID_ARG;
    if (!h->has_gpu) return fail(h, ALT_HIP_ERROR, "no GPU device available");
    void *ws = nullptr;
    hipError_t e = static_scratch(&ws);
    if (e != hipSuccess) return fail(h, ALT_HIP_ERROR, "alt_conv2d_static: no address for the static workspace: %s", hipGetErrorString(e));
    // (an explicitly requested variant whose partial tiles exceed the array fails in igemm_run with
    // ALT_WORKSPACE_TOO_SMALL and the two sizes; variant = -1 only picks variants that fit)
    return conv2d_impl(h, d, x, w, bias, nullptr, y, ws, kStaticScratchBytes, stream, "alt_conv2d_static");
}

alt_status_t alt_conv2d_add(alt_handle_t h, const alt_conv_desc_t *d, const void *x, const void *w, const float *bias,
                            const void *addend, void *y, void *workspace, size_t ws_bytes, void *stream)
{
    if (h && !addend) return fail(h, ALT_INVALID_ARG, "alt_conv2d_add: null addend");
    return conv2d_impl(h, d, x, w, bias, addend, y, workspace, ws_bytes, stream, "alt_conv2d_add");
}

alt_status_t alt_conv2d_multi(alt_handle_t h, const alt_conv_call_t *calls, int32_t n)
{
    if (!h) return ALT_INVALID_ARG;
    if (n < 0 || (n > 0 && !calls)) return fail(h, ALT_INVALID_ARG, "alt_conv2d_multi: bad call list");
    for (int32_t i = 0; i < n; ++i) {
        const alt_conv_call_t &c = calls[i];
        alt_status_t s = alt_conv2d(h, c.d, c.x, c.w, c.bias, c.y, c.workspace, c.ws_bytes, c.stream);
        if (s != ALT_OK) return s;
    }
    return ALT_OK;
}

alt_status_t alt_conv2d_workspace_size(alt_handle_t h, const alt_conv_desc_t *d, size_t *bytes)
{
    if (!h) return ALT_INVALID_ARG;
    if (!d || !bytes) return fail(h, ALT_INVALID_ARG, "null argument");
    Problem pb;
    // alignment of real pointers is unknown here: assume 16-byte aligned buffers
    alt_status_t s = conv_problem(h, d, (void *)16, (void *)16, nullptr, (void *)16, &pb);
    if (s != ALT_OK) return s;
    if (pb.depthwise) { *bytes = 0; return ALT_OK; }
    int v = pick_variant(h, pb, d->variant, conv_key(h, d), (size_t)-1);
    if (v < 0) return fail(h, ALT_UNSUPPORTED, "no kernel variant applies");
    *bytes = igemm_workspace(pb, kSplits[v % kNumSplits]);
    return ALT_OK;
}

alt_status_t alt_conv2d_variant_count(alt_handle_t h, const alt_conv_desc_t *d, int *count)
{
    if (!h) return ALT_INVALID_ARG;
    if (!d || !count) return fail(h, ALT_INVALID_ARG, "null argument");
    *count = igemm_variant_count();
    return ALT_OK;
}

alt_status_t alt_conv2d_variant_name(alt_handle_t h, const alt_conv_desc_t *d, int variant, char *buf, size_t buflen)
{
    if (!h) return ALT_INVALID_ARG;
    if (!d || !buf || buflen == 0) return fail(h, ALT_INVALID_ARG, "null argument");
    Problem pb;
    alt_status_t s = conv_problem(h, d, (void *)16, (void *)16, nullptr, (void *)16, &pb);
    if (s != ALT_OK) return s;
    if (pb.depthwise) return fail(h, ALT_UNSUPPORTED, "depth-wise convolutions have no kernel variants");
    if (variant < 0) {                               // the variant alt_conv2d would run with variant = -1 and any workspace
        variant = pick_variant(h, pb, -1, conv_key(h, d), (size_t)-1);
        if (variant < 0) return fail(h, ALT_UNSUPPORTED, "no kernel variant applies");
    }
    std::string n = igemm_variant_name(variant);
    if (n.empty()) return fail(h, ALT_INVALID_ARG, "variant %d out of range", variant);
    std::snprintf(buf, buflen, "%s", n.c_str());
    std::string why;
    const auto &tab = igemm_table();
    if (!igemm_applicable(pb, tab[variant / kNumSplits], kSplits[variant % kNumSplits], nullptr, &why))
        return fail(h, ALT_UNSUPPORTED, "%s: %s", n.c_str(), why.c_str());
    return ALT_OK;
}

alt_status_t alt_pack_weights(alt_handle_t h, const alt_conv_desc_t *d, const void *w_oihw, void *w_packed, void *stream)
{
    if (!h) return ALT_INVALID_ARG;
    if (!d || !w_oihw || !w_packed) return fail(h, ALT_INVALID_ARG, "alt_pack_weights: null argument");
    const int64_t G = d->groups > 1 ? d->groups : 1;
    if (d->C % G) return fail(h, ALT_INVALID_ARG, "alt_pack_weights: groups must divide C");
    const int64_t wsh[4] = {d->K, d->C / G, d->R, d->S};
    alt_layout_t plain;
    alt_layout_parse("OIHW->OIHW", &plain);
    BoundLayout bs, bd;
    std::string err;
    alt_status_t s;
    if ((s = bind_layout(&plain, 4, wsh, &bs, &err)) != ALT_OK) return fail(h, s, "%s", err.c_str());
    if ((s = bind_layout(&d->w_layout, 4, wsh, &bd, &err)) != ALT_OK) return fail(h, s, "w_layout: %s", err.c_str());
    return transform_bound(h, (int)dtype_size(d->in_dtype), bs, w_oihw, bd, w_packed, (hipStream_t)stream);
}

alt_status_t alt_gemm(alt_handle_t h, const alt_gemm_desc_t *d, const void *A, const void *B, void *C,
                      void *workspace, size_t ws_bytes, void *stream)
{
    if (!h) return ALT_INVALID_ARG;
    if (!d || !A || !B || !C) return fail(h, ALT_INVALID_ARG, "alt_gemm: null argument");
    const size_t ws_limit = workspace ? ws_bytes : 0;
    const unsigned sig = align_sig(A, B, nullptr, C);
    if (MemoEntry *m = memo_find(h, d, sizeof *d, sig, ws_limit)) {
        m->pb.p.x = A; m->pb.p.w = B; m->pb.p.y = C;
        return igemm_run(h, m->pb, m->variant, workspace, ws_bytes, (hipStream_t)stream);
    }
    Problem pb;
    alt_status_t s = gemm_problem(h, d, A, B, C, &pb);
    if (s != ALT_OK) return s;
    int v = pick_variant(h, pb, d->variant, d->variant >= 0 ? std::string() : gemm_key(h, d), ws_limit);
    if (v < 0) return fail(h, ALT_UNSUPPORTED, "alt_gemm: no kernel variant applies");
    memo_store(h, d, sizeof *d, sig, ws_limit, pb, v);
    return igemm_run(h, pb, v, workspace, ws_bytes, (hipStream_t)stream);
}

alt_status_t alt_splitk_status(alt_handle_t h, alt_splitk_status_t *out)
{
    if (!h) return ALT_INVALID_ARG;
    if (!out) return fail(h, ALT_INVALID_ARG, "alt_splitk_status: null argument");
    std::memset(out, 0, sizeof *out);
    if (!h->has_gpu) return fail(h, ALT_HIP_ERROR, "no GPU device available");
    int bound = 0, nonzero = 0;
    dconv_splitk_state(&bound, &nonzero);
    out->streams_bound = bound; out->counters_nonzero = nonzero;
    out->max_streams = kDconvSlots;
    if (nonzero < 0) return fail(h, ALT_HIP_ERROR, "alt_splitk_status: could not read the counters");
    return ALT_OK;
}

alt_status_t alt_gemm_workspace_size(alt_handle_t h, const alt_gemm_desc_t *d, size_t *bytes)
{
    if (!h) return ALT_INVALID_ARG;
    if (!d || !bytes) return fail(h, ALT_INVALID_ARG, "null argument");
    Problem pb;
    alt_status_t s = gemm_problem(h, d, (void *)16, (void *)16, (void *)16, &pb);
    if (s != ALT_OK) return s;
    int v = pick_variant(h, pb, d->variant, gemm_key(h, d), (size_t)-1);
    if (v < 0) return fail(h, ALT_UNSUPPORTED, "no kernel variant applies");
    *bytes = igemm_workspace(pb, kSplits[v % kNumSplits]);
    return ALT_OK;
}

alt_status_t alt_gemm_variant_count(alt_handle_t h, const alt_gemm_desc_t *d, int *count)
{
    if (!h) return ALT_INVALID_ARG;
    if (!d || !count) return fail(h, ALT_INVALID_ARG, "null argument");
    *count = igemm_variant_count();
    return ALT_OK;
}

alt_status_t alt_gemm_variant_name(alt_handle_t h, const alt_gemm_desc_t *d, int variant, char *buf, size_t buflen)
{
    if (!h) return ALT_INVALID_ARG;
    if (!d || !buf || buflen == 0) return fail(h, ALT_INVALID_ARG, "null argument");
    Problem pb;
    alt_status_t s = gemm_problem(h, d, (void *)16, (void *)16, (void *)16, &pb);
    if (s != ALT_OK) return s;
    if (variant < 0) {                               // the variant alt_gemm would run with variant = -1 and any workspace
        variant = pick_variant(h, pb, -1, gemm_key(h, d), (size_t)-1);
        if (variant < 0) return fail(h, ALT_UNSUPPORTED, "no kernel variant applies");
    }
    std::string n = igemm_variant_name(variant);
    if (n.empty()) return fail(h, ALT_INVALID_ARG, "variant %d out of range", variant);
    std::snprintf(buf, buflen, "%s", n.c_str());
    std::string why;
    const auto &tab = igemm_table();
    if (!igemm_applicable(pb, tab[variant / kNumSplits], kSplits[variant % kNumSplits], nullptr, &why))
        return fail(h, ALT_UNSUPPORTED, "%s: %s", n.c_str(), why.c_str());
    return ALT_OK;
}

}  // extern "C"

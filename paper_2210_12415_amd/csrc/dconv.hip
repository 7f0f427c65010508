// Host side of the patch-resident direct convolution (dconv.h) and of the
// streaming kernel (dstream.h): which problems each covers, their launch
// parameters, and the arrival counters of the fused split-K reduction.
#include <atomic>

#include "dstream.h"
#include "ops.h"

namespace alt {

namespace {

// Arrival counters of the fused split-K reduction: zero when the module is
// loaded, and every launch leaves them zero again.  kDconvSlots sets are
// handed out round-robin so that launches in flight on different streams do
// not share one (more than kDconvSlots overlapping split-K launches would).
__device__ __align__(256) uint32_t g_dconv_counters[kDconvSlots * kDconvMaxTiles];

constexpr int kMaxDevices = 16;
uint32_t *g_counter_ptr[kMaxDevices];
int g_round_robin[kMaxDevices];      // 0 = not probed, 1 = workgroup ids go round the XCDs in order, -1 = they do not

// Each workgroup reports the XCD it runs on.
__global__ void xcd_probe_kernel(uint32_t *out)
{
    if (threadIdx.x == 0) out[blockIdx.x] = __builtin_amdgcn_s_getreg(GETREG_IMMED(3, 0, 20)) & 0xf;   // XCC_ID
}
std::atomic<unsigned> g_next_slot{0};

bool dense(const Dim2 &d, int64_t extent, int64_t stride)
{
    return extent == 1 || (d.f >= extent && d.si == stride);
}

}  // namespace

// Device address of the counters on the current device (looked up once per device).
hipError_t dconv_counters(uint32_t **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    if (!g_counter_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_dconv_counters));
        if (e != hipSuccess) return e;
        g_counter_ptr[dev] = (uint32_t *)ptr;
    }
    *out = g_counter_ptr[dev];
    return hipSuccess;
}

// Whether workgroup i of a launch runs on the same XCD as every workgroup j with
// j = i (mod 8), which lets the slices of a split-K tile meet in one L2.  Probed once per
// device with a small launch whose workgroups report their XCD, using the counter array
// as scratch (it is zeroed again); synchronises, so it runs when a handle is created.
bool dconv_round_robin_xcds()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return false;
    if (g_round_robin[dev] != 0) return g_round_robin[dev] > 0;
    g_round_robin[dev] = -1;
    if (const char *e = std::getenv("ALT_SPLITK_SCOPE"))
        if (std::strcmp(e, "device") == 0) return false;
    uint32_t *buf = nullptr;
    if (dconv_counters(&buf) != hipSuccess) return false;
    constexpr int kBlocks = 1024;
    static_assert(kBlocks <= kDconvSlots * kDconvMaxTiles, "probe scratch");
    uint32_t host[kBlocks];
    bool ok = true;
    for (int rep = 0; rep < 3 && ok; ++rep) {
        hipLaunchKernelGGL(xcd_probe_kernel, dim3(kBlocks), dim3(64), 0, 0, buf);
        if (hipMemcpy(host, buf, sizeof host, hipMemcpyDeviceToHost) != hipSuccess) { ok = false; break; }
        for (int b = 8; b < kBlocks; ++b) ok = ok && host[b] == host[b & 7];
    }
    (void)hipMemset(buf, 0, sizeof host);
    (void)hipDeviceSynchronize();
    if (ok) g_round_robin[dev] = 1;
    return ok;
}

// The same for a streaming kernel (dstream.h): 1x1 filters, stride 1, no padding (a GEMM
// is lowered to that), any number of channels that splits into 64-channel steps.
static bool dstream_setup(const Problem &pb, const IgemmLaunch &k, int splitk, DconvParams *out, size_t *lds_bytes,
                          std::string *why)
{
    auto no = [&](const char *m) { if (why) *why = m; return false; };
    const IgemmParams &p = pb.p;
    if (pb.dtype != ALT_BF16) return no("streaming kernel is bf16 only");
    if (p.R != 1 || p.S != 1 || p.stride_h != 1 || p.stride_w != 1 || p.pad_h != 0 || p.pad_w != 0)
        return no("streaming kernel needs a 1x1 filter, stride 1, no padding");
    if (p.OH != p.H || p.OW != p.W) return no("streaming kernel needs output size = input size");
    const int64_t C = p.C, H = p.H, W = p.W, K = p.Nc, N = p.M / (H * W);
    if (!(dense(p.xc, C, 1) && dense(p.xw, W, C) && dense(p.xh, H, W * C) && dense(p.xn, N, H * W * C)))
        return no("A is not dense with K contiguous");
    if (!(dense(p.wi, C, 1) && dense(p.wo, K, C))) return no("B is not dense with K contiguous");
    if (!(dense(p.yk, K, 1) && dense(p.yw, W, K) && dense(p.yh, H, W * K) && dense(p.yn, N, H * W * K)))
        return no("output is not dense with N contiguous");
    const int64_t osz = p.out_bf16 ? 2 : 4;
    if ((uintptr_t)p.x % 16 || (uintptr_t)p.w % 16 || (uintptr_t)p.y % 16) return no("operands are not 16-byte aligned");
    if (p.batch > 1 && ((p.x_bstride * 2) % 16 || (p.w_bstride * 2) % 16 || (p.y_bstride * osz) % 16))
        return no("batch entries are not 16-byte aligned");
    if (p.batch > 65535) return no("too many batch entries for one launch");
    if (p.addend && p.batch > 1) return no("the fused sum is not built for batched problems");
    if (splitk < 1 || (splitk > 1 && p.batch > 1)) return no("split-K is not built for batched problems");
    if (C % ((int64_t)k.BK * splitk * k.kw)) return no("K does not split into whole steps per slice and K group");
    if (pb.x_elems * 2 >= 0x7fffffff || pb.w_elems * 2 >= 0x7fffffff || p.y_bytes == 0)
        return no("operand of 2 GiB or more");
    if ((int64_t)p.M * K * 4 >= 0x7fffffff) return no("output too large for 32-bit offsets");
    if (K % 4 || (p.epilogue & ALT_EPI_BIAS && (uintptr_t)p.bias % 16)) return no("streaming kernel stores four output columns at a time");
    const size_t lds = dstream_lds_bytes(k.BM, k.BN, k.BK, k.prefetch + 1, k.wgn, k.kw);
    if (lds > 160 * 1024) return no("stages do not fit LDS");
    const int tiles_m = (p.M + k.BM - 1) / k.BM, tiles_n = (p.Nc + k.BN - 1) / k.BN;
    if (splitk > 1 && (int64_t)tiles_m * tiles_n > kDconvMaxTiles) return no("too many output tiles for the split-K counters");
    if ((int64_t)tiles_m * tiles_n * splitk > 0x7fffffff) return no("grid too large");
    if (!out) return true;
    DconvParams d;
    std::memset(&d, 0, sizeof d);
    d.x = p.x; d.w = p.w; d.bias = p.bias; d.y = p.y; d.addend = p.addend;
    d.x_bytes = p.x_bytes; d.w_bytes = p.w_bytes; d.y_bytes = p.y_bytes;
    d.partial_bytes = (uint32_t)((int64_t)p.M * K * 4);
    d.M = p.M; d.Nc = p.Nc; d.C = p.C; d.Cs = (int32_t)(C / splitk);
    d.H = p.H; d.W = p.W; d.R = 1; d.S = 1;
    d.tiles_m = tiles_m; d.tiles_n = tiles_n; d.splitk = splitk;
    d.flags = (p.epilogue & (ALT_EPI_BIAS | ALT_EPI_RELU)) | (p.out_bf16 ? kDconvOutBf16 : 0);
    d.d_hw = make_div32((uint32_t)(p.H * p.W));
    d.d_w = make_div32((uint32_t)p.W);
    d.d_tm = make_div32((uint32_t)tiles_m);
    d.d_tn = make_div32((uint32_t)tiles_n);
    d.ncc = (int32_t)(C / splitk / k.kw / k.BK);
    d.bk = k.BK;
    d.d_sk = make_div32((uint32_t)splitk);
    d.batch = p.batch;
    d.x_bstride = p.x_bstride * 2; d.w_bstride = p.w_bstride * 2; d.y_bstride = p.y_bstride * osz;
    {
        int dev = 0;
        d.xcd_local = splitk > 1 && hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < kMaxDevices &&
                      g_round_robin[dev] > 0 && (int64_t)(tiles_m * tiles_n + 7) / 8 * 8 * splitk <= 0x7fffffff;
    }
    *out = d;
    *lds_bytes = lds;
    return true;
}

// Fills the launch parameters of direct kernel `k` for `pb` split into `splitk`
// channel slices, or says why the kernel does not cover the problem.
bool dconv_setup(const Problem &pb, const IgemmLaunch &k, int splitk, DconvParams *out, size_t *lds_bytes, std::string *why)
{
    if (k.stream) return dstream_setup(pb, k, splitk, out, lds_bytes, why);
    auto no = [&](const char *m) { if (why) *why = m; return false; };
    const IgemmParams &p = pb.p;
    if (pb.dtype != ALT_BF16) return no("direct kernel is bf16 only");
    if (p.batch != 1) return no("direct kernel takes no batch");
    if (p.stride_h != p.stride_w || (p.stride_h != 1 && p.stride_h != 2) || p.dil_h != p.dil_w || p.dil_h < 1)
        return no("direct kernel needs stride 1 or 2 and one dilation for both directions");
    if (p.pad_h < 0 || p.pad_w < 0 || 2 * p.pad_h > p.dil_h * (p.R - 1) || 2 * p.pad_w > p.dil_w * (p.S - 1))
        return no("direct kernel needs padding between none and same-size");
    const int st_ = p.stride_h;
    // (then OH <= ceil(H / stride) and likewise OW: the input pixel under an output pixel never moves backwards)
    if ((int64_t)(p.OH - 1) * st_ >= p.H || (int64_t)(p.OW - 1) * st_ >= p.W) return no("output larger than the strided input");
    const int64_t C = p.C, H = p.H, W = p.W, OH = p.OH, OW = p.OW, K = p.Nc, R = p.R, S = p.S, N = p.M / (OH * OW);
    if (!(dense(p.xc, C, 1) && dense(p.xw, W, C) && dense(p.xh, H, W * C) && dense(p.xn, N, H * W * C)))
        return no("activations are not dense NHWC");
    if (!(dense(p.wi, C, 1) && dense(p.ws, S, C) && dense(p.wr, R, S * C) && dense(p.wo, K, R * S * C)))
        return no("weights are not dense OHWI");
    if (!(dense(p.yk, K, 1) && dense(p.yw, OW, K) && dense(p.yh, OH, OW * K) && dense(p.yn, N, OH * OW * K)))
        return no("output is not dense NHWC");
    if ((uintptr_t)p.x % 16 || (uintptr_t)p.w % 16) return no("operands are not 16-byte aligned");
    if (splitk < 1 || C % splitk) return no("split factor does not divide the channels");
    const int64_t Cs = C / splitk;
    if (Cs % 64 || (Cs & (Cs - 1)) || Cs > 512) return no("channels per slice must be 64, 128, 256 or 512");
    // K groups: each takes Cs / kw channels, in steps of k.BK (64, or 32: built for 3x3 filters over
    // 32 or 64 channels per group)
    const int kw = k.kw, bk = k.BK;
    if (Cs % kw) return no("K groups do not divide the slice");
    const int64_t Csg = Cs / kw;
    if (Csg % bk) return no("too few channels per K group");
    if (bk == 32 && !(R == 3 && S == 3 && Csg <= 64)) return no("32-channel K steps are built for 3x3 filters over 32 or 64 channels per group");
    if (pb.x_elems * 2 >= 0x7fffffff || pb.w_elems * 2 >= 0x7fffffff || p.y_bytes == 0)
        return no("operand of 2 GiB or more");
    if ((int64_t)p.M * K * 4 >= 0x7fffffff) return no("output too large for 32-bit offsets");
    if (K % 4 || (uintptr_t)p.y % 16 || ((p.epilogue & ALT_EPI_BIAS) && (uintptr_t)p.bias % 16))
        return no("direct kernel stores four output channels at a time");
    const size_t lds = dconv_lds_bytes(k.BM, k.BN, k.prefetch + 1, k.wgn, kw, bk, (int)Cs,
                                       dconv_patch_pixels(k.BM, p.M, p.H, p.W, p.OH, p.OW, p.R, p.S, p.pad_h, p.pad_w, st_, p.dil_h));
    if (lds > 160 * 1024) return no("patch does not fit LDS");
    const int tiles_m = (p.M + k.BM - 1) / k.BM, tiles_n = (p.Nc + k.BN - 1) / k.BN;
    if (splitk > 1 && (int64_t)tiles_m * tiles_n > kDconvMaxTiles) return no("too many output tiles for the split-K counters");
    if ((int64_t)tiles_m * tiles_n * splitk > 0x7fffffff) return no("grid too large");
    if (!out) return true;
    DconvParams d;
    std::memset(&d, 0, sizeof d);
    d.x = p.x; d.w = p.w; d.bias = p.bias; d.y = p.y; d.addend = p.addend;
    d.x_bytes = p.x_bytes; d.w_bytes = p.w_bytes; d.y_bytes = p.y_bytes;
    d.partial_bytes = (uint32_t)((int64_t)p.M * K * 4);
    d.M = p.M; d.Nc = p.Nc; d.C = p.C; d.Cs = (int32_t)Cs;
    d.H = p.H; d.W = p.W; d.R = p.R; d.S = p.S; d.pad_h = p.pad_h; d.pad_w = p.pad_w;
    d.tiles_m = tiles_m; d.tiles_n = tiles_n; d.splitk = splitk;
    d.flags = (p.epilogue & (ALT_EPI_BIAS | ALT_EPI_RELU)) | (p.out_bf16 ? kDconvOutBf16 : 0);
    d.OH = p.OH; d.OW = p.OW; d.stride = st_; d.dil = p.dil_h;
    if (N * H * W > 0x7fffffff) return no("input too large for 32-bit pixel indices");
    d.in_px = (int32_t)(N * H * W);
    d.d_hw = make_div32((uint32_t)(p.OH * p.OW));
    d.d_w = make_div32((uint32_t)p.OW);
    d.d_tm = make_div32((uint32_t)tiles_m);
    d.d_tn = make_div32((uint32_t)tiles_n);
    int l2 = 0;
    while ((8 << l2) < Cs) ++l2;
    d.log2_cpp = l2;
    d.d_slots = make_div32((uint32_t)(Cs / 8 + 1));
    d.ncc = (int32_t)(Csg / bk);
    d.bk = bk;
    d.d_sk = make_div32((uint32_t)splitk);
    {
        int dev = 0;
        d.xcd_local = splitk > 1 && hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < kMaxDevices &&
                      g_round_robin[dev] > 0 && (int64_t)(tiles_m * tiles_n + 7) / 8 * 8 * splitk <= 0x7fffffff;
    }
    *out = d;
    *lds_bytes = lds;
    return true;
}

hipError_t dconv_run(const IgemmLaunch &k, DconvParams d, size_t lds, float *partial, hipStream_t st)
{
    if (d.splitk > 1) {
        uint32_t *base = nullptr;
        hipError_t e = dconv_counters(&base);
        if (e != hipSuccess) return e;
        d.counters = base + (size_t)(g_next_slot.fetch_add(1) % kDconvSlots) * kDconvMaxTiles;
        d.partial = partial;
    }
#ifdef ALT_PHASE_TIMING
    if (d.splitk == 1) d.partial = partial;    // developer builds: workgroup timestamps go to the workspace
#endif
    return k.launch_direct(d, lds, st);
}

}  // namespace alt

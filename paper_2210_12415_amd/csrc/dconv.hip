// Host side of the patch-resident direct convolution (dconv.h) and of the
// streaming kernel (dstream.h): which problems each covers, their launch
// parameters, and the arrival counters of the fused split-K reduction.
#include <mutex>

#include "dplanar.h"
#include "dstream.h"
#include "ops.h"

namespace alt {

namespace {

// Arrival counters of the fused split-K reduction: zero when the module is
// loaded, and every launch leaves them zero again.  There are kDconvSlots sets;
// a set is bound to the first stream that issues a split-K launch and stays
// with it (launches on one stream run one after the other, so they can share
// a set; launches on different streams never do).
__device__ __align__(256) uint32_t g_dconv_counters[kDconvSlots * kDconvMaxTiles];
constexpr int kMaxDevices = 16;

struct SlotTable {
    hipStream_t stream[kDconvSlots];
    bool used[kDconvSlots], pinned[kDconvSlots];   // pinned: a captured graph carries this set's address
};

struct DeviceState {
    uint32_t *counters = nullptr;
    SlotTable slots{};
};
DeviceState g_dev[kMaxDevices];
std::mutex g_mutex;

bool dense(const Dim2 &d, int64_t extent, int64_t stride)
{
    return extent == 1 || (d.f >= extent && d.si == stride);
}

// Whether four per-dimension maps describe a dense activation tensor with the channels of a pixel contiguous
// (NHWC: *blk = 0) or in blocks of b = 2^*blk >= 8 channels (N C/b H W b, b dividing C).
bool nhwc_or_blocked(const Dim2 &c, const Dim2 &w, const Dim2 &h, const Dim2 &n, int64_t C, int64_t H, int64_t W, int64_t N,
                     int *blk)
{
    if (dense(c, C, 1) && dense(w, W, C) && dense(h, H, W * C) && dense(n, N, H * W * C)) { *blk = 0; return true; }
    const int64_t b = c.f;
    if (c.si != 1 || b < 8 || b >= C || (b & (b - 1)) || C % b || c.so != H * W * b) return false;
    if (!(dense(w, W, b) && dense(h, H, W * b) && dense(n, N, C * H * W))) return false;
    int l = 0;
    while (((int64_t)1 << l) < b) ++l;
    *blk = l;
    return true;
}

DeviceState *device_state()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    return &g_dev[dev];
}

}  // namespace

// Device address of the counters on the current device (looked up once per device).
hipError_t dconv_counters(uint32_t **out)
{
    DeviceState *ds = device_state();
    if (!ds) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_mutex);
    if (!ds->counters) {
        void *ptr = nullptr;
        hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_dconv_counters));
        if (e != hipSuccess) return e;
        ds->counters = (uint32_t *)ptr;
    }
    *out = ds->counters;
    return hipSuccess;
}

// Counter sets bound to streams on the current device, and how many counters are not zero once
// the device is idle (-1 if they cannot be read): waits for the device.
void dconv_splitk_state(int *slots_bound, int *counters_nonzero)
{
    DeviceState *ds = device_state();
    *slots_bound = 0;
    *counters_nonzero = -1;
    if (!ds) return;
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        for (int i = 0; i < kDconvSlots; ++i) *slots_bound += ds->slots.used[i] ? 1 : 0;
    }
    uint32_t *base = nullptr;
    if (dconv_counters(&base) != hipSuccess || hipDeviceSynchronize() != hipSuccess) return;
    std::vector<uint32_t> host((size_t)kDconvSlots * kDconvMaxTiles);
    if (hipMemcpy(host.data(), base, host.size() * 4, hipMemcpyDeviceToHost) != hipSuccess) return;
    int nz = 0;
    for (uint32_t v : host) nz += v != 0;
    *counters_nonzero = nz;
}

// The counter set of `st` on the current device: the one bound to it, else a free one.  When
// every set is bound the host waits until the device is idle and releases all sets except
// those a captured graph carries the address of.  hipErrorNotReady if that leaves none, or
// if the wait would be needed while `st` is being captured.
static hipError_t counter_slot(DeviceState *ds, hipStream_t st, int *slot)
{
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (st) (void)hipStreamIsCapturing(st, &cap);
    const bool capturing = cap != hipStreamCaptureStatusNone;
    std::lock_guard<std::mutex> lock(g_mutex);
    SlotTable &t = ds->slots;
    int free_slot = -1;
    for (int i = 0; i < kDconvSlots; ++i) {
        if (t.used[i] && t.stream[i] == st) { t.pinned[i] |= capturing; *slot = i; return hipSuccess; }
        if (!t.used[i] && free_slot < 0) free_slot = i;
    }
    if (free_slot < 0) {
        // Every set is bound.  Sets whose address a captured graph carries stay; the others are
        // released once nothing is in flight on the device.
        if (capturing) return hipErrorNotReady;
        hipError_t e = hipDeviceSynchronize();
        if (e != hipSuccess) return e;
        for (int i = 0; i < kDconvSlots; ++i)
            if (!t.pinned[i]) { t.used[i] = false; if (free_slot < 0) free_slot = i; }
        if (free_slot < 0) return hipErrorNotReady;
    }
    t.used[free_slot] = true;
    t.pinned[free_slot] = capturing;
    t.stream[free_slot] = st;
    *slot = free_slot;
    return hipSuccess;
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
    int x_blk = 0, y_blk = 0;
    if (!nhwc_or_blocked(p.xc, p.xw, p.xh, p.xn, C, H, W, N, &x_blk)) return no("A is not dense with K contiguous (whole or in blocks)");
    if (x_blk && k.BK % (1 << x_blk)) return no("channel blocks larger than a K step");
    if (k.bt) {
        if (!(dense(p.wo, K, 1) && dense(p.wi, C, K))) return no("B is not dense with N contiguous");
        if (K % 8) return no("row-major B is loaded eight columns at a time");
    } else if (!(dense(p.wi, C, 1) && dense(p.wo, K, C))) {
        return no("B is not dense with K contiguous");
    }
    if (!nhwc_or_blocked(p.yk, p.yw, p.yh, p.yn, K, H, W, N, &y_blk)) return no("output is not dense with N contiguous (whole or in blocks)");
    if ((x_blk || y_blk) && p.batch > 1) return no("blocked tensors are not built for batched problems");
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
    const size_t lds = dstream_lds_bytes(k.BM, k.BN, k.BK, k.prefetch + 1, k.wgm, k.wgn, k.kw);
    if (lds > 160 * 1024) return no("stages do not fit LDS");
    if (dstream_banded(k.BM, k.BN, k.wgn, k.kw) && splitk > 1) return no("tiles this large take no split-K");
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
    d.OH = p.H; d.OW = p.W; d.x_blk = x_blk; d.y_blk = y_blk;
    d.d_ihw = make_div32((uint32_t)(p.H * p.W));
    d.x_bstride = p.x_bstride * 2; d.w_bstride = p.w_bstride * 2; d.y_bstride = p.y_bstride * osz;
    *out = d;
    *lds_bytes = lds;
    return true;
}

// The same for a channel-planar kernel (dplanar.h): NCHW activations, OIHW weights, NCHW output, all dense.
static bool dplanar_setup(const Problem &pb, const IgemmLaunch &k, int splitk, DconvParams *out, size_t *lds_bytes,
                          std::string *why)
{
    auto no = [&](const char *m) { if (why) *why = m; return false; };
    const IgemmParams &p = pb.p;
    if (pb.dtype != ALT_BF16) return no("planar kernel is bf16 only");
    if (p.batch != 1) return no("planar kernel takes no batch");
    if (splitk != 1) return no("planar kernel takes no split-K");
    if (p.addend) return no("planar kernel has no fused sum");
    if (!((p.R == 3 && p.S == 3) || (p.R == 1 && p.S == 1))) return no("planar kernel is built for 1x1 and 3x3 filters");
    if (p.stride_h != p.stride_w || (p.stride_h != 1 && p.stride_h != 2) || p.dil_h != p.dil_w || p.dil_h < 1)
        return no("planar kernel needs stride 1 or 2 and one dilation for both directions");
    if (p.pad_h < 0 || p.pad_w < 0 || 2 * p.pad_h > p.dil_h * (p.R - 1) || 2 * p.pad_w > p.dil_w * (p.S - 1))
        return no("planar kernel needs padding between none and same-size");
    const int st_ = p.stride_h;
    if ((int64_t)(p.OH - 1) * st_ >= p.H || (int64_t)(p.OW - 1) * st_ >= p.W) return no("output larger than the strided input");
    const int64_t C = p.C, H = p.H, W = p.W, OH = p.OH, OW = p.OW, K = p.Nc, R = p.R, S = p.S, N = p.M / (OH * OW);
    if (!(dense(p.xw, W, 1) && dense(p.xh, H, W) && dense(p.xc, C, H * W) && dense(p.xn, N, C * H * W)))
        return no("activations are not dense NCHW");
    if (!(dense(p.ws, S, 1) && dense(p.wr, R, S) && dense(p.wi, C, R * S) && dense(p.wo, K, C * R * S)))
        return no("weights are not dense OIHW");
    const bool y_nchw = dense(p.yw, OW, 1) && dense(p.yh, OH, OW) && dense(p.yk, K, OH * OW) && dense(p.yn, N, K * OH * OW);
    const bool y_nhwc = dense(p.yk, K, 1) && dense(p.yw, OW, K) && dense(p.yh, OH, OW * K) && dense(p.yn, N, OH * OW * K);
    if (!y_nchw && !y_nhwc) return no("output is neither dense NCHW nor dense NHWC");
    if (!y_nchw && (K % 8 || (uintptr_t)p.y % 16)) return no("NHWC output is stored eight channels at a time");
    if (C % 64) return no("channels must be a multiple of 64");
    if (H * W < 8) return no("images of fewer than eight pixels");
    if ((uintptr_t)p.w % 16 || (uintptr_t)p.x % 2) return no("weights are not 16-byte aligned");
    if ((p.epilogue & ALT_EPI_BIAS) && (uintptr_t)p.bias % 4) return no("bias is not aligned");
    if (pb.x_elems * 2 >= 0x7fffffff || pb.w_elems * 2 >= 0x7fffffff || p.y_bytes == 0 || (int64_t)p.M * K * 4 >= 0x7fffffff)
        return no("operand of 2 GiB or more");
    if (N * H * W > 0x7fffffff) return no("input too large for 32-bit pixel indices");
    const size_t lds = dplanar_lds_bytes(k.BM, k.BN, k.kw, (int)(R * S), (int)C,
                                         dconv_patch_pixels(k.BM, p.M, p.H, p.W, p.OH, p.OW, p.R, p.S, p.pad_h, p.pad_w, st_, p.dil_h));
    if (lds > 160 * 1024) return no("patch and weight stages do not fit LDS");
    const int tiles_m = (p.M + k.BM - 1) / k.BM, tiles_n = (p.Nc + k.BN - 1) / k.BN;
    if ((int64_t)tiles_m * tiles_n > 0x7fffffff) return no("grid too large");
    if (!out) return true;
    DconvParams d;
    std::memset(&d, 0, sizeof d);
    d.x = p.x; d.w = p.w; d.bias = p.bias; d.y = p.y;
    d.x_bytes = p.x_bytes; d.w_bytes = p.w_bytes; d.y_bytes = p.y_bytes;
    d.M = p.M; d.Nc = p.Nc; d.C = p.C; d.Cs = p.C;
    d.H = p.H; d.W = p.W; d.R = p.R; d.S = p.S; d.pad_h = p.pad_h; d.pad_w = p.pad_w;
    d.tiles_m = tiles_m; d.tiles_n = tiles_n; d.splitk = 1;
    d.flags = (p.epilogue & (ALT_EPI_BIAS | ALT_EPI_RELU)) | (p.out_bf16 ? kDconvOutBf16 : 0) | (y_nchw ? 0 : kPlanarOutNhwc);
    d.OH = p.OH; d.OW = p.OW; d.stride = st_; d.dil = p.dil_h;
    d.in_px = (int32_t)(N * H * W);
    d.d_hw = make_div32((uint32_t)(p.OH * p.OW));
    d.d_w = make_div32((uint32_t)p.OW);
    d.d_tm = make_div32((uint32_t)tiles_m);
    d.d_tn = make_div32((uint32_t)tiles_n);
    d.d_ihw = make_div32((uint32_t)(H * W));
    d.d_sk = make_div32(1);
    d.bk = 64;
    *out = d;
    *lds_bytes = lds;
    return true;
}

// Fills the launch parameters of direct kernel `k` for `pb` split into `splitk`
// channel slices, or says why the kernel does not cover the problem.
bool dconv_setup(const Problem &pb, const IgemmLaunch &k, int splitk, DconvParams *out, size_t *lds_bytes, std::string *why)
{
    if (k.stream == 2) return dplanar_setup(pb, k, splitk, out, lds_bytes, why);
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
    int x_blk = 0, y_blk = 0;
    if (!nhwc_or_blocked(p.xc, p.xw, p.xh, p.xn, C, H, W, N, &x_blk)) return no("activations are not dense NHWC or N C/b H W b");
    if (!(dense(p.wi, C, 1) && dense(p.ws, S, C) && dense(p.wr, R, S * C) && dense(p.wo, K, R * S * C)))
        return no("weights are not dense OHWI");
    if (!nhwc_or_blocked(p.yk, p.yw, p.yh, p.yn, K, OH, OW, N, &y_blk)) return no("output is not dense NHWC or N K/b H W b");
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
    d.x_blk = x_blk; d.y_blk = y_blk;
    d.d_ihw = make_div32((uint32_t)(H * W));
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
        DeviceState *ds = device_state();
        int slot = 0;
        e = counter_slot(ds, st, &slot);
        if (e != hipSuccess) return e;
        d.counters = base + (size_t)slot * kDconvMaxTiles;
        d.partial = partial;
    }
    return k.launch_direct(d, lds, st);
}

}  // namespace alt

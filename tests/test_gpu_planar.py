"""GPU parity of the channel-planar direct convolution (NCHW activations, OIHW weights, NCHW
output: the kernels named *_planar_*) against the oracle.  Integer-valued inputs make every
summation order exact, so every tile shape and K-group count must match bit for bit; the
cases put image boundaries, rows of odd length and the ends of the tensors inside the
eight-pixel runs the kernel loads."""
import numpy as np
import pytest

import oracle
import paper_2210_12415_amd as alt
from workloads import RESNET_LAYERS, f32_to_bf16_bits, normal_f32, small_ints_f32

from gpu_util import applicable_variants, err_measures
from test_gpu_conv import run_conv

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def h():
    return alt.Handle()


PLANAR_CASES = [
    dict(N=3, C=128, H=9, W=10, K=96, R=3, S=3, pad=1),              # 90-pixel planes: runs straddle images, ragged M and K
    dict(N=5, C=64, H=7, W=7, K=64, R=3, S=3, pad=1),                # 49-pixel planes: every run address is odd
    dict(N=2, C=64, H=20, W=17, K=64, R=3, S=3, pad=1),              # several tiles per image
    dict(N=2, C=256, H=13, W=6, K=160, R=1, S=1, pad=0),             # 1x1: no halo, four super-steps
    dict(N=9, C=512, H=3, W=3, K=64, R=3, S=3, pad=1),               # nine-pixel planes: a run holds parts of two images
    dict(N=3, C=64, H=12, W=10, K=96, R=3, S=3, pad=1, stride=2),    # stride 2
    dict(N=2, C=128, H=14, W=18, K=64, R=1, S=1, pad=0, stride=2),   # the strided 1x1 of a projection shortcut
    dict(N=3, C=64, H=12, W=11, K=64, R=3, S=3, pad=0),              # no padding: the output is smaller than the input
    dict(N=2, C=64, H=13, W=12, K=64, R=3, S=3, pad=2, dil=2),       # dilated, same-size
    dict(N=1, C=192, H=14, W=14, K=40, R=3, S=3, pad=1),             # three super-steps, K below one tile
]


@pytest.mark.parametrize("yl", ["NCHW", "NHWC"])
@pytest.mark.parametrize("case", PLANAR_CASES, ids=lambda c: "c%d_%dx%d_k%d_%dx%d_s%d_p%d_d%d" % (
    c["C"], c["H"], c["W"], c["K"], c["R"], c["S"], c.get("stride", 1), c["pad"], c.get("dil", 1)))
def test_planar_kernels_exact_integers_every_variant(h, case, yl):
    """(yl = NHWC: the layer converts the layout for an NHWC consumer by itself.)"""
    c = case
    x = small_ints_f32(71, (c["N"], c["C"], c["H"], c["W"]), -3, 3)
    w = small_ints_f32(72, (c["K"], c["C"], c["R"], c["S"]), -3, 3)
    b = small_ints_f32(73, (c["K"],), -50, 50)
    st, dil = c.get("stride", 1), c.get("dil", 1)
    cfg = dict(stride=st, pad=c["pad"], dil=dil)
    ref = oracle.conv2d(x, w, stride=st, pad=c["pad"], dil=dil)
    ref_br = oracle.conv2d(x, w, stride=st, pad=c["pad"], dil=dil, bias=b, relu=True)
    xb, wb = f32_to_bf16_bits(x), f32_to_bf16_bits(w)
    d0 = alt.conv_desc(c["N"], c["C"], c["H"], c["W"], c["K"], c["R"], c["S"], stride=st, pad=c["pad"], dil=dil,
                       in_dtype=alt.BF16, x_layout="NCHW->NCHW", w_layout="OIHW->OIHW", y_layout="NCHW->" + yl)
    variants = [(v, n) for v, n in applicable_variants(h, d0) if "planar" in n]
    assert len(variants) >= 2, "planar kernels should cover this case"
    for v, name in variants:
        print(name, flush=True)
        got, _ = run_conv(h, xb, wb, cfg, "NCHW", "OIHW", yl, alt.BF16, variant=v)
        assert np.array_equal(got, ref), name
        got, _ = run_conv(h, xb, wb, cfg, "NCHW", "OIHW", yl, alt.BF16, bias=b, relu=True, variant=v)
        assert np.array_equal(got, ref_br), name
        got16, _ = run_conv(h, xb, wb, cfg, "NCHW", "OIHW", yl, alt.BF16, out_dtype=alt.BF16, bias=b, relu=True,
                            variant=v)
        assert np.array_equal(got16, f32_to_bf16_bits(ref_br)), name


def test_planar_kernel_is_the_default_for_the_default_layouts(h):
    """Without a tuned entry the library's own choice for NCHW / OIHW / NCHW is a planar kernel."""
    L = RESNET_LAYERS[0]
    d = alt.conv_desc(16, L["C"], L["H"], L["W"], L["K"], L["R"], L["S"], stride=L["stride"], pad=L["pad"],
                      in_dtype=alt.BF16, out_dtype=alt.BF16, x_layout="NCHW->NCHW", w_layout="OIHW->OIHW",
                      y_layout="NCHW->NCHW")
    assert "planar" in h.conv2d_variant_name(d, -1)


@pytest.mark.parametrize("layer", RESNET_LAYERS, ids=lambda L: L["name"])
def test_planar_kernels_on_the_benchmark_layers(h, layer):
    """Batch 2 of each benchmark layer, normal inputs, bf16 output: every planar variant within the bf16 bound."""
    L = layer
    x = f32_to_bf16_bits(normal_f32(81, (2, L["C"], L["H"], L["W"])))
    w = f32_to_bf16_bits(normal_f32(82, (L["K"], L["C"], L["R"], L["S"]), 0.05))
    from workloads import bf16_bits_to_f32
    ref = oracle.conv2d(bf16_bits_to_f32(x), bf16_bits_to_f32(w), stride=L["stride"], pad=L["pad"])
    cfg = dict(stride=L["stride"], pad=L["pad"])
    d0 = alt.conv_desc(2, L["C"], L["H"], L["W"], L["K"], L["R"], L["S"], stride=L["stride"], pad=L["pad"],
                       in_dtype=alt.BF16, x_layout="NCHW->NCHW", w_layout="OIHW->OIHW", y_layout="NCHW->NCHW")
    variants = [(v, n) for v, n in applicable_variants(h, d0) if "planar" in n]
    assert variants
    for v, name in variants:
        print(name, flush=True)
        got, _ = run_conv(h, x, w, cfg, "NCHW", "OIHW", "NCHW", alt.BF16, out_dtype=alt.BF16, variant=v)
        e = err_measures(bf16_bits_to_f32(got), ref)
        assert e["floored"] <= 2e-2, (name, e)


@pytest.mark.parametrize("x_shift,y_shift", [(1, 0), (0, 3), (5, 7)])
def test_planar_kernels_take_buffers_at_any_element_offset(h, x_shift, y_shift):
    """Activations and output that start at an odd element of an allocation (2-byte aligned, nothing more):
    the 16-byte runs the kernel loads and stores are then misaligned everywhere, and must still be exact."""
    import torch
    from gpu_util import dev, host, to_layout, from_layout
    N, C, H, W, K = 3, 64, 14, 14, 64
    x = small_ints_f32(101, (N, C, H, W), -3, 3)
    w = small_ints_f32(102, (K, C, 3, 3), -3, 3)
    ref = f32_to_bf16_bits(oracle.conv2d(x, w, stride=1, pad=1, relu=True))
    d0 = alt.conv_desc(N, C, H, W, K, 3, 3, stride=1, pad=1, in_dtype=alt.BF16, out_dtype=alt.BF16, epilogue=alt.EPI_RELU,
                       x_layout="NCHW->NCHW", w_layout="OIHW->OIHW", y_layout="NCHW->NCHW")
    xb = f32_to_bf16_bits(x).reshape(-1)
    xd_whole = dev(np.concatenate([np.zeros(x_shift, np.uint16), xb, np.zeros(8, np.uint16)]))
    wd = dev(f32_to_bf16_bits(w).reshape(-1))
    n_out = N * K * H * W
    for v, name in [(v, n) for v, n in applicable_variants(h, d0) if "planar" in n]:
        d0.variant = v
        y_whole = torch.full((n_out + y_shift + 64,), 0x5A5A, dtype=torch.int16, device="cuda")
        h.conv2d(d0, xd_whole[x_shift:], wd, y_whole[y_shift:])
        got = host(y_whole, np.uint16)
        assert np.array_equal(got[y_shift:y_shift + n_out].reshape(ref.shape), ref), name
        assert (got[:y_shift] == 0x5A5A).all() and (got[y_shift + n_out:] == 0x5A5A).all(), name

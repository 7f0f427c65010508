"""GPU parity of the register-weights direct convolution (kernels named *_regw_*: 3x3 filters
over 32 or 64 channels into at most 64, workgroups resident on the compute units, each
walking several output tiles) against the oracle.  Integer-valued inputs make every summation
order exact, so the results must match bit for bit; the large cases give every resident
workgroup four to seven tiles (both patch buffers and both accumulator sets reused, odd and
even tile counts, a ragged last tile), the small ones fewer tiles than compute units."""
import numpy as np
import pytest

import oracle
import paper_2210_12415_amd as alt
from workloads import bf16_bits_to_f32, f32_to_bf16_bits, normal_f32, small_ints_f32

from gpu_util import applicable_variants, err_measures
from test_gpu_conv import run_conv

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def h():
    return alt.Handle()


def regw_variants(h, N, C, H, W, K, xl, yl):
    d0 = alt.conv_desc(N, C, H, W, K, 3, 3, stride=1, pad=1, in_dtype=alt.BF16,
                       x_layout="NCHW->" + xl, w_layout="OIHW->OHWI", y_layout="NCHW->" + yl)
    return [(v, n) for v, n in applicable_variants(h, d0) if "_regw_" in n]


REGW_CASES = [
    # (N, C, H, W, K, x layout, y layout)
    (2, 64, 20, 17, 64, "NHWC", "NHWC"),            # a few tiles: one per workgroup, ragged last tile
    (1, 64, 5, 6, 64, "NHWC", "NHWC"),              # less than one tile
    (3, 32, 9, 10, 48, "NHWC", "NHWC"),             # 32 input channels, 48 output channels: a ragged column tile
    (5, 64, 7, 7, 8, "NCHW32c", "NCHW8c"),          # blocked tensors, eight output channels
    (70, 64, 50, 57, 64, "NHWC", "NHWC"),           # 1558.6 tiles: six to seven per workgroup, ragged end
    (40, 32, 60, 61, 48, "NCHW16c", "NCHW16c"),     # 1143.75 tiles, blocked tensors, ragged channels
    (64, 64, 56, 56, 64, "NCHW32c", "NHWC"),        # the benchmark layer at batch 64: whole tiles only
    (3, 64, 56, 56, 64, "NHWC", "NHWC"),            # 73.5 tiles: fewer than compute units, not a multiple of eight
    (11, 64, 56, 56, 64, "NHWC", "NHWC"),           # 269.5 tiles: one or two per workgroup, some workgroups end early
]


@pytest.mark.parametrize("case", REGW_CASES, ids=lambda c: "n%d_c%d_%dx%d_k%d_%s_%s" % c)
def test_regw_kernels_exact_integers(h, case):
    N, C, H, W, K, xl, yl = case
    x = small_ints_f32(131, (N, C, H, W), -3, 3)
    w = small_ints_f32(132, (K, C, 3, 3), -3, 3)
    b = small_ints_f32(133, (K,), -50, 50)
    cfg = dict(stride=1, pad=1)
    ref = oracle.conv2d(x, w, stride=1, pad=1)
    ref_br = oracle.conv2d(x, w, stride=1, pad=1, bias=b, relu=True)
    xb, wb = f32_to_bf16_bits(x), f32_to_bf16_bits(w)
    variants = regw_variants(h, N, C, H, W, K, xl, yl)
    assert len(variants) == 1, "the register-weights kernel should cover this case"
    for v, name in variants:
        print(name, flush=True)
        got, _ = run_conv(h, xb, wb, cfg, xl, "OHWI", yl, alt.BF16, variant=v)
        assert np.array_equal(got, ref), name
        got16, _ = run_conv(h, xb, wb, cfg, xl, "OHWI", yl, alt.BF16, out_dtype=alt.BF16, bias=b, relu=True, variant=v)
        assert np.array_equal(got16, f32_to_bf16_bits(ref_br)), name
        got, _ = run_conv(h, xb, wb, cfg, xl, "OHWI", yl, alt.BF16, bias=b, relu=True, variant=v)
        assert np.array_equal(got, ref_br), name


def test_regw_kernels_normal_inputs_within_the_bf16_bound(h):
    """The benchmark layer at batch 32 with normal inputs, bf16 output: every output against the oracle."""
    N, C, H, W, K = 32, 64, 56, 56, 64
    x = f32_to_bf16_bits(normal_f32(141, (N, C, H, W)))
    w = f32_to_bf16_bits(normal_f32(142, (K, C, 3, 3), 0.05))
    ref = oracle.conv2d(bf16_bits_to_f32(x), bf16_bits_to_f32(w), stride=1, pad=1)
    for v, name in regw_variants(h, N, C, H, W, K, "NHWC", "NHWC"):
        print(name, flush=True)
        got, _ = run_conv(h, x, w, dict(stride=1, pad=1), "NHWC", "OHWI", "NHWC", alt.BF16, out_dtype=alt.BF16, variant=v)
        e = err_measures(bf16_bits_to_f32(got), ref)
        assert e["floored"] <= 2e-2, (name, e)


def test_regw_kernels_leave_other_problems_alone(h):
    """Strides, other filter sizes, wider layers, unpadded and dilated problems are not theirs."""
    for kw in [dict(C=128), dict(K=96), dict(stride=2), dict(pad=0), dict(R=1, S=1, pad=0), dict(pad=2, dil=2)]:
        a = dict(N=2, C=64, H=12, W=12, K=64, R=3, S=3, stride=1, pad=1, dil=1)
        a.update(kw)
        d0 = alt.conv_desc(a["N"], a["C"], a["H"], a["W"], a["K"], a["R"], a["S"], stride=a["stride"], pad=a["pad"],
                           dil=a["dil"], in_dtype=alt.BF16, x_layout="NCHW->NHWC", w_layout="OIHW->OHWI",
                           y_layout="NCHW->NHWC")
        assert not [n for _, n in applicable_variants(h, d0) if "_regw_" in n], kw

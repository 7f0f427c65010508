"""Seeded random sweeps through the C ABI against the oracle: convolutions, products and conversions drawn
from the library's documented range (channel counts from 8 to 512, filters 1x1 to 5x5, strides, dilation,
padding, every named activation / weight / output layout that divides the shape, fp32 and bf16 operands and
outputs, bias and ReLU, ragged GEMM sizes, blocked GEMM operands), each run with the library's own choice of
kernel and with a few kernels picked at random from those that apply.  Integer-valued inputs make every
summation order exact, so every result must match bit for bit."""
import random

import numpy as np
import pytest

import oracle
import paper_2210_12415_amd as alt
from workloads import f32_to_bf16_bits, small_ints_f32

from gpu_util import applicable_variants, canary_dev, canary_ok, dev, host, to_layout
from test_gpu_conv import run_conv
from test_gpu_gemm import run_gemm

pytestmark = pytest.mark.gpu

ACT = ["NCHW", "NHWC", "NCHW8c", "NCHW16c", "NCHW32c"]
WGT = ["OIHW", "OHWI", "OIHW16o16i", "OIHW16i16o"]


def block(name):
    return int(name[4:-1]) if name[4:] else 1


@pytest.fixture(scope="module")
def h():
    return alt.Handle()


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_convolutions(h, seed):
    rng = random.Random(seed)
    for case in range(60):
        C = rng.choice([8, 16, 24, 32, 64, 96, 128, 192, 256, 512])
        K = rng.choice([8, 24, 32, 48, 64, 96, 128, 160, 200])
        R = rng.choice([1, 3, 3, 3, 5])
        st = rng.choice([1, 1, 1, 2])
        dil = rng.choice([1, 1, 1, 2]) if R > 1 else 1
        pad = rng.choice([0, (R - 1) * dil // 2])
        N = rng.choice([1, 2, 3, 5])
        H = rng.randint(max(3, dil * (R - 1) + 1), 24)
        W = rng.randint(max(3, dil * (R - 1) + 1), 24)
        xl = rng.choice([l for l in ACT if C % block(l) == 0])
        wl = rng.choice(WGT if C % 16 == 0 and K % 16 == 0 else WGT[:2])
        yl = rng.choice([l for l in ACT if K % block(l) == 0])
        relu, use_bias = rng.random() < 0.5, rng.random() < 0.5
        idt = rng.choice([alt.BF16, alt.BF16, alt.F32])
        odt = rng.choice([alt.F32, alt.BF16])
        what = (seed, case, N, C, H, W, K, R, st, pad, dil, xl, wl, yl, relu, use_bias, idt, odt)
        x = small_ints_f32(seed * 1000 + case, (N, C, H, W), -3, 3)
        w = small_ints_f32(seed * 1000 + case + 500, (K, C, R, R), -3, 3)
        b = small_ints_f32(7, (K,), -50, 50) if use_bias else None
        ref = oracle.conv2d(x, w, stride=st, pad=pad, dil=dil, bias=b, relu=relu)
        if odt == alt.BF16:
            ref = f32_to_bf16_bits(ref)
        xb, wb = (f32_to_bf16_bits(x), f32_to_bf16_bits(w)) if idt == alt.BF16 else (x, w)
        d0 = alt.conv_desc(N, C, H, W, K, R, R, stride=st, pad=pad, dil=dil, in_dtype=idt, x_layout="NCHW->" + xl,
                           w_layout="OIHW->" + wl, y_layout="NCHW->" + yl)
        variants = applicable_variants(h, d0)
        assert variants, what
        for v, name in [(-1, "the library's choice")] + rng.sample(variants, min(3, len(variants))):
            got, _ = run_conv(h, xb, wb, dict(stride=st, pad=pad, dil=dil), xl, wl, yl, idt, out_dtype=odt, bias=b,
                              relu=relu, variant=v)
            assert np.array_equal(got, ref), (what, name)


@pytest.mark.parametrize("seed", [21, 22])
def test_random_products(h, seed):
    rng = random.Random(seed)
    for case in range(60):
        batch = rng.choice([1, 1, 2, 3])
        M = rng.choice([1, 7, 64, 96, 100, 128, 160, 200, 256, 320, 513])
        N = rng.choice([8, 24, 64, 72, 96, 128, 192, 256, 328])
        K = rng.choice([8, 16, 32, 40, 64, 96, 128, 192, 256, 384, 1024])
        al = rng.choice(["MK", "KM", "MK32m16k"])
        bl = rng.choice(["KN", "NK", "NK32n16k", "KN16k32n"])
        cl = rng.choice(["MN", "NM", "MN16m8n"])
        if cl == "MN16m8n" and (M % 16 or N % 8):
            cl = "MN"
        if al == "MK32m16k" and (M % 32 or K % 16):
            al = "MK"
        if bl == "NK32n16k" and (N % 32 or K % 16):
            bl = "NK"
        if bl == "KN16k32n" and (N % 32 or K % 16):
            bl = "KN"
        idt = rng.choice([alt.BF16, alt.BF16, alt.F32])
        odt = rng.choice([alt.F32, alt.BF16])
        what = (seed, case, batch, M, N, K, al, bl, cl, idt, odt)
        A = small_ints_f32(seed * 1000 + case, (batch, M, K))
        B = small_ints_f32(seed * 1000 + case + 500, (batch, K, N))
        ref = oracle.gemm(A, B)
        if odt == alt.BF16:
            ref = f32_to_bf16_bits(ref)
        Ab, Bb = (f32_to_bf16_bits(A), f32_to_bf16_bits(B)) if idt == alt.BF16 else (A, B)
        d0 = alt.gemm_desc(M, N, K, batch=batch, in_dtype=idt, a_layout="MK->" + al, b_layout="KN->" + bl,
                           c_layout="MN->" + cl)
        variants = applicable_variants(h, d0, "gemm")
        assert variants, what
        for v, name in [(-1, "the library's choice")] + rng.sample(variants, min(4, len(variants))):
            got, _ = run_gemm(h, Ab, Bb, al, bl, cl, idt, out_dtype=odt, variant=v)
            assert np.array_equal(got, ref), (what, name)


@pytest.mark.parametrize("seed", [31])
def test_random_conversions(h, seed):
    rng = random.Random(seed)
    for case in range(200):
        N = rng.choice([1, 2, 3, 7])
        C = rng.choice([16, 32, 64, 96, 160])
        H, W = rng.randint(1, 20), rng.randint(1, 20)
        src = rng.choice([l for l in ACT if C % block(l) == 0])
        dst = rng.choice([l for l in ACT if C % block(l) == 0])
        bf16 = rng.random() < 0.5
        what = (seed, case, N, C, H, W, src, dst, bf16)
        a = small_ints_f32(seed * 1000 + case, (N, C, H, W), -100, 100)
        if bf16:
            a = f32_to_bf16_bits(a)
        flat, ref = to_layout(a, "NCHW", src), to_layout(a, "NCHW", dst)
        whole, out = canary_dev(flat.size, flat.dtype)
        h.layout_transform(alt.BF16 if bf16 else alt.F32, (N, C, H, W), "NCHW->" + src, dev(flat), "NCHW->" + dst, out)
        assert np.array_equal(host(out, flat.dtype), ref), what
        assert canary_ok(whole, flat.size), what

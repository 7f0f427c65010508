"""Pins for the oracle's convolution, matrix product and bf16 rounding:
brute-force loops written here, an independently written im2col product,
closed forms (delta kernel, all-ones), exact-arithmetic properties (linearity,
translation, stride sub-sampling) and library routines as special cases
(numpy matmul, torch's float64 conv2d, torch's bf16 cast).  Expected values
never come from the oracle itself."""
import itertools

import numpy as np
import pytest
import torch

from workloads import (bf16_bits_to_f32, f32_to_bf16_bits, normal_f32, small_ints_f32,
                       uniform_f32)


def _brute_conv(x, w, stride, pad, dil=1):
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    OH = (H + 2 * pad - dil * (R - 1) - 1) // stride + 1
    OW = (W + 2 * pad - dil * (S - 1) - 1) // stride + 1
    y = np.zeros((N, K, OH, OW), dtype=np.float64)
    for n, k, oh, ow in itertools.product(range(N), range(K), range(OH), range(OW)):
        acc = 0.0
        for c, r, s in itertools.product(range(C), range(R), range(S)):
            ih, iw = oh * stride - pad + r * dil, ow * stride - pad + s * dil
            if 0 <= ih < H and 0 <= iw < W:
                acc += float(x[n, c, ih, iw]) * float(w[k, c, r, s])
        y[n, k, oh, ow] = acc
    return y


def _im2col_conv(x, w, stride, pad):
    """Separate formulation: gather patches into a matrix, one matmul."""
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    xp = np.zeros((N, C, H + 2 * pad, W + 2 * pad), dtype=np.float64)
    xp[:, :, pad:pad + H, pad:pad + W] = x
    OH = (H + 2 * pad - R) // stride + 1
    OW = (W + 2 * pad - S) // stride + 1
    cols = np.empty((N, OH, OW, C, R, S), dtype=np.float64)
    for r in range(R):
        for s in range(S):
            cols[:, :, :, :, r, s] = xp[:, :, r:r + stride * OH:stride, s:s + stride * OW:stride].transpose(0, 2, 3, 1)
    out = cols.reshape(N * OH * OW, C * R * S) @ w.reshape(K, C * R * S).astype(np.float64).T
    return out.reshape(N, OH, OW, K).transpose(0, 3, 1, 2)


@pytest.mark.parametrize("stride,pad,dil", [(1, 1, 1), (2, 1, 1), (1, 0, 1), (2, 0, 1), (1, 2, 2), (3, 2, 1)])
def test_conv_brute_force_tiny(oracle, stride, pad, dil):
    x = uniform_f32(1, (2, 3, 6, 7))
    w = uniform_f32(2, (4, 3, 3, 2))
    want = _brute_conv(x, w, stride, pad, dil)
    got = oracle.conv2d(x, w, stride=stride, pad=pad, dil=dil)
    assert got.shape == want.shape
    assert np.array_equal(got, want.astype(np.float32))


@pytest.mark.parametrize("stride,pad", [(1, 1), (2, 1), (1, 0)])
def test_conv_vs_im2col_and_torch(oracle, stride, pad):
    x = normal_f32(3, (2, 5, 9, 8))
    w = normal_f32(4, (6, 5, 3, 3), std=0.05)
    got = oracle.conv2d(x, w, stride=stride, pad=pad).astype(np.float64)
    alt = _im2col_conv(x, w, stride, pad)
    lib = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                     stride=stride, padding=pad).numpy()
    scale = np.abs(lib).max()
    assert np.abs(got - alt).max() <= 2e-7 * scale
    assert np.abs(got - lib).max() <= 2e-7 * scale


def test_conv_small_config_shape(oracle):
    # the N=1, C=16, 14x14, K=16, 3x3 case: output keeps 14x14 with pad 1
    x = uniform_f32(0xA18, (1, 16, 14, 14))
    w = uniform_f32(0xA19, (16, 16, 3, 3))
    y = oracle.conv2d(x, w, stride=1, pad=1)
    assert y.shape == (1, 16, 14, 14)
    assert np.abs(y - _im2col_conv(x, w, 1, 1)).max() < 1e-5


def test_conv_delta_kernel_is_identity(oracle):
    C = 5
    x = uniform_f32(7, (2, C, 6, 6))
    w = np.zeros((C, C, 3, 3), dtype=np.float32)
    for c in range(C):
        w[c, c, 1, 1] = 1.0
    assert np.array_equal(oracle.conv2d(x, w, stride=1, pad=1), x)
    # a delta off centre shifts the image: y[h, w] = x[h-1, w+1], zero outside
    w2 = np.zeros_like(w)
    for c in range(C):
        w2[c, c, 0, 2] = 1.0
    y = oracle.conv2d(x, w2, stride=1, pad=1)
    want = np.zeros_like(x)
    want[:, :, 1:, :-1] = x[:, :, :-1, 1:]
    assert np.array_equal(y, want)


def test_conv_all_ones_counts_taps(oracle):
    C, H, W, R, S, pad = 3, 5, 6, 3, 3, 1
    x = np.ones((1, C, H, W), dtype=np.float32)
    w = np.ones((2, C, R, S), dtype=np.float32)
    y = oracle.conv2d(x, w, stride=1, pad=pad)
    for oh in range(H):
        for ow in range(W):
            rows = sum(0 <= oh - pad + r < H for r in range(R))
            cols = sum(0 <= ow - pad + s < W for s in range(S))
            assert y[0, 0, oh, ow] == C * rows * cols
            assert y[0, 1, oh, ow] == C * rows * cols


def test_conv_linearity_exact(oracle):
    x1 = small_ints_f32(8, (2, 4, 7, 7))
    x2 = small_ints_f32(9, (2, 4, 7, 7))
    w = small_ints_f32(10, (3, 4, 3, 3))
    a = 4.0
    lhs = oracle.conv2d(a * x1 + x2, w, stride=1, pad=1)
    rhs = a * oracle.conv2d(x1, w, stride=1, pad=1) + oracle.conv2d(x2, w, stride=1, pad=1)
    assert np.array_equal(lhs, rhs)


def test_conv_stride2_is_subsampled_stride1(oracle):
    x = small_ints_f32(12, (1, 3, 9, 9))
    w = small_ints_f32(13, (2, 3, 3, 3))
    y1 = oracle.conv2d(x, w, stride=1, pad=1)
    y2 = oracle.conv2d(x, w, stride=2, pad=1)
    assert np.array_equal(y2, y1[:, :, ::2, ::2])


def test_conv_translation(oracle):
    x = small_ints_f32(14, (1, 2, 8, 8))
    w = small_ints_f32(15, (2, 2, 3, 3))
    xs = np.zeros_like(x)
    xs[:, :, :, 1:] = x[:, :, :, :-1]                 # shift right by one pixel
    y, ys = oracle.conv2d(x, w, pad=1), oracle.conv2d(xs, w, pad=1)
    # columns whose windows never see the pixel column that fell off the right edge
    assert np.array_equal(ys[:, :, :, 1:-1], y[:, :, :, :-2])


def test_conv_1x1_is_matrix_product(oracle):
    N, C, H, W, K = 2, 6, 4, 5, 3
    x = small_ints_f32(16, (N, C, H, W))
    w = small_ints_f32(17, (K, C, 1, 1))
    y = oracle.conv2d(x, w)
    A = x.transpose(0, 2, 3, 1).reshape(N * H * W, C)
    want = (A.astype(np.float64) @ w.reshape(K, C).T.astype(np.float64)).reshape(N, H, W, K).transpose(0, 3, 1, 2)
    assert np.array_equal(y, want.astype(np.float32))
    # and the two oracles agree with each other through that identity
    g = oracle.gemm(A, np.ascontiguousarray(w.reshape(K, C).T))
    assert np.array_equal(g.reshape(N, H, W, K).transpose(0, 3, 1, 2), y)


def test_conv_bias_relu_and_bf16(oracle):
    x = f32_to_bf16_bits(normal_f32(18, (2, 8, 6, 6)))
    w = f32_to_bf16_bits(normal_f32(19, (4, 8, 3, 3), std=0.05))
    b = normal_f32(20, (4,), std=0.1)
    xf, wf = bf16_bits_to_f32(x), bf16_bits_to_f32(w)
    ref = torch.nn.functional.conv2d(torch.from_numpy(xf).double(), torch.from_numpy(wf).double(),
                                     torch.from_numpy(b).double(), padding=1).clamp_min(0).numpy()
    y32 = oracle.conv2d(x, w, pad=1, bias=b, relu=True)
    assert np.abs(y32 - ref).max() <= 1e-6 * np.abs(ref).max()
    assert (y32 >= 0).all() and (y32 == 0).any()
    y16 = oracle.conv2d(x, w, pad=1, bias=b, relu=True, out_bf16=True)
    want16 = torch.from_numpy(y32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(y16, want16)


def test_conv_at_matches_full(oracle):
    x = normal_f32(21, (2, 4, 6, 6))
    w = normal_f32(22, (5, 4, 3, 3))
    full = _im2col_conv(x, w, 2, 1)
    flat = np.array([0, 7, 13, full.size - 1, 29])
    got = oracle.conv2d_at(x, w, flat, stride=2, pad=1)
    assert np.allclose(got, full.reshape(-1)[flat], rtol=1e-12, atol=1e-12)


# -------------------------------------------------------------------- gemm ----

def test_gemm_identity_and_permutation(oracle):
    A = uniform_f32(30, (7, 9))
    assert np.array_equal(oracle.gemm(A, np.eye(9, dtype=np.float32)), A)
    perm = np.array([3, 0, 8, 1, 7, 2, 6, 4, 5])
    P = np.zeros((9, 9), dtype=np.float32)
    P[perm, np.arange(9)] = 1.0
    assert np.array_equal(oracle.gemm(A, P), A[:, perm])


def test_gemm_vs_numpy_and_transpose_rule(oracle):
    A = normal_f32(31, (13, 17))
    B = normal_f32(32, (17, 11))
    want = A.astype(np.float64) @ B.astype(np.float64)
    got = oracle.gemm(A, B)
    assert np.array_equal(got, want.astype(np.float32)) or np.abs(got - want).max() < 1e-6
    gt = oracle.gemm(np.ascontiguousarray(B.T), np.ascontiguousarray(A.T))
    assert np.abs(gt.T - got).max() <= 1e-6


def test_gemm_non_square_catches_transposed_operand(oracle):
    A = small_ints_f32(33, (3, 5))
    B = small_ints_f32(34, (5, 4))
    want = np.zeros((3, 4))
    for m, n, k in itertools.product(range(3), range(4), range(5)):
        want[m, n] += A[m, k] * B[k, n]
    assert np.array_equal(oracle.gemm(A, B), want.astype(np.float32))


def test_gemm_batched_is_loop_of_singles(oracle):
    A = normal_f32(35, (4, 6, 8))
    B = normal_f32(36, (4, 8, 5))
    C = oracle.gemm(A, B)
    for b in range(4):
        assert np.array_equal(C[b], oracle.gemm(A[b], B[b]))
        assert np.abs(C[b] - A[b].astype(np.float64) @ B[b].astype(np.float64)).max() < 1e-6


def test_gemm_bf16_inputs_and_at(oracle):
    A = f32_to_bf16_bits(normal_f32(37, (9, 32), std=0.02))
    B = f32_to_bf16_bits(normal_f32(38, (32, 6), std=0.02))
    want = bf16_bits_to_f32(A).astype(np.float64) @ bf16_bits_to_f32(B).astype(np.float64)
    got = oracle.gemm(A, B)
    assert np.array_equal(got, want.astype(np.float32))
    at = oracle.gemm_at(A, B, np.array([0, 5, 53]))
    assert np.allclose(at, want.reshape(-1)[[0, 5, 53]], rtol=1e-13, atol=0)


# -------------------------------------------------------------------- bf16 ----

def test_bf16_rounding_matches_library_cast(oracle):
    v = np.concatenate([normal_f32(40, (4000,)), np.array(
        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-40, -1e-40, np.inf, -np.inf],
        dtype=np.float32)])
    want = torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oracle.f32_to_bf16_bits(v), want)
    assert np.array_equal(f32_to_bf16_bits(v), want)          # the input generator's rounding too
    # ties go to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert oracle.f32_to_bf16_bits(np.array([1.00390625], dtype=np.float32))[0] == 0x3F80
    assert oracle.f32_to_bf16_bits(np.array([1.01171875], dtype=np.float32))[0] == 0x3F82
    nan = oracle.f32_to_bf16_bits(np.array([np.nan], dtype=np.float32))[0]
    assert (nan & 0x7F80) == 0x7F80 and (nan & 0x7F) != 0


def _bf16_exact(bits):
    """bf16 bit pattern -> exact Fraction."""
    from fractions import Fraction
    bits = int(bits)
    sign = -1 if bits >> 15 else 1
    e, m = (bits >> 7) & 0xff, bits & 0x7f
    if e == 0:
        return sign * Fraction(m, 1 << 7) * Fraction(2) ** (-126)
    return sign * (1 + Fraction(m, 1 << 7)) * Fraction(2) ** (e - 127)


def _round_to_bf16_exact(q):
    """Nearest bf16 (ties to even) of an exact rational, by search over the two neighbours."""
    from fractions import Fraction
    if q == 0:
        return 0
    sign = 0x8000 if q < 0 else 0
    a = abs(q)
    lo, hi = 0, 0x7f7f                      # finite positive patterns are ordered like their values
    while hi - lo > 1:
        mid = (lo + hi) // 2
        if _bf16_exact(mid) <= a:
            lo = mid
        else:
            hi = mid
    dl, dh = a - _bf16_exact(lo), _bf16_exact(hi) - a
    pick = lo if dl < dh or (dl == dh and lo % 2 == 0) else hi
    return sign | pick


def test_eltwise_add_bf16_is_one_exact_rounding(oracle):
    """Pin: exact rational arithmetic on every pair of a few hundred patterns that
    include wide exponent gaps, ties, cancellation and subnormals."""
    rng = np.random.RandomState(5)
    pats = set(rng.randint(0x0080, 0x7f00, 40).tolist())
    pats |= {0x0000, 0x8000, 0x0001, 0x007f, 0x0080, 0x3f80, 0x3f81, 0x3fff, 0x4000, 0x3b80, 0x3380, 0x2f80, 0x2b80,
             0x2380, 0x1f80, 0x7f7f, 0x7f00, 0x3f00, 0x3e80}
    pats |= {p | 0x8000 for p in list(pats)[:20]}
    pats = sorted(pats)
    a = np.array([p for p in pats for _ in pats], dtype=np.uint16)
    b = np.array([q for _ in pats for q in pats], dtype=np.uint16)
    got = oracle.eltwise_add(a, b)
    for i in range(a.size):
        q = _bf16_exact(a[i]) + _bf16_exact(b[i])
        if abs(q) >= _bf16_exact(0x7f7f) + (_bf16_exact(0x7f7f) - _bf16_exact(0x7f7e)) / 2:
            continue                         # overflows to infinity
        want = _round_to_bf16_exact(q)
        if q == 0:
            assert got[i] & 0x7fff == 0
        else:
            assert got[i] == want, (hex(a[i]), hex(b[i]), hex(got[i]), hex(want))


def test_eltwise_add_closed_forms(oracle):
    x = uniform_f32(91, (3, 5, 7))
    y = uniform_f32(92, (3, 5, 7))
    z = np.zeros_like(x)
    assert np.array_equal(oracle.eltwise_add(x, z), x)                      # a + 0 = a
    assert np.array_equal(oracle.eltwise_add(x, None), x)
    assert np.array_equal(oracle.eltwise_add(x, y), oracle.eltwise_add(y, x))   # commutative
    assert np.array_equal(oracle.eltwise_add(x, y), (x.astype(np.float64) + y).astype(np.float32))  # one fp32 rounding
    r = oracle.eltwise_add(x, y, relu=True)
    assert (r >= 0).all() and np.array_equal(r, np.maximum(oracle.eltwise_add(x, y), 0))
    assert np.array_equal(oracle.eltwise_add(x, -x), z)                     # exact cancellation
    xb = f32_to_bf16_bits(x)
    assert np.array_equal(oracle.eltwise_add(xb, None), xb)                 # bf16 identity keeps the bits
    nb = f32_to_bf16_bits(-np.abs(x))
    assert (oracle.eltwise_add(nb, None, relu=True) & 0x7fff == 0).all()     # relu of negatives is zero
    # torch's bf16 addition (fp32 add, one rounding) as a library special case
    yb = f32_to_bf16_bits(y)
    t = (torch.from_numpy(bf16_bits_to_f32(xb)).bfloat16() + torch.from_numpy(bf16_bits_to_f32(yb)).bfloat16())
    assert np.array_equal(oracle.eltwise_add(xb, yb), f32_to_bf16_bits(t.float().numpy()))


def test_grouped_conv_is_block_diagonal_dense_conv(oracle):
    """Pins for groups > 1: equal to the dense convolution whose weights are zero outside the
    group blocks, to torch's float64 grouped conv2d (library special case), and, depth-wise,
    to a per-channel brute-force loop."""
    rng = np.random.RandomState(13)
    for (N, C, K, G, R, stride, pad, dil) in [(2, 8, 12, 4, 3, 1, 1, 1), (1, 6, 6, 2, 3, 2, 1, 1), (2, 5, 5, 5, 3, 1, 1, 2),
                                              (1, 4, 8, 4, 1, 1, 0, 1)]:
        x = rng.randint(-3, 4, (N, C, 9, 7)).astype(np.float32)
        w = rng.randint(-3, 4, (K, C // G, R, R)).astype(np.float32)
        b = rng.randint(-5, 6, K).astype(np.float32)
        got = oracle.conv2d(x, w, stride=stride, pad=pad, dil=dil, groups=G, bias=b, relu=True)
        dense = np.zeros((K, C, R, R), dtype=np.float32)
        cg, kg = C // G, K // G
        for g in range(G):
            dense[g * kg:(g + 1) * kg, g * cg:(g + 1) * cg] = w[g * kg:(g + 1) * kg]
        assert np.array_equal(got, oracle.conv2d(x, dense, stride=stride, pad=pad, dil=dil, bias=b, relu=True))
        t = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                       torch.from_numpy(b).double(), stride, pad, dil, G).clamp_min(0)
        assert np.array_equal(got.astype(np.float64), t.numpy())
    # depth-wise against loops written here
    x = rng.randint(-3, 4, (1, 3, 5, 6)).astype(np.float32)
    w = rng.randint(-3, 4, (3, 1, 3, 3)).astype(np.float32)
    got = oracle.conv2d(x, w, stride=1, pad=1, groups=3)
    for c, oh, ow in itertools.product(range(3), range(5), range(6)):
        acc = 0.0
        for r, s in itertools.product(range(3), range(3)):
            ih, iw = oh - 1 + r, ow - 1 + s
            if 0 <= ih < 5 and 0 <= iw < 6:
                acc += float(x[0, c, ih, iw]) * float(w[c, 0, r, s])
        assert got[0, c, oh, ow] == acc
    with pytest.raises(ValueError):
        oracle.conv2d(x, w, groups=2)


def test_conv_unit_height_is_numpy_correlate(oracle):
    """H = R = 1 reduces the C2D to a 1-D cross-correlation per channel pair: numpy's own
    correlate, summed over input channels (integers, so exact), with per-axis stride,
    padding and dilation on the width alone."""
    x = small_ints_f32(71, (2, 3, 1, 23), -4, 4)
    w = small_ints_f32(72, (4, 3, 1, 5), -4, 4)
    for stride, pad, dil in [(1, 0, 1), (2, 3, 1), (1, 4, 2), (3, 2, 2)]:
        got = oracle.conv2d(x, w, stride=(1, stride), pad=(0, pad), dil=(1, dil))
        xp = np.pad(x[:, :, 0, :], ((0, 0), (0, 0), (pad, pad))).astype(np.float64)
        wd = np.zeros((4, 3, (5 - 1) * dil + 1))
        wd[:, :, ::dil] = w[:, :, 0, :]
        ref = np.stack([np.stack([sum(np.correlate(xp[n, c], wd[k, c], "valid") for c in range(3))[::stride]
                                  for k in range(4)]) for n in range(2)])
        assert got.shape == (2, 4, 1, ref.shape[-1])
        assert np.array_equal(got[:, :, 0, :].astype(np.float64), ref), (stride, pad, dil)


@pytest.mark.parametrize("stride,pad,dil", [(1, 0, 1), (1, 1, 1), (2, 1, 1), (2, 0, 1), (3, 2, 2), (2, 2, 2)])
def test_conv_transpose_vs_library_routine(oracle, stride, pad, dil):
    """Against torch's conv_transpose2d in float64 (same weight convention (C, K, R, S))."""
    x = normal_f32(81, (2, 5, 6, 7)).astype(np.float64).astype(np.float32)
    w = normal_f32(82, (5, 3, 3, 4))
    got = oracle.conv2d_transpose(x, w, stride=stride, pad=pad, dil=dil)
    ref = torch.nn.functional.conv_transpose2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                               stride=stride, padding=pad, dilation=dil).numpy()
    assert got.shape == ref.shape == oracle.conv2d_transpose_out_shape(x.shape, w.shape, stride, pad, dil)
    assert np.allclose(got, ref, rtol=1e-6, atol=1e-6)


@pytest.mark.parametrize("stride,pad,dil", [(1, 1, 1), (2, 1, 1), (2, 0, 2), (3, 1, 1)])
def test_conv_transpose_is_the_adjoint_of_conv(oracle, stride, pad, dil):
    """<conv(a, w), b> == <a, conv_transpose(b, w)> for every a, b: with small integers both
    sides are exact.  The filter (K, C, R, S) of the forward C2D is the (in = K, out = C, R, S)
    filter of its adjoint."""
    # input extents that the strided windows cover exactly, so that the adjoint returns a's own shape
    H, W = stride * 4 + dil * 2 + 1 - 2 * pad, stride * 3 + dil * 2 + 1 - 2 * pad
    a = small_ints_f32(91, (2, 4, H, W), -3, 3)
    w = small_ints_f32(92, (6, 4, 3, 3), -3, 3)
    fwd = oracle.conv2d(a, w, stride=stride, pad=pad, dil=dil)
    b = small_ints_f32(93, fwd.shape, -3, 3)
    back = oracle.conv2d_transpose(b, w, stride=stride, pad=pad, dil=dil)
    assert back.shape == a.shape
    lhs = float(np.sum(fwd.astype(np.float64) * b))
    rhs = float(np.sum(a.astype(np.float64) * back))
    assert lhs == rhs


def test_conv_transpose_stride1_is_conv_with_flipped_filter(oracle):
    x = small_ints_f32(95, (2, 3, 7, 6), -4, 4)
    w = small_ints_f32(96, (3, 5, 3, 2), -4, 4)
    got = oracle.conv2d_transpose(x, w, stride=1, pad=0)
    wf = np.ascontiguousarray(w[:, :, ::-1, ::-1].transpose(1, 0, 2, 3))
    ref = oracle.conv2d(x, wf, stride=1, pad=(2, 1))
    assert np.array_equal(got, ref)
    # one input pixel scatters one copy of the filter
    d = np.zeros((1, 1, 4, 4), dtype=np.float32)
    d[0, 0, 1, 2] = 2.0
    k = small_ints_f32(97, (1, 1, 3, 3), -4, 4)
    y = oracle.conv2d_transpose(d, k, stride=2, pad=0)
    assert y.shape == (1, 1, 9, 9)
    exp = np.zeros((9, 9), dtype=np.float32)
    exp[2:5, 4:7] = 2.0 * k[0, 0]
    assert np.array_equal(y[0, 0], exp)


@pytest.mark.parametrize("stride,pad,dil", [((2, 1, 1), (1, 0, 2), (1, 1, 1)), ((1, 2, 1), (2, 1, 0), (2, 1, 2)),
                                            ((1, 1, 2), (0, 2, 1), (1, 3, 1))])
def test_conv3d_with_different_stride_padding_dilation_per_direction(oracle, stride, pad, dil):
    """Each direction takes its own stride, padding and dilation: against torch's conv3d in float64
    (values that differ per direction, so an exchanged pair of directions shows)."""
    x = normal_f32(111, (2, 3, 7, 8, 9))
    w = normal_f32(112, (4, 3, 3, 2, 3))
    got = oracle.conv3d(x, w, stride=stride, pad=pad, dil=dil)
    ref = torch.nn.functional.conv3d(torch.from_numpy(x).double(), torch.from_numpy(w).double(), stride=stride,
                                     padding=pad, dilation=dil).numpy()
    assert got.shape == ref.shape
    assert np.allclose(got, ref, rtol=1e-6, atol=1e-6)


@pytest.mark.parametrize("stride,pad,dil", [(1, 0, 1), (2, 1, 1), ((2, 1, 3), (1, 0, 2), (1, 1, 1)), ((1, 2, 2), (2, 1, 0), (2, 1, 2))])
def test_conv3d_transpose_vs_library_routine_adjoint_and_2d_special_case(oracle, stride, pad, dil):
    """The transposed C3D against torch's conv_transpose3d in float64; as the adjoint of the oracle's own
    C3D (<conv3d(u), v> = <u, conv3d_transpose(v)> for the same filter, in exact integers); and with one
    slice and one depth tap it is the transposed C2D."""
    x = normal_f32(121, (2, 3, 4, 5, 6))
    w = normal_f32(122, (3, 4, 3, 2, 3))
    got = oracle.conv3d_transpose(x, w, stride=stride, pad=pad, dil=dil)
    ref = torch.nn.functional.conv_transpose3d(torch.from_numpy(x).double(), torch.from_numpy(w).double(), stride=stride,
                                               padding=pad, dilation=dil).numpy()
    assert got.shape == ref.shape
    assert np.allclose(got, ref, rtol=1e-6, atol=1e-6)
    # adjoint: v has the shape of x, u the shape of the transposed result when the forward sizes cover it
    v = small_ints_f32(123, (2, 3, 4, 5, 6), -4, 4)
    wi = small_ints_f32(124, (3, 4, 3, 2, 3), -4, 4)
    tv = oracle.conv3d_transpose(v, wi, stride=stride, pad=pad, dil=dil)
    u = small_ints_f32(125, tv.shape, -4, 4)
    fu = oracle.conv3d(u, wi, stride=stride, pad=pad, dil=dil)          # the filter (C,K,..) read as (K'=C, C'=K, ..)
    assert fu.shape == v.shape
    assert float(np.sum(fu.astype(np.float64) * v)) == float(np.sum(u.astype(np.float64) * tv))
    if not isinstance(stride, tuple):
        x1 = small_ints_f32(126, (2, 3, 1, 5, 6), -4, 4)
        w1 = small_ints_f32(127, (3, 4, 1, 2, 3), -4, 4)
        assert np.array_equal(oracle.conv3d_transpose(x1, w1, stride=(1, stride, stride), pad=(0, pad, pad))[:, :, 0],
                              oracle.conv2d_transpose(x1[:, :, 0], w1[:, :, 0], stride=stride, pad=pad))


@pytest.mark.parametrize("stride,pad", [(1, 0), (1, 1), (2, 1), (2, 0)])
def test_conv3d_vs_library_routine_and_2d_special_case(oracle, stride, pad):
    """Against torch's conv3d in float64; with a depth of one tap and one slice it is the C2D."""
    x = normal_f32(101, (2, 3, 6, 7, 5))
    w = normal_f32(102, (4, 3, 3, 2, 3))
    got = oracle.conv3d(x, w, stride=stride, pad=pad)
    ref = torch.nn.functional.conv3d(torch.from_numpy(x).double(), torch.from_numpy(w).double(), stride=stride, padding=pad).numpy()
    assert got.shape == ref.shape
    assert np.allclose(got, ref, rtol=1e-6, atol=1e-6)
    xi = small_ints_f32(103, (2, 3, 1, 7, 5), -4, 4)
    wi = small_ints_f32(104, (4, 3, 1, 3, 3), -4, 4)
    if pad == 0:
        assert np.array_equal(oracle.conv3d(xi, wi, stride=stride, pad=0)[:, :, 0],
                              oracle.conv2d(xi[:, :, 0], wi[:, :, 0], stride=stride, pad=0))

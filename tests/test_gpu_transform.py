"""GPU parity: alt_layout_transform against the oracle's conversion operator,
bit for bit, on small ragged shapes (every kernel path), on the full
benchmark shapes, and on general primitive sequences."""
import numpy as np
import pytest
import torch

import oracle
import paper_2210_12415_amd as alt
from workloads import TRANSFORM_SHAPES, special_bit_patterns

from gpu_util import canary_dev, canary_ok, dev, host

pytestmark = pytest.mark.gpu

NP = {alt.F32: np.uint32, alt.BF16: np.uint16}


@pytest.fixture(scope="module")
def h():
    return alt.Handle()


def _run(h, dtype, shape, src_name, dst_name, seed=1):
    logical = src_name.split("->")[0]
    bits = 32 if dtype == alt.F32 else 16
    data = special_bit_patterns(seed, shape, bits).reshape(-1)       # the physical source buffer
    s_seq = oracle.seq_from_string(src_name, shape)
    d_seq = oracle.seq_from_string(logical + "->" + dst_name.split("->")[1], shape)
    want = oracle.layout_transform(data, shape, s_seq, d_seq)
    src = dev(data)
    whole, dst = canary_dev(data.size, NP[dtype])
    h.layout_transform(dtype, shape, src_name, src, dst_name, dst)
    got = host(dst, NP[dtype])
    assert canary_ok(whole, data.size), "wrote outside the destination"
    assert np.array_equal(got, want), (src_name, dst_name, shape)


PAIRS4 = [("NCHW->NCHW", "NCHW->NHWC"), ("NCHW->NHWC", "NCHW->NCHW"),
          ("NCHW->NCHW", "NCHW->NCHW16c"), ("NCHW->NCHW16c", "NCHW->NCHW"),
          ("NCHW->NCHW", "NCHW->NCHW32c"), ("NCHW->NHWC", "NCHW->NCHW16c"),
          ("NCHW->NCHW16c", "NCHW->NHWC"), ("NCHW->NCHW16c", "NCHW->NCHW32c"),
          ("NCHW->NCHW32c", "NCHW->NCHW8c"), ("NCHW->NCHW", "NCHW->HWNC"),
          ("NCHW->NHWC", "NCHW->NHWC"), ("NCHW->CNHW", "NCHW->NCHW4c")]
SMALL4 = [(2, 32, 5, 7), (3, 64, 14, 14), (1, 32, 1, 1), (2, 96, 7, 7), (1, 32, 9, 40)]


@pytest.mark.parametrize("dtype", [alt.F32, alt.BF16])
@pytest.mark.parametrize("shape", SMALL4)
@pytest.mark.parametrize("pair", PAIRS4)
def test_transform_small(h, dtype, shape, pair):
    _run(h, dtype, shape, pair[0], pair[1])


@pytest.mark.parametrize("dtype", [alt.F32, alt.BF16])
@pytest.mark.parametrize("shape", TRANSFORM_SHAPES)
@pytest.mark.parametrize("pair", [("NCHW->NCHW", "NCHW->NHWC"), ("NCHW->NHWC", "NCHW->NCHW"),
                                  ("NCHW->NCHW", "NCHW->NCHW16c"), ("NCHW->NCHW", "NCHW->NCHW32c")])
def test_transform_benchmark_shapes(h, dtype, shape, pair):
    _run(h, dtype, shape, pair[0], pair[1], seed=7)


@pytest.mark.parametrize("dtype", [alt.F32, alt.BF16])
def test_transform_weights_and_matrices(h, dtype):
    _run(h, dtype, (64, 32, 3, 3), "OIHW->OIHW", "OIHW->OHWI")
    _run(h, dtype, (64, 32, 3, 3), "OIHW->OIHW", "OIHW->OIHW16o16i")
    _run(h, dtype, (64, 32, 3, 3), "OIHW->OIHW", "OIHW->OIHW16i32o")
    _run(h, dtype, (48, 24, 1, 1), "OIHW->OIHW8i4o", "OIHW->OIHW12o8i")      # blocks that do not nest
    _run(h, dtype, (100, 72), "MK->MK", "MK->KM")
    _run(h, dtype, (128, 96), "MK->MK", "MK->MK32m16k")
    _run(h, dtype, (96, 128), "KN->KN", "KN->NK64n32k")
    _run(h, dtype, (7, 13), "MK->MK", "MK->KM")


@pytest.mark.parametrize("dtype", [alt.F32, alt.BF16])
def test_transform_general_sequences(h, dtype):
    """Sequences with a fuse cut across the old dimensions (Section 4.1.1's
    N(O/4)(HW)4 example) go through the per-element kernel."""
    N, H, W, O = 2, 3, 5, 8
    shape = (N, H, W, O)
    bits = 32 if dtype == alt.F32 else 16
    data = special_bit_patterns(3, shape, bits).reshape(-1)
    oseq = [oracle.fuse(1, 3), oracle.split(1, [O // 4, 4, H * W]), oracle.reorder([0, 1, 3, 2])]
    L = alt.layout_from_prims(shape, [alt.fuse(1, 3), alt.split(1, [O // 4, 4, H * W]), alt.reorder([0, 1, 3, 2])])
    plain = alt.layout_parse("NHWO->NHWO")
    want = oracle.layout_transform(data, shape, [], oseq)
    dst = torch.empty_like(dev(data))
    h.layout_transform(dtype, shape, plain, dev(data), L, dst)
    assert np.array_equal(host(dst, NP[dtype]), want)
    back = torch.empty_like(dst)
    h.layout_transform(dtype, shape, L, dst, plain, back)
    assert np.array_equal(host(back, NP[dtype]), data)


def test_transform_round_trip_and_composition(h):
    shape = (4, 64, 14, 14)
    data = special_bit_patterns(5, shape, 16).reshape(-1)
    a, b, c = dev(data), torch.empty_like(dev(data)), torch.empty_like(dev(data))
    d = torch.empty_like(a)
    h.layout_transform(alt.BF16, shape, "NCHW->NCHW", a, "NCHW->NHWC", b)
    h.layout_transform(alt.BF16, shape, "NCHW->NHWC", b, "NCHW->NCHW16c", c)
    h.layout_transform(alt.BF16, shape, "NCHW->NCHW", a, "NCHW->NCHW16c", d)
    assert torch.equal(c, d)
    h.layout_transform(alt.BF16, shape, "NCHW->NCHW16c", c, "NCHW->NCHW", b)
    assert np.array_equal(host(b, np.uint16), data)


def test_transform_errors(h):
    a = torch.zeros(64, dtype=torch.float32, device="cuda")
    b = torch.zeros(64, dtype=torch.float32, device="cuda")
    with pytest.raises(alt.AltError) as e:
        h.layout_transform(alt.F32, (1, 24, 1, 1), "NCHW->NCHW", a, "NCHW->NCHW16c", b)
    assert e.value.status == 3
    with pytest.raises(alt.AltError) as e:
        h.layout_transform(alt.F32, (2, 4, 2, 4), "NCHW->NCHW", a, "NCHW->NHWC", a)
    assert e.value.status == 1
    with pytest.raises(alt.AltError) as e:
        h.layout_transform(7, (2, 4, 2, 4), "NCHW->NCHW", a, "NCHW->NHWC", b)
    assert e.value.status == 1


@pytest.mark.parametrize("case", [((3, 12, 8), 1, 4, 2), ((2, 3, 10), 2, 6, 4), ((9, 5), 0, 3, 3), ((2, 11, 3), 1, 4, 3),
                                  ((4, 6), 1, 8, 2), ((2, 8, 20, 24), 2, 6, 4), ((2, 8, 20, 24), 3, 10, 8)],
                         ids=lambda c: "x".join(map(str, c[0])) + "_d%d_B%d_S%d" % c[1:])
@pytest.mark.parametrize("dtype", [alt.BF16, alt.F32])
def test_unfold_bit_exact(h, case, dtype):
    """The unfold primitive on the device against the oracle's: tiles overlap by B - S, the
    ragged last tile is zero-filled, nothing is written past the output."""
    shape, dim, B, S = case
    numel = int(np.prod(shape))
    ids = np.arange(1, numel + 1, dtype=np.int64).reshape(shape)        # distinct, non-zero, exact in float64
    want = oracle.unfold(ids, dim, B, S).astype(np.int64)
    oshape = alt.unfold_shape(shape, dim, B, S)
    assert tuple(want.shape) == oshape
    npdt = np.uint16 if dtype == alt.BF16 else np.uint32
    src = special_bit_patterns(31, shape, 16 if dtype == alt.BF16 else 32)   # NaN payloads, -0, denormals, random bits
    expect = np.where(want > 0, src.reshape(-1)[np.maximum(want, 1) - 1], 0).astype(npdt)
    n_out = int(np.prod(oshape))
    whole, dst = canary_dev(n_out, npdt)
    h.unfold(dtype, shape, dim, B, S, dev(src.reshape(-1)), dst)
    got = host(dst, npdt)[:n_out].reshape(oshape)
    assert np.array_equal(got, expect)
    assert canary_ok(whole, n_out)
    # Eq. 1 of the paper on the data: element V*i + r of the dimension is at (tile, within)
    if (shape[dim] - B) % S == 0 and B >= 3:
        M, V = 3, 1
        per_tile = (B - M) // V + 1
        if S == V * per_tile:
            line = np.moveaxis(src, dim, -1).reshape(-1, shape[dim])[0]
            unf = np.moveaxis(np.moveaxis(got, dim + 1, -1), dim, -2).reshape(-1, oshape[dim], B)[0]
            for i in range((shape[dim] - M) // V + 1):
                for r in range(M):
                    t, w = oracle.unfold_access(V, i, r, B, S, M)
                    assert unf[t][w] == line[V * i + r]


def test_unfold_rejects_bad_arguments(h):
    a = torch.zeros(64, dtype=torch.float32, device="cuda")
    b = torch.zeros(256, dtype=torch.float32, device="cuda")
    for shape, dim, B, S in [((4, 4), 2, 2, 1), ((4, 4), 0, 0, 1), ((4, 4), 0, 2, 0)]:
        with pytest.raises(alt.AltError) as e:
            h.unfold(alt.F32, shape, dim, B, S, a, b)
        assert e.value.status == 1
    with pytest.raises(alt.AltError) as e:
        h.unfold(alt.F32, (4, 4), 0, 2, 1, a, a)                         # overlapping buffers
    assert e.value.status == 1


def test_transform_of_more_than_2_to_the_31_elements(h):
    """Maximum sizes: a bf16 tensor of 2.2e9 elements (4.4 GB, offsets beyond 32 bits) from NCHW to NHWC.
    Every element of dst must be the element of src with the same logical index; checked on the
    first and last 4096 elements of dst and on four million sampled indices, offsets from the
    closed forms of the two layouts (the source holds a hash of its own offset)."""
    N, C, H, W = 33, 64, 1024, 1024
    numel = N * C * H * W
    assert numel > 2 ** 31
    def pattern(off):                                   # int64 offsets -> int16 values
        return (((off * 2654435761) >> 13) & 0xFFFF).to(torch.int16)
    src = torch.empty(numel, dtype=torch.int16, device="cuda")
    step = 1 << 27
    for a in range(0, numel, step):
        b = min(numel, a + step)
        src[a:b] = pattern(torch.arange(a, b, dtype=torch.int64, device="cuda"))
    dst = torch.full((numel + 128,), 0x5A5A, dtype=torch.int16, device="cuda")
    h.layout_transform(alt.BF16, (N, C, H, W), "NCHW->NCHW", src, "NCHW->NHWC", dst[64:64 + numel])
    torch.cuda.synchronize()
    assert bool((dst[:64] == 0x5A5A).all()) and bool((dst[64 + numel:] == 0x5A5A).all()), "wrote outside dst"
    out = dst[64:64 + numel]
    def src_off_of_dst(o):                              # NHWC offset -> NCHW offset of the same logical index
        c = o % C; r = o // C
        w = r % W; r = r // W
        hh = r % H; n = r // H
        return ((n * C + c) * H + hh) * W + w
    gen = torch.Generator(device="cuda").manual_seed(77)
    sample = torch.randint(0, numel, (1 << 22,), dtype=torch.int64, device="cuda", generator=gen)
    edges = torch.cat([torch.arange(0, 4096, dtype=torch.int64, device="cuda"),
                       torch.arange(numel - 4096, numel, dtype=torch.int64, device="cuda"),
                       torch.arange(2 ** 31 - 2048, 2 ** 31 + 2048, dtype=torch.int64, device="cuda")])
    for o in (edges, sample):
        assert torch.equal(out[o], pattern(src_off_of_dst(o)))



@pytest.mark.parametrize("dtype", [alt.F32, alt.BF16])
@pytest.mark.parametrize("case", [
    ((3, 60, 7, 5), "NCHW->NCHW", (3, 64, 7, 5), "NCHW->NCHW16c"),      # channels padded to the next block
    ((3, 60, 7, 5), "NCHW->NHWC", (3, 64, 9, 5), "NCHW->NCHW32c"),      # channels and height, blocked destination
    ((2, 64, 6, 7), "NCHW->NCHW16c", (2, 50, 6, 7), "NCHW->NHWC"),      # unpad
    ((4, 10, 3, 3), "NCHW->NCHW", (2, 16, 3, 5), "NCHW->NCHW8c"),       # one extent shrinks, others grow
], ids=["pad_c", "pad_ch", "unpad_c", "mixed"])
def test_pad_transform_bit_exact(h, dtype, case):
    """alt_layout_transform_pad against the oracle's pad transform: NaN payloads, -0 and denormals move
    unchanged, everything outside the source is all-bits-zero, nothing outside the destination is touched."""
    src_shape, src_name, dst_shape, dst_name = case
    bits = 32 if dtype == alt.F32 else 16
    data = special_bit_patterns(17, src_shape, bits).reshape(-1)
    s_seq = oracle.seq_from_string(src_name, src_shape)
    d_seq = oracle.seq_from_string(dst_name, dst_shape)
    want = oracle.pad_transform(data, src_shape, s_seq, dst_shape, d_seq)
    src = dev(data)
    n_out = int(np.prod(dst_shape))
    for shift in (0, 1):                                   # destination at an aligned and at an odd element offset
        whole, dst = canary_dev(n_out, NP[dtype], pad=64 + shift)
        h.layout_transform_pad(dtype, src_shape, src_name, src, dst_shape, dst_name, dst)
        got = host(dst, NP[dtype])
        assert canary_ok(whole, n_out, pad=64 + shift), "wrote outside the destination"
        assert np.array_equal(got, want), (case, shift)


def test_convolution_over_padded_channels_equals_the_unpadded_one(h):
    """C = 60 does not divide into blocks of 16: padded to 64 (activations and weights) the blocked layouts
    apply, and the zeros add nothing: the result equals the oracle's convolution of the unpadded tensors."""
    from workloads import small_ints_f32, f32_to_bf16_bits
    from gpu_util import from_layout
    N, C, Cp, H, W, K = 2, 60, 64, 9, 8, 32
    x = small_ints_f32(301, (N, C, H, W), -3, 3)
    w = small_ints_f32(302, (K, C, 3, 3), -3, 3)
    ref = oracle.conv2d(x, w, stride=1, pad=1)
    xd, wd = dev(f32_to_bf16_bits(x).reshape(-1)), dev(f32_to_bf16_bits(w).reshape(-1))
    xp = torch.empty(N * Cp * H * W, dtype=torch.int16, device="cuda")
    wp = torch.empty(K * Cp * 9, dtype=torch.int16, device="cuda")
    h.layout_transform_pad(alt.BF16, (N, C, H, W), "NCHW->NCHW", xd, (N, Cp, H, W), "NCHW->NCHW16c", xp)
    h.layout_transform_pad(alt.BF16, (K, C, 3, 3), "OIHW->OIHW", wd, (K, Cp, 3, 3), "OIHW->OIHW16o16i", wp)
    d = alt.conv_desc(N, Cp, H, W, K, 3, 3, stride=1, pad=1, in_dtype=alt.BF16, out_dtype=alt.F32,
                      x_layout="NCHW->NCHW16c", w_layout="OIHW->OIHW16o16i", y_layout="NCHW->NCHW16c")
    y = torch.empty(N * K * H * W, dtype=torch.float32, device="cuda")
    ws = torch.empty(1 << 22, dtype=torch.uint8, device="cuda")
    h.conv2d(d, xp, wp, y, workspace=ws, ws_bytes=ws.numel())
    got = from_layout(host(y, np.float32), (N, K, H, W), "NCHW", "NCHW16c")
    assert np.array_equal(got, ref)

"""Pins for the oracle's layout algebra and conversion operator: the paper's
printed examples, closed forms written independently here, bijection and
inverse properties, and numpy's reshape/transpose as the library special case.
None of these call the oracle to produce their expected values."""
import itertools
import json
import os

import numpy as np
import pytest

from workloads import special_bit_patterns, uniform_f32

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_examples.json")))


def _ev(expr, env):
    return expr if isinstance(expr, int) else eval(expr, {}, env)


def test_paper_blocked_channel_sequence(oracle):
    g = GOLD["blocked_channel_sequence"]
    N, O, H, W, ot = 2, 32, 3, 5, 16
    env = dict(N=N, O=O, H=H, W=W, o_t=ot)
    seq = oracle.paper_seq([(p[0], p[1], [_ev(f, env) for f in p[2]]) if p[0] == "split"
                            else (p[0], p[1]) for p in g["seq"]])
    shape = (N, O, H, W)
    assert oracle.layout_shape(shape, seq) == tuple(_ev(s, env) for s in g["result_shape"])
    offs = oracle.layout_offsets(shape, seq)
    for n, o, h, w in itertools.product(range(N), range(O), range(H), range(W)):
        closed = (((n * (O // ot) + o // ot) * H + h) * W + w) * ot + o % ot
        assert offs[n, o, h, w] == closed
    # the same thing through numpy: position of each element after reshape+transpose
    iota = np.arange(N * O * H * W).reshape(N, O // ot, ot, H, W).transpose(0, 1, 3, 4, 2).reshape(-1)
    inv = np.empty_like(iota)
    inv[iota] = np.arange(iota.size)
    assert np.array_equal(offs.reshape(-1), inv)
    # and the string form names the same layout
    assert oracle.seq_from_string("NCHW->NCHW16c", shape) == seq


def test_paper_spatial_pack_sequence(oracle):
    g = GOLD["spatial_pack_sequence"]
    N, H, W, O = 2, 3, 5, 8
    env = dict(N=N, H=H, W=W, O=O)
    raw = []
    for p in g["seq"]:
        if p[0] == "split":
            raw.append(("split", p[1], [_ev(f, env) for f in p[2]]))
        else:
            raw.append((p[0], p[1]))
    seq = oracle.paper_seq(raw)
    shape = (N, H, W, O)
    for step in range(3):
        assert oracle.layout_shape(shape, seq[:step + 1]) == tuple(_ev(s, env) for s in g["shapes"][step])
    for n, h, w, o in itertools.product(range(N), range(H), range(W), range(O)):
        e = h * (W * O) + w * O + o
        assert oracle.layout_index(shape, seq[:1], (n, h, w, o))[0] == (n, e)
        assert oracle.layout_index(shape, seq[:2], (n, h, w, o))[0] == \
            (n, e // (H * W * 4), (e // (H * W)) % 4, e % (H * W))
        assert oracle.layout_index(shape, seq, (n, h, w, o))[0] == \
            (n, e // (H * W * 4), e % (H * W), (e // (H * W)) % 4)


def test_split_factors_of_actor_example(oracle):
    g = GOLD["split_actor_example"]
    seq = [oracle.split(0, g["factors"])]
    assert oracle.layout_shape((g["O"],), seq) == (g["O"] // g["o_t"], g["o_t"])
    for o in range(g["O"]):
        assert oracle.layout_index((g["O"],), seq, (o,))[0] == (o // g["o_t"], o % g["o_t"])


def test_overlapped_conv_output_shape(oracle):
    N, O, H, W, ot = 2, 32, 8, 12, 8
    env = dict(N=N, O=O, H=H, W=W, o_t=ot)
    # NOHW: split O, H, W, then reorder to N 2 2 (O/o_t) (H/2) (W/2) o_t
    seq = [oracle.split(1, [O // ot, ot]), oracle.split(3, [2, H // 2]), oracle.split(5, [2, W // 2]),
           oracle.reorder([0, 3, 5, 1, 4, 6, 2])]
    want = tuple(_ev(s, env) for s in GOLD["overlapped_conv_shape"]["shape"])
    assert oracle.layout_shape((N, O, H, W), seq) == want
    idx, _ = oracle.layout_index((N, O, H, W), seq, (1, 19, 5, 7))
    assert idx == (1, 5 // 4, 7 // 6, 19 // 8, 5 % 4, 7 % 6, 19 % 8)


def test_three_way_split_matches_table1(oracle):
    # i -> (i / (F2 F3), (i / F3) mod F2, i mod F3)
    F = [3, 4, 5]
    seq = [oracle.split(1, F)]
    for i in range(60):
        idx, off = oracle.layout_index((2, 60), seq, (1, i))
        assert idx == (1, i // 20, (i // 5) % 4, i % 5)
        assert off == 60 + i          # a split alone never moves data


def test_bijection_and_inverses(oracle):
    shape = (2, 12, 3, 4)
    seqs = [
        [],
        oracle.seq_from_string("NCHW->NHWC", shape),
        oracle.seq_from_string("NCHW->NCHW4c", shape),
        oracle.seq_from_string("NCHW->HWNC", shape),
        [oracle.fuse(1, 3), oracle.split(1, [4, 3, 12]), oracle.reorder([0, 2, 3, 1])],
    ]
    n = int(np.prod(shape))
    for seq in seqs:
        offs = oracle.layout_offsets(shape, seq).reshape(-1)
        assert np.array_equal(np.sort(offs), np.arange(n))
    # split then fuse of the same dims is the identity map
    ident = oracle.layout_offsets(shape, [oracle.split(1, [3, 4]), oracle.fuse(1, 2)])
    assert np.array_equal(ident.reshape(-1), np.arange(n))
    # reorder p then its inverse is the identity map
    p = [2, 0, 3, 1]
    pinv = [p.index(i) for i in range(4)]
    ident = oracle.layout_offsets(shape, [oracle.reorder(p), oracle.reorder(pinv)])
    assert np.array_equal(ident.reshape(-1), np.arange(n))


def test_blocked_degenerate_cases(oracle):
    shape = (2, 8, 3, 5)
    nhwc = oracle.layout_offsets(shape, oracle.seq_from_string("NCHW->NHWC", shape))
    full = oracle.layout_offsets(shape, oracle.seq_from_string("NCHW->NCHW8c", shape))
    one = oracle.layout_offsets(shape, oracle.seq_from_string("NCHW->NCHW1c", shape))
    assert np.array_equal(nhwc, full)
    assert np.array_equal(one.reshape(-1), np.arange(one.size))


def test_weight_and_gemm_templates(oracle):
    # Ker: (O/o')(I/i') KH KW i' o'   (Section 5.1)
    K, C, R, S, it, ot = 8, 6, 3, 2, 3, 4
    shape = (K, C, R, S)
    offs = oracle.layout_offsets(shape, oracle.seq_from_string("OIHW->OIHW3i4o", shape))
    assert oracle.layout_shape(shape, oracle.seq_from_string("OIHW->OIHW3i4o", shape)) == \
        (K // ot, C // it, R, S, it, ot)
    for k, c, r, s in itertools.product(range(K), range(C), range(R), range(S)):
        closed = ((((k // ot) * (C // it) + c // it) * R + r) * S + s) * it * ot + (c % it) * ot + k % ot
        assert offs[k, c, r, s] == closed
    # A: (M/m_t)(K/k_t) m_t k_t
    M, Kd, mt, kt = 6, 8, 3, 4
    offs = oracle.layout_offsets((M, Kd), oracle.seq_from_string("MK->MK3m4k", (M, Kd)))
    for m, k in itertools.product(range(M), range(Kd)):
        assert offs[m, k] == (((m // mt) * (Kd // kt) + k // kt) * mt + m % mt) * kt + k % kt


def test_malformed_sequences_are_rejected(oracle):
    with pytest.raises(ValueError):
        oracle.layout_shape((2, 10), [oracle.split(1, [3, 4])])       # product != extent
    with pytest.raises(ValueError):
        oracle.layout_shape((2, 10), [oracle.reorder([0, 0])])        # not a permutation
    with pytest.raises(ValueError):
        oracle.layout_shape((2, 10), [oracle.fuse(1, 2)])             # runs past the rank


# ------------------------------------------------------------------ unfold ----

def test_unfold_paper_example(oracle):
    g = GOLD["unfold_example"]
    got = oracle.unfold_1d(g["array"], g["B"], g["S"])
    assert got.tolist() == [[float(v) for v in row] for row in g["result"]]
    assert oracle.unfold_tiles(5, 3, 2) == 2


def test_unfold_sizes_and_overlap(oracle):
    for H, KH in [(8, 3), (56, 3), (14, 7), (6, 1)]:
        B, S = H // 2 + (KH - 1), H // 2
        D = H + KH - 1                     # stride-1 input extent
        assert oracle.unfold_tiles(D, B, S) == 2
        assert B - S == KH - 1             # rows shared by neighbouring tiles
    for D, B, S in [(10, 4, 3), (11, 4, 3), (7, 7, 5), (9, 2, 2)]:
        assert oracle.unfold_tiles(D, B, S) == -(-(D - B) // S) + 1


def test_unfold_access_rewrite(oracle):
    # special case of Eq. 1 quoted with the C2D template: V=1, B=h_t+KH-1, M=KH, S=h_t
    for ht, KH in [(4, 3), (7, 1), (2, 5)]:
        for i in range(3 * ht):
            for r in range(KH):
                assert oracle.unfold_access(1, i, r, ht + KH - 1, ht, KH) == (i // ht, i % ht + r)
    # general case against the data: unfolded[tile][within] is the element V*i + r
    for V, M, per in [(1, 3, 4), (2, 3, 3), (2, 7, 5), (3, 1, 2)]:
        B = V * (per - 1) + M
        S = V * per
        nwin = 3 * per
        D = V * (nwin - 1) + M
        src = np.arange(100, 100 + D, dtype=np.float64)
        unf = oracle.unfold_1d(src, B, S)
        for i in range(nwin):
            for r in range(M):
                t, w = oracle.unfold_access(V, i, r, B, S, M)
                assert unf[t, w] == src[V * i + r]


# ------------------------------------------------------ conversion operator ----

@pytest.mark.parametrize("bits", [16, 32])
def test_transform_equals_numpy_transpose(oracle, bits):
    N, C, H, W = 3, 16, 5, 7
    shape = (N, C, H, W)
    src = special_bit_patterns(11, shape, bits)
    nchw = []
    nhwc = oracle.seq_from_string("NCHW->NHWC", shape)
    c8 = oracle.seq_from_string("NCHW->NCHW8c", shape)
    got = oracle.layout_transform(src, shape, nchw, nhwc)
    assert np.array_equal(got, src.transpose(0, 2, 3, 1).reshape(-1))
    got8 = oracle.layout_transform(src, shape, nchw, c8)
    assert np.array_equal(got8, src.reshape(N, C // 8, 8, H, W).transpose(0, 1, 3, 4, 2).reshape(-1))
    # round trip is the identity, bit for bit (NaN payloads, -0, denormals included)
    back = oracle.layout_transform(got, shape, nhwc, nchw)
    assert np.array_equal(back, src.reshape(-1))
    # composition: NCHW -> NHWC -> NCHW8c equals NCHW -> NCHW8c
    assert np.array_equal(oracle.layout_transform(got, shape, nhwc, c8), got8)


def test_transform_of_iota_lists_source_offsets(oracle):
    shape = (2, 8, 3, 5)
    a = oracle.seq_from_string("NCHW->NHWC", shape)
    b = oracle.seq_from_string("NCHW->NCHW4c", shape)
    iota = np.arange(int(np.prod(shape)), dtype=np.uint32)
    dst = oracle.layout_transform(iota, shape, a, b)
    offa = oracle.layout_offsets(shape, a).reshape(-1)
    offb = oracle.layout_offsets(shape, b).reshape(-1)
    want = np.empty_like(iota)
    want[offb] = offa
    assert np.array_equal(dst, want)


def test_transform_gemm_operand_is_matrix_transpose(oracle):
    A = uniform_f32(5, (6, 10))
    got = oracle.layout_transform(A, (6, 10), [], oracle.seq_from_string("MK->KM", (6, 10)))
    assert np.array_equal(got.reshape(10, 6), A.T)


@pytest.mark.parametrize("bits", [16, 32])
def test_pad_transform_against_an_index_loop_and_its_inverse(oracle, bits):
    """pad (Section 4.1.2) carried by the conversion operator: against a per-element loop written out
    here (channel-blocked destination, closed-form offset), zeros exactly where the index leaves the
    source, unpad as the inverse bit for bit, and the plain conversion when the shapes agree."""
    N, C, H, W, x = 2, 5, 3, 4, 8
    src_shape, dst_shape = (N, C, H, W), (N, 8, H, W + 2)       # channels padded to one block of 8, width by 2
    src = special_bit_patterns(21, src_shape, bits)
    nhwc = oracle.seq_from_string("NCHW->NHWC", src_shape)
    c8 = oracle.seq_from_string("NCHW->NCHW8c", dst_shape)
    stored = oracle.layout_transform(src, src_shape, [], nhwc)
    got = oracle.pad_transform(stored, src_shape, nhwc, dst_shape, c8)
    want = np.zeros(int(np.prod(dst_shape)), dtype=src.dtype)
    Wp = W + 2
    for n in range(N):
        for c in range(C):
            for h in range(H):
                for w in range(W):
                    want[(((n * 1 + c // x) * H + h) * Wp + w) * x + c % x] = src[n, c, h, w]
    assert np.array_equal(got, want)
    assert np.count_nonzero(got) <= src.size                    # everything else is all-bits-zero
    back = oracle.pad_transform(got, dst_shape, c8, src_shape, nhwc)
    assert np.array_equal(back, stored)
    same = oracle.pad_transform(stored, src_shape, nhwc, src_shape, oracle.seq_from_string("NCHW->NCHW", src_shape))
    assert np.array_equal(same, src.reshape(-1))


def test_unfold_nd_against_sliding_windows(oracle):
    """N-D unfold against numpy's sliding windows (written independently of the oracle):
    tile t of a dimension is the window starting at t*S; the ragged last tile is zero-filled."""
    rng = np.random.RandomState(11)
    for shape, dim, B, S in [((3, 12, 4), 1, 4, 2), ((2, 3, 10), 2, 6, 4), ((9, 5), 0, 3, 3), ((2, 11, 3), 1, 4, 3),
                             ((4, 6), 1, 8, 2)]:
        x = rng.randint(-1000, 1000, shape).astype(np.float64)
        got = oracle.unfold(x, dim, B, S)
        D = shape[dim]
        T = 1 if D <= B else -(-(D - B) // S) + 1
        padded = np.concatenate([x, np.zeros(shape[:dim] + ((T - 1) * S + B - D,) + shape[dim + 1:])], axis=dim) \
            if (T - 1) * S + B > D else x
        win = np.lib.stride_tricks.sliding_window_view(padded, B, axis=dim)      # window axis goes last
        win = np.take(win, np.arange(T) * S, axis=dim)
        want = np.moveaxis(win, -1, dim + 1)
        assert got.shape == shape[:dim] + (T, B) + shape[dim + 1:]
        assert np.array_equal(got, want)

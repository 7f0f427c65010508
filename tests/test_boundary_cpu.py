"""Host-only checks of the C-ABI library: it loads, exports every symbol the
header declares, its layout index math agrees with the oracle bit for bit, its
chain planner finds known shortest paths, and argument errors come back as
status codes.  No kernel is launched."""
import itertools
import os
import re

import numpy as np
import pytest

import paper_2210_12415_amd as alt
from workloads import small_ints_f32

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "alt.h")).read()
    declared = set(re.findall(r"\b(alt_[a-z0-9_]+)\s*\(", header))
    declared -= {"alt_context"}
    lib = alt.lib()
    for name in sorted(declared):
        assert hasattr(lib, name), name
    assert declared == set(alt.exported_symbols())
    assert alt.version() == "0.1"


LAYOUTS = [("NCHW->NCHW", (2, 8, 3, 5)), ("NCHW->NHWC", (2, 8, 3, 5)), ("NCHW->NCHW4c", (2, 8, 3, 5)),
           ("NCHW->HWNC", (2, 8, 3, 5)), ("NCHW->NCHW2c4c", (1, 16, 2, 3)), ("OIHW->OIHW4i2o", (4, 8, 3, 3)),
           ("OIHW->OIHW2o4i", (4, 8, 3, 3)), ("OIHW->OHWI", (4, 8, 3, 3)), ("MK->KM", (6, 10)),
           ("MK->MK3m5k", (6, 10)), ("KN->NK2n5k", (10, 6))]


@pytest.mark.parametrize("name,shape", LAYOUTS)
def test_layout_offsets_match_oracle(oracle, name, shape):
    L = alt.layout_parse(name)
    if name == "NCHW->NCHW2c4c":
        seq = [oracle.split(1, [shape[1] // 8, 2, 4]), oracle.reorder([0, 1, 4, 5, 2, 3])]
    else:
        seq = oracle.seq_from_string(name, shape)
    want = oracle.layout_offsets(shape, seq)
    assert alt.layout_physical_shape(L, shape) == oracle.layout_shape(shape, seq)
    for idx in itertools.product(*map(range, shape)):
        off = alt.layout_offset(L, shape, idx)
        assert off == want[idx]
        assert alt.layout_index_of(L, shape, off) == idx


def test_layout_from_primitive_sequences(oracle):
    # the paper's two worked sequences (Section 4.1.1), 0-based
    N, O, H, W, ot = 2, 32, 3, 5, 16
    L = alt.layout_from_prims((N, O, H, W), [alt.split(1, [O // ot, ot]), alt.reorder([0, 1, 3, 4, 2])])
    assert L.separable == 1
    want = oracle.layout_offsets((N, O, H, W), oracle.seq_from_string("NCHW->NCHW16c", (N, O, H, W)))
    for idx in itertools.product(range(N), range(O), range(H), range(W)):
        assert alt.layout_offset(L, (N, O, H, W), idx) == want[idx]
    N, H, W, O = 2, 3, 5, 8
    shape = (N, H, W, O)
    L2 = alt.layout_from_prims(shape, [alt.fuse(1, 3), alt.split(1, [O // 4, 4, H * W]), alt.reorder([0, 1, 3, 2])])
    assert L2.separable == 0                      # the fuse is cut across the old dimensions
    seq = [oracle.fuse(1, 3), oracle.split(1, [O // 4, 4, H * W]), oracle.reorder([0, 1, 3, 2])]
    want = oracle.layout_offsets(shape, seq)
    assert alt.layout_physical_shape(L2, shape) == (N, O // 4, H * W, 4)
    for idx in itertools.product(*map(range, shape)):
        off = alt.layout_offset(L2, shape, idx)
        assert off == want[idx]
        assert alt.layout_index_of(L2, shape, off) == idx
    # fuse then split back along the old boundaries stays separable
    L3 = alt.layout_from_prims((2, 6, 4), [alt.fuse(1, 2), alt.split(1, [3, 8]), alt.reorder([1, 0, 2])])
    assert L3.separable == 1
    seq3 = [oracle.fuse(1, 2), oracle.split(1, [3, 8]), oracle.reorder([1, 0, 2])]
    want3 = oracle.layout_offsets((2, 6, 4), seq3)
    for idx in itertools.product(range(2), range(6), range(4)):
        assert alt.layout_offset(L3, (2, 6, 4), idx) == want3[idx]


def test_layout_errors():
    for bad in ["NCHW", "NCHW->", "NCHW->NCH", "NCHW->NCHWW", "NCHW->NCHW16", "NCHW->NCHWc", "NCHW->NCHW0c",
                "nchw->NCHW", "NCHW->NCHX", "NNHW->NNHW", "NCHW->16NCHW"]:
        with pytest.raises(alt.AltError) as e:
            alt.layout_parse(bad)
        assert e.value.status == 2, bad
    L = alt.layout_parse("NCHW->NCHW16c")
    with pytest.raises(alt.AltError) as e:
        alt.layout_offset(L, (1, 24, 2, 2), (0, 0, 0, 0))       # 16 does not divide 24
    assert e.value.status == 3
    with pytest.raises(alt.AltError) as e:
        alt.layout_offset(L, (1, 32, 2, 2), (0, 32, 0, 0))      # index out of range
    assert e.value.status == 1
    with pytest.raises(alt.AltError) as e:
        alt.layout_from_prims((2, 10), [alt.split(1, [3, 4])])  # factors do not multiply to the extent
    assert e.value.status == 3
    with pytest.raises(alt.AltError) as e:
        alt.layout_from_prims((2, 10), [alt.reorder([0, 0])])
    assert e.value.status == 2


def test_hand_filled_general_layouts_are_checked_before_use():
    """A descriptor whose primitive list a caller wrote by hand (not through alt_layout_from_prims) is walked
    with the same checks before anything evaluates it: every corruption below used to index outside the
    descriptor's arrays; now each is an error status."""
    N, H, W, O = 2, 3, 5, 8
    shape = (N, H, W, O)
    good = alt.layout_from_prims(shape, [alt.fuse(1, 3), alt.split(1, [O // 4, 4, H * W]), alt.reorder([0, 1, 3, 2])])
    assert good.separable == 0
    assert alt.layout_offset(good, shape, (1, 2, 4, 7)) >= 0

    def broken(edit):
        L = alt.Layout.from_buffer_copy(bytes(good))
        edit(L)
        return L

    def set_v(q, j, val):
        def f(L):
            L.prims[q].v[j] = val
        return f

    def set_field(q, name, val):
        def f(L):
            setattr(L.prims[q], name, val)
        return f

    cases = [(set_v(2, 1, 9), 2),                 # reorder entry outside the rank
             (set_v(2, 1, 0), 2),                 # reorder repeats a dimension
             (set_field(2, "count", 7), 2),       # reorder of another rank
             (set_field(1, "dim", 5), 2),         # split of a dimension that does not exist
             (set_field(1, "count", 9), 2),       # more factors than the descriptor holds
             (set_v(1, 0, 3), 3),                 # factors no longer multiply to the extent
             (set_v(1, 1, -4), 2),                # negative factor
             (set_field(0, "count", 6), 2),       # fuse beyond the last dimension
             (set_field(0, "kind", 17), 2)]       # unknown primitive
    for edit, status in cases:
        L = broken(edit)
        for call in (lambda: alt.layout_offset(L, shape, (0, 0, 0, 0)), lambda: alt.layout_index_of(L, shape, 0),
                     lambda: alt.layout_physical_shape(L, shape)):
            with pytest.raises(alt.AltError) as e:
                call()
            assert e.value.status == status


def test_plan_chain_known_shortest_paths():
    inf = float("inf")
    # two layouts; op0 is fast only when writing layout 1, op1 only when reading layout 1
    op = [[[10, 4], [10, 4]], [[9, 9], [3, 3]]]
    cv = [[[0, 1], [1, 0]], [[0, 1], [1, 0]]]
    ins, outs, total = alt.plan_chain(op, cv, 0)
    assert (ins, outs, total) == ([0, 1], [1, 0], 7.0)            # producer writes the consumer's layout
    # an expensive conversion keeps everything in the input layout
    cv2 = [[[0, 100], [100, 0]], [[0, 100], [100, 0]]]
    op2 = [[[10, 50], [1, 1]], [[9, 9], [3, 3]]]
    ins, outs, total = alt.plan_chain(op2, cv2, 0)
    assert (ins, outs, total) == ([0, 0], [0, 0], 19.0)
    # a cheap conversion is inserted exactly where layouts differ
    op3 = [[[10, inf], [inf, 2]]]
    cv3 = [[[0, 3], [3, 0]]]
    ins, outs, total = alt.plan_chain(op3, cv3, 0)
    assert (ins, outs, total) == ([1], [1], 5.0)
    # brute force on a random 3-op, 3-layout table
    rng = np.random.RandomState(0)
    opc = rng.uniform(1, 10, (3, 3, 3)).astype(np.float32)
    cvc = rng.uniform(0.5, 3, (3, 3, 3)).astype(np.float32)
    best = inf
    for a in itertools.product(range(3), repeat=3):
        for b in itertools.product(range(3), repeat=3):
            prev, c = 1, 0.0
            for i in range(3):
                c += (0.0 if prev == a[i] else float(cvc[i][prev][a[i]])) + float(opc[i][a[i]][b[i]])
                prev = b[i]
            best = min(best, c)
    _, _, total = alt.plan_chain(opc.tolist(), cvc.tolist(), 1)
    assert abs(total - best) < 1e-4


def test_plan_graph_residual_block_rules():
    """Layout propagation over a residual block (conv, conv, add of the block input):
    the sum reads both inputs in the layout it writes, a tensor with two consumers is
    stored once, conversions appear exactly on the edges whose layouts differ."""
    inf = float("inf")
    K, A = alt.NODE_CONV, alt.NODE_ADD
    kind, in0, in1 = [K, K, A], [0, 1, 2], [0, 0, 0]
    zero = [[0, 0], [0, 0]]
    # convolutions are fast only in layout 1; conversions cost 2; the input arrives in layout 0
    op = [[[20, 20], [20, 5]], [[20, 20], [20, 5]], zero]
    cv = [[[0, 2], [2, 0]], [[0, 2], [2, 0]], [[0, 3], [3, 0]], [[0, 2], [2, 0]]]
    tl, rl, total = alt.plan_graph(kind, in0, in1, op, cv, [0, 0, 1.0], 0)
    # the input is converted to layout 1 once and that copy serves both conv0 and the sum
    assert tl == [0, 1, 1, 1] and rl == [[1, -1], [1, -1], [1, 1]] and total == 2 + 5 + 5 + 1
    # expensive conversions: everything stays in the input layout
    cvx = [[[0, 100], [100, 0]]] * 4
    tl, rl, total = alt.plan_graph(kind, in0, in1, op, cvx, [0, 0, 1.0], 0)
    assert tl == [0, 0, 0, 0] and rl == [[0, -1], [0, -1], [0, 0]] and total == 41.0
    # the input already in layout 1: no conversion anywhere
    tl, rl, total = alt.plan_graph(kind, in0, in1, op, cv, [0, 0, 1.0], 1)
    assert tl == [1, 1, 1, 1] and total == 11.0
    # impossible combinations are never chosen
    op_inf = [[[inf, inf], [inf, 5]], [[inf, 7], [inf, inf]], zero]
    tl, rl, total = alt.plan_graph(kind, in0, in1, op_inf, cv, [0, 0, 1.0], 0)
    assert rl[0][0] == 1 and tl[1] == 1 and rl[1][0] == 0 and tl[2] == 1
    # brute force over every assignment on random tables, three layouts, two-consumer tensors
    rng = np.random.RandomState(3)
    kind, in0, in1 = [K, K, A, K, A], [0, 1, 2, 3, 4], [0, 0, 0, 0, 1]
    n, nl = 5, 3
    opc = rng.uniform(1, 10, (n, nl, nl)).astype(np.float32)
    cvc = rng.uniform(0.5, 4, (n + 1, nl, nl)).astype(np.float32)
    addc = rng.uniform(0.5, 2, n).astype(np.float32)
    cc = lambda t, a, b: 0.0 if a == b else float(cvc[t][a][b])
    best = inf
    # (every stored layout and every layout each convolution reads; a copy of a tensor in one
    # layout is paid for once)
    convs = [i for i in range(n) if kind[i] == K]
    for s in itertools.product(range(nl), repeat=n):
        st = (2,) + s
        for reads in itertools.product(range(nl), repeat=len(convs)):
            made, tot = set(), 0.0
            def conv_to(t, b):
                if st[t] == b or (t, b) in made:
                    return 0.0
                made.add((t, b))
                return float(cvc[t][st[t]][b])
            for i in range(n):
                if kind[i] == K:
                    a = reads[convs.index(i)]
                    tot += conv_to(in0[i], a) + float(opc[i][a][st[i + 1]])
                else:
                    tot += float(addc[i]) + conv_to(in0[i], st[i + 1]) + conv_to(in1[i], st[i + 1])
            best = min(best, tot)
    tl, rl, total = alt.plan_graph(kind, in0, in1, opc.tolist(), cvc.tolist(), addc.tolist(), 2)
    assert abs(total - best) < 1e-3
    for i in range(n):
        if kind[i] == A:
            assert rl[i] == [tl[i + 1], tl[i + 1]]       # element-wise: output in the layout it reads
    # malformed graphs are refused
    with pytest.raises(alt.AltError):
        alt.plan_graph([K], [1], [0], [zero], [zero, zero], [0], 0)     # reads its own output


def test_calls_without_gpu_fail_loudly_not_silently():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    h = alt.Handle()
    d = alt.conv_desc(1, 16, 8, 8, 16, 3, 3, pad=1, in_dtype=alt.F32)
    assert h.conv2d_output_shape(d) == (1, 16, 8, 8)
    with pytest.raises(alt.AltError) as e:
        import ctypes
        alt.lib().alt_conv2d  # symbol exists
        h.conv2d(d, 16, 16, 16, stream=0)
    assert e.value.status == 6
    with pytest.raises(alt.AltError) as e:
        h.layout_transform(alt.F32, (2, 4), "MK->MK", 16, "MK->KM", 4096, stream=0)
    assert e.value.status == 6
    # argument errors are reported before any device work
    with pytest.raises(alt.AltError) as e:
        h.layout_transform(alt.F32, (2, 4), "MK->MK", 16, "MK->KM", 16, stream=0)
    assert e.value.status == 1
    # the pad form checks its layouts against their own shapes and refuses overlapping buffers before any device work
    with pytest.raises(alt.AltError) as e:
        h.layout_transform_pad(alt.BF16, (2, 12, 3, 3), "NCHW->NCHW", 16, (2, 12, 3, 3), "NCHW->NCHW16c", 8192, stream=0)
    assert e.value.status == 3                           # 16 does not divide the destination's 12 channels
    with pytest.raises(alt.AltError) as e:
        h.layout_transform_pad(alt.BF16, (2, 12, 3, 3), "NCHW->NCHW", 16, (2, 16, 3, 3), "NCHW->NCHW16c", 64, stream=0)
    assert e.value.status == 1
    bad = alt.conv_desc(1, 24, 8, 8, 16, 3, 3, pad=1, x_layout="NCHW->NCHW16c")
    with pytest.raises(alt.AltError) as e:
        h.conv2d(bad, 16, 16, 16, stream=0)
    assert e.value.status == 3
    # the other compute entry points refuse too (no host fallback anywhere)
    nhwc = alt.conv_desc(1, 64, 8, 8, 64, 3, 3, pad=1, in_dtype=alt.BF16, x_layout="NCHW->NHWC", w_layout="OIHW->OHWI",
                         y_layout="NCHW->NHWC")
    for call in (lambda: h.conv2d_add(nhwc, 16, 16, 16, 16, stream=0),
                 lambda: h.conv2d_transpose(alt.conv_desc(1, 16, 8, 8, 16, 3, 3, stride=2, pad=1), 16, 16, 16, workspace=16,
                                            ws_bytes=1 << 20, stream=0),
                 lambda: h.pack_weights_transpose(d, 16, 16, stream=0),
                 lambda: h.conv3d(alt.conv3d_desc(1, 16, 4, 8, 8, 16, 3, 3, 3, pad=1), 16, 16, 16, workspace=16, ws_bytes=1 << 20,
                                  stream=0),
                 lambda: h.conv3d(alt.conv3d_desc(1, 16, 4, 8, 8, 16, 1, 3, 3, pad=(0, 1, 1)), 16, 16, 16, stream=0),
                 lambda: h.pack_weights3d(alt.conv3d_desc(1, 16, 4, 8, 8, 16, 3, 3, 3, pad=1), 16, 16, stream=0),
                 lambda: h.conv3d_transpose(alt.conv3d_desc(1, 16, 4, 8, 8, 16, 3, 3, 3, stride=2, pad=1), 16, 16, 16, workspace=16,
                                            ws_bytes=1 << 24, stream=0),
                 lambda: h.pack_weights3d_transpose(alt.conv3d_desc(1, 16, 4, 8, 8, 16, 3, 3, 3, pad=1), 16, 16, stream=0),
                 lambda: h.tune_conv2d_multi([dict(d=nhwc, x=16, w=16, y=16, stream=0)]),
                 lambda: h.eltwise_add(alt.BF16, 64, 16, 16, 16, stream=0),
                 lambda: h.layout_transform_pad(alt.BF16, (2, 12, 3, 3), "NCHW->NCHW", 16, (2, 16, 3, 3), "NCHW->NCHW16c", 8192,
                                                stream=0),
                 lambda: h.unfold(alt.BF16, (4, 8), 0, 2, 1, 16, 4096, stream=0)):
        with pytest.raises(alt.AltError) as e:
            call()
        assert e.value.status == 6


def test_conv_transpose_sub_pixel_form_host_side(oracle):
    """Which descriptors take the sub-pixel form and the shape of their packed filter; and the identity the form
    rests on, checked with the oracle alone: the stride-1 convolution of x with the merged filter gives
    y'[n, (ph*sw + pw)*K + k, q, p] = y[n, k, q*sh + ph, p*sw + pw] of the transposed convolution."""
    h = alt.Handle()
    K, C = 8, 4
    for (H, W, R, S, stride, pad, dil, want) in [(6, 5, 4, 4, 2, 1, 1, (4 * K, C, 3, 3)), (5, 7, 2, 2, 2, 0, 1, (4 * K, C, 1, 1)),
                                                 (6, 5, 6, 6, 2, 2, 1, (4 * K, C, 3, 3)), (4, 5, 8, 8, 4, 2, 1, (16 * K, C, 3, 3)),
                                                 (6, 7, 2, 2, 2, 1, 3, (4 * K, C, 3, 3)), (5, 4, 2, 2, 3, 1, 1, (9 * K, C, 2, 2)),
                                                 (7, 9, 3, 3, 2, 1, 1, (K, C, 3, 3)), (5, 6, 3, 3, 1, 1, 1, (K, C, 3, 3)),
                                                 (8, 5, 3, 3, 2, 2, 2, (K, C, 3, 3))]:
        d = alt.conv_desc(2, C, H, W, K, R, S, stride=stride, pad=pad, dil=dil)
        got = h.conv2d_transpose_weight_shape(d)
        assert got == want, (R, S, stride, pad, dil, got)
        if got[0] == K:
            continue
        Rm, Sm = got[2], got[3]
        x = small_ints_f32(701, (2, C, H, W), -3, 3)
        w = small_ints_f32(702, (C, K, R, S), -3, 3)
        y = oracle.conv2d_transpose(x, w, stride=stride, pad=pad, dil=dil)
        # the window of tap offsets (ph + pad - r*dil)/stride over all phases, and the merged filter over it
        deltas = [(ph + pad - r * dil) // stride for ph in range(stride) for r in range(R) if (ph + pad - r * dil) % stride == 0]
        pm = -min(deltas)
        assert max(deltas) - min(deltas) + 1 == Rm == Sm
        wm = np.zeros((stride * stride * K, C, Rm, Sm), np.float32)
        for ph in range(stride):
            for pw in range(stride):
                for a in range(Rm):
                    for b in range(Sm):
                        nr, ns = ph + pad - stride * (a - pm), pw + pad - stride * (b - pm)
                        if nr >= 0 and ns >= 0 and nr % dil == 0 and ns % dil == 0 and nr // dil < R and ns // dil < S:
                            wm[(ph * stride + pw) * K:(ph * stride + pw + 1) * K, :, a, b] = w[:, :, nr // dil, ns // dil].T
        yq = oracle.conv2d(x, wm, stride=1, pad=pm)
        assert yq.shape == (2, stride * stride * K, y.shape[2] // stride, y.shape[3] // stride)
        back = yq.reshape(2, stride, stride, K, yq.shape[2], yq.shape[3]).transpose(0, 3, 4, 1, 5, 2).reshape(y.shape)
        assert np.array_equal(back, y)
    # blocked layouts: the merged extents must fit them (24*4 channels in blocks of 8 do), else the zero-insertion form
    d = alt.conv_desc(2, 16, 6, 5, 24, 4, 4, stride=2, pad=1, y_layout="NCHW->NCHW8c")
    assert h.conv2d_transpose_weight_shape(d) == (96, 16, 3, 3)
    d = alt.conv_desc(2, 16, 6, 5, 8, 2, 2, stride=3, pad=1, w_layout="OIHW->OIHW16o16i", x_layout="NCHW->NCHW16c")
    assert h.conv2d_transpose_weight_shape(d) == (8, 16, 2, 2)          # 9*8 output channels are no multiple of 16


def test_conv3d_transpose_sub_pixel_form_host_side(oracle):
    """The 3-D sub-pixel form: which descriptors take it, and, with the oracle alone, that the forward 3-D
    convolution of x with the merged filter holds the transposed result phase by phase."""
    h = alt.Handle()
    K, C = 4, 3
    assert h.conv3d_transpose_weight_shape(alt.conv3d_desc(2, C, 3, 4, 5, K, 3, 3, 3, stride=2, pad=1)) == (K, 3 * C, 3, 3)
    assert h.conv3d_transpose_weight_shape(alt.conv3d_desc(2, C, 3, 4, 5, K, 2, 2, 2, stride=2, pad=0)) == (8 * K, C, 1, 1)
    D, H, W, T, R, S, stride, pad = 3, 4, 5, 4, 4, 4, 2, 1
    d = alt.conv3d_desc(2, C, D, H, W, K, T, R, S, stride=stride, pad=pad)
    assert h.conv3d_transpose_weight_shape(d) == (8 * K, 3 * C, 3, 3)
    x = small_ints_f32(711, (2, C, D, H, W), -3, 3)
    w = small_ints_f32(712, (C, K, T, R, S), -3, 3)
    y = oracle.conv3d_transpose(x, w, stride=stride, pad=pad)
    pm, Tm = 1, 3
    wm = np.zeros((8 * K, C, Tm, Tm, Tm), np.float32)
    for pd in range(2):
        for ph in range(2):
            for pw in range(2):
                for a in range(Tm):
                    for b in range(Tm):
                        for c in range(Tm):
                            nt, nr, ns = pd + pad - stride * (a - pm), ph + pad - stride * (b - pm), pw + pad - stride * (c - pm)
                            if 0 <= nt < T and 0 <= nr < R and 0 <= ns < S:
                                j = (pd * 2 + ph) * 2 + pw
                                wm[j * K:(j + 1) * K, :, a, b, c] = w[:, :, nt, nr, ns].T
    yq = oracle.conv3d(x, wm, stride=1, pad=pm)
    assert yq.shape == (2, 8 * K, D, H, W)
    back = yq.reshape(2, 2, 2, 2, K, D, H, W).transpose(0, 4, 5, 1, 6, 2, 7, 3).reshape(y.shape)
    assert np.array_equal(back, y)


def test_conv3d_host_side(oracle):
    """Output shape of the 3-D convolution against the shape of the oracle's result, and the argument
    checks that need no device."""
    h = alt.Handle()
    for (D, H, W, T, R, S, stride, pad, dil) in [(7, 9, 8, 3, 3, 3, 1, 1, 1), (6, 7, 5, 3, 2, 3, (2, 1, 1), (1, 0, 2), (1, 1, 1)),
                                                 (9, 8, 7, 2, 3, 3, (1, 2, 1), (2, 1, 0), (3, 1, 2))]:
        d = alt.conv3d_desc(2, 4, D, H, W, 8, T, R, S, stride=stride, pad=pad, dil=dil)
        ref = oracle.conv3d(np.zeros((2, 4, D, H, W), np.float32), np.zeros((8, 4, T, R, S), np.float32), stride=stride, pad=pad, dil=dil)
        assert h.conv3d_output_shape(d) == ref.shape
    with pytest.raises(alt.AltError) as e:
        h.conv3d_workspace_size(alt.conv3d_desc(1, 16, 3, 8, 8, 16, 5, 3, 3, pad=(0, 1, 1)))   # filter deeper than the input
    assert e.value.status == 1
    with pytest.raises(alt.AltError) as e:
        h.conv3d_workspace_size(alt.conv3d_desc(1, 16, 4, 8, 8, 16, 3, 3, 3, pad=1, groups=2))
    assert e.value.status == 4
    with pytest.raises(alt.AltError) as e:
        h.conv3d_workspace_size(alt.conv3d_desc(1, 16, 4, 8, 8, 16, 3, 3, 3, stride=(0, 1, 1), pad=1))
    assert e.value.status == 1
    for (D, H, W, T, R, S, stride, pad, dil) in [(4, 5, 6, 3, 2, 3, 2, 1, 1), (3, 4, 5, 3, 3, 2, (2, 1, 3), (1, 0, 1), (1, 2, 1))]:
        d = alt.conv3d_desc(2, 4, D, H, W, 8, T, R, S, stride=stride, pad=pad, dil=dil)
        ref = oracle.conv3d_transpose(np.zeros((2, 4, D, H, W), np.float32), np.zeros((4, 8, T, R, S), np.float32), stride=stride,
                                      pad=pad, dil=dil)
        assert h.conv3d_transpose_output_shape(d) == ref.shape
    with pytest.raises(alt.AltError) as e:
        h.conv3d_transpose_workspace_size(alt.conv3d_desc(1, 16, 4, 8, 8, 16, 3, 3, 3, stride=2, pad=(3, 1, 1)))
    assert e.value.status == 4
    # the 2-D problems behind the 3-D operators (what alt_tune_conv2d is given to tune them)
    f = h.conv3d_problem(alt.conv3d_desc(2, 16, 6, 8, 7, 32, 3, 3, 3, stride=(2, 1, 1), pad=1))
    assert (f.N, f.C, f.H, f.W, f.K, f.R, f.S, f.stride_h, f.pad_h) == (2 * 3, 3 * 16, 8, 7, 32, 3, 3, 1, 1)
    f = h.conv3d_transpose_problem(alt.conv3d_desc(2, 16, 3, 4, 5, 32, 3, 3, 3, stride=2, pad=1))
    assert (f.N, f.C, f.H, f.W, f.K, f.stride_h, f.stride_w, f.pad_h, f.pad_w) == (2 * 5, 3 * 16, 7, 9, 32, 1, 1, 1, 1)
    f = h.conv2d_transpose_problem(alt.conv_desc(2, 16, 6, 5, 8, 4, 4, stride=2, pad=1))
    assert (f.N, f.C, f.H, f.W, f.K, f.R, f.S, f.stride_h, f.pad_h) == (2, 16, 6, 5, 32, 3, 3, 1, 1)
    f = h.conv2d_transpose_problem(alt.conv_desc(2, 16, 6, 5, 8, 3, 3, stride=2, pad=1))
    assert (f.N, f.C, f.H, f.W, f.K, f.R, f.S, f.stride_h, f.pad_h) == (2, 16, 11, 9, 8, 3, 3, 1, 1)
    # the unfolded input is counted: T*C channels for every output slice
    d = alt.conv3d_desc(2, 16, 6, 8, 8, 16, 3, 3, 3, stride=(2, 1, 1), pad=1, in_dtype=alt.BF16)
    assert h.conv3d_workspace_size(d) >= 2 * 3 * (3 * 16) * 8 * 8 * 2


def test_conv_transpose_host_side(oracle):
    """Output shape of the transposed C2D against the oracle's, argument checks that need no
    device, and the multi-call entry's handling of an empty or bad list."""
    for (H, W, R, S, stride, pad, dil) in [(7, 9, 3, 3, 2, 1, 1), (5, 6, 4, 4, 2, 1, 1), (4, 7, 3, 2, 3, 0, 1), (8, 5, 3, 3, 2, 2, 2)]:
        d = alt.conv_desc(2, 16, H, W, 32, R, S, stride=stride, pad=pad, dil=dil)
        h = alt.Handle()
        assert h.conv2d_transpose_output_shape(d) == oracle.conv2d_transpose_out_shape((2, 16, H, W), (16, 32, R, S), stride, pad, dil)
    h = alt.Handle()
    with pytest.raises(alt.AltError) as e:
        h.conv2d_transpose(alt.conv_desc(1, 16, 8, 8, 16, 3, 3, stride=2, pad=3), 16, 16, 16, workspace=16, ws_bytes=1 << 20, stream=0)
    assert e.value.status == 4                                      # padding beyond dil*(R-1)
    with pytest.raises(alt.AltError) as e:
        h.conv2d_transpose(alt.conv_desc(1, 16, 8, 8, 16, 3, 3, stride=2, pad=1, groups=2), 16, 16, 16, workspace=16, ws_bytes=1 << 20, stream=0)
    assert e.value.status == 4
    with pytest.raises(alt.AltError) as e:
        h.conv2d_transpose_workspace_size(alt.conv_desc(1, 16, 8, 8, 16, 3, 3, stride=0, pad=1))
    assert e.value.status == 1
    h.conv2d_multi([])                                              # nothing to issue: fine
    import ctypes
    assert alt.lib().alt_conv2d_multi(h._h, None, ctypes.c_int32(2)) == 1
    assert alt.lib().alt_conv2d_multi(h._h, None, ctypes.c_int32(-1)) == 1


# ---- the conversion operator's launch plan, replayed on the host -------------------------------------

_PLAN_PAIRS = [("NCHW->NCHW", "NCHW->NHWC"), ("NCHW->NHWC", "NCHW->NCHW"), ("NCHW->NCHW", "NCHW->NCHW16c"),
               ("NCHW->NCHW16c", "NCHW->NCHW"), ("NCHW->NCHW", "NCHW->NCHW32c"), ("NCHW->NCHW", "NCHW->HWNC"),
               ("NCHW->CNHW", "NCHW->NCHW4c"), ("NCHW->NCHW32c", "NCHW->NHWC")]
_PLAN_SHAPES = [(2, 32, 5, 7), (3, 64, 14, 14), (1, 32, 1, 1), (2, 96, 7, 7), (1, 32, 9, 40), (2, 64, 56, 56),
                (4, 256, 14, 14), (8, 512, 7, 7), (40, 512, 7, 7), (5, 32, 49, 1)]


@pytest.mark.parametrize("shape", _PLAN_SHAPES)
def test_transform_plan_replays_to_the_index_maps(shape):
    """Every workgroup of the tile kernel's launch plan, replayed on the host (alt_layout_transform_plan):
    each destination element is written exactly once, from the source element that the two layouts' index
    maps name; every LDS index lies inside the tile; every vector access is aligned and inside its buffer.
    Both element sizes, aligned buffers and buffers off by one element or by eight bytes."""
    h = alt.Handle()
    tiles = 0
    for a, b in _PLAN_PAIRS:
        for dt, es in ((alt.F32, 4), (alt.BF16, 2)):
            for sm, dm in ((0, 0), (es, 0), (0, es), (8, 8)):
                p = h.layout_transform_plan(dt, shape, a, b, sm, dm, replay=True)
                assert p.kind in (0, 1, 2, 3)
                if p.kind == 3:
                    tiles += 1
                    assert p.mismatches == 0, (shape, a, b, dt, sm, dm, p.mismatches, p.src_flat, p.dst_flat,
                                               p.tile_a, p.tile_b, p.tile_g)
                    assert p.lds_bytes <= 64 * 1024 and p.workgroups >= 1
    assert tiles > 0 or shape[2] * shape[3] == 1        # (a 1x1 image leaves nothing to transpose)


def test_transform_plan_takes_contiguous_runs_where_rows_are_odd():
    """49-element rows (7x7 images) take no 16-byte vectors on their own; the plan moves them as part of
    one contiguous run per tile (a flat side) with 16-byte accesses, on the side where they are contiguous."""
    h = alt.Handle()
    for dt in (alt.F32, alt.BF16):
        p = h.layout_transform_plan(dt, (64, 512, 7, 7), "NCHW->NCHW", "NCHW->NHWC")
        assert p.kind == 3 and p.src_flat == 1 and p.load_bytes == 16 and p.store_bytes == 16 and p.tile_a == 49
        p = h.layout_transform_plan(dt, (64, 512, 7, 7), "NCHW->NHWC", "NCHW->NCHW")
        assert p.kind == 3 and p.dst_flat == 1 and p.load_bytes == 16 and p.store_bytes == 16 and p.tile_b == 49
        p = h.layout_transform_plan(dt, (64, 512, 7, 7), "NCHW->NCHW", "NCHW->NCHW16c")
        assert p.kind == 3 and p.src_flat == 1 and p.load_bytes == 16 and p.store_bytes == 16
    # buffers that are not 16-byte aligned cannot be flat
    p = h.layout_transform_plan(alt.BF16, (64, 512, 7, 7), "NCHW->NCHW", "NCHW->NHWC", 2, 0)
    assert p.kind == 3 and p.src_flat == 0 and p.load_bytes == 2
    with pytest.raises(alt.AltError):
        h.layout_transform_plan(alt.F32, (2, 4, 2, 2), "NCHW->NCHW", "NCHW->NHWC", 2, 0)     # not a multiple of the element size


def test_kernel_families_follow_the_layouts():
    """Which kernel family covers which layouts (host-side applicability only, no GPU needed): the patch-resident
    and streaming kernels take NHWC or channel-blocked activations and output with OHWI weights, the
    channel-planar kernels NCHW activations and OIHW weights with NCHW or NHWC output, the transpose-read
    streaming kernels row-major B; and without a tuned entry the library picks from the family written for the layout."""
    h = alt.Handle()

    def families(d, kind="conv"):
        count = h.conv2d_variant_count(d) if kind == "conv" else h.gemm_variant_count(d)
        fam = set()
        for v in range(count):
            try:
                name = h.conv2d_variant_name(d, v) if kind == "conv" else h.gemm_variant_name(d, v)
            except alt.AltError as e:
                assert e.status == 4
                continue
            for key in ("_direct_", "_stream_", "_streamkn_", "_planar_"):
                if key in name:
                    fam.add(key.strip("_"))
        return fam

    def conv(xl, wl, yl, R=3, C=128, K=128):
        return alt.conv_desc(16, C, 28, 28, K, R, R, stride=1, pad=R // 2, in_dtype=alt.BF16, out_dtype=alt.BF16,
                             x_layout="NCHW->" + xl, w_layout="OIHW->" + wl, y_layout="NCHW->" + yl)

    assert families(conv("NHWC", "OHWI", "NHWC")) == {"direct"}
    assert families(conv("NCHW16c", "OHWI", "NCHW32c")) == {"direct"}
    assert families(conv("NCHW64c", "OHWI", "NHWC", R=1)) == {"direct", "stream"}
    assert families(conv("NCHW", "OIHW", "NCHW")) == {"planar"}
    assert families(conv("NCHW", "OIHW", "NHWC")) == {"planar"}
    assert families(conv("NCHW", "OHWI", "NCHW")) == set()            # planar kernels scatter OIHW rows
    assert families(conv("NCHW16c", "OIHW16o16i", "NCHW16c")) == set()        # blocked weights: implicit-GEMM kernels
    assert families(conv("NCHW", "OIHW", "NCHW", C=96)) == set()      # channels not a multiple of 64
    assert "_planar_" in h.conv2d_variant_name(conv("NCHW", "OIHW", "NCHW"), -1)
    assert "_direct_" in h.conv2d_variant_name(conv("NCHW32c", "OHWI", "NCHW32c"), -1)

    def gemm(bl, N=768):
        return alt.gemm_desc(2048, N, 768, in_dtype=alt.BF16, out_dtype=alt.F32, b_layout="KN->" + bl)

    assert families(gemm("NK"), "gemm") == {"stream", "direct"}       # (a product is a 1x1 convolution to the patch kernels)
    assert families(gemm("KN"), "gemm") == {"streamkn"}
    assert families(gemm("KN", N=772), "gemm") == set()               # row-major B is loaded eight columns at a time
    assert "_streamkn_" in h.gemm_variant_name(gemm("KN"), -1)
    assert "_stream_" in h.gemm_variant_name(gemm("NK"), -1)

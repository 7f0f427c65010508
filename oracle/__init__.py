"""Python face of the CPU oracle (oracle/alt_oracle.c).

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the benchmark's
cpu_baseline leg may import this package; the GPU library and its binding never
do, and it never imports them.

Layouts are primitive sequences exactly as in Table 1 of the paper (split,
reorder, fuse), with 0-based dimension numbers; `paper_seq` converts the
paper's 1-based notation.  Convolution and matrix product are computed on
logical NCHW / OIHW / row-major arrays; other layouts are reached through
`layout_transform`.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "alt_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force=False):
    """Compile the oracle with gcc (plain C, OpenMP over the outermost
    independent loop).  Rebuilds when the source is newer than the library."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    tmp = _LIB + ".tmp%d" % os.getpid()
    subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
                           "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
    os.replace(tmp, _LIB)
    return _LIB


class _Prim(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("k", ctypes.c_int32), ("m", ctypes.c_int32),
                ("pad_", ctypes.c_int32), ("v", ctypes.c_int64 * 8)]


class _Conv(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in
                ("N", "C", "H", "W", "K", "R", "S", "stride_h", "stride_w",
                 "pad_h", "pad_w", "dil_h", "dil_w")] + \
               [(n, ctypes.c_int32) for n in ("in_bf16", "out_bf16", "has_bias", "relu")]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        L.orc_layout_offset.restype = ctypes.c_int64
        L.orc_unfold_tiles.restype = ctypes.c_int64
        L.orc_unfold_tiles.argtypes = [ctypes.c_int64] * 3
        L.orc_conv_out_h.restype = ctypes.c_int64
        L.orc_conv_out_w.restype = ctypes.c_int64
        L.orc_f32_to_bf16.restype = ctypes.c_uint16
        L.orc_f32_to_bf16.argtypes = [ctypes.c_float]
        _lib = L
    return _lib


def num_threads():
    return int(lib().orc_num_threads())


# ---------------------------------------------------------------- layouts ----

def split(k, factors):
    return ("split", int(k), [int(f) for f in factors])


def reorder(perm):
    return ("reorder", [int(p) for p in perm])


def fuse(k, m):
    """Fuse the m dimensions k .. k+m-1."""
    return ("fuse", int(k), int(m))


def paper_seq(seq):
    """Convert a sequence written as in the paper (1-based dims; fuse given as
    the list of dims) to this module's 0-based form."""
    out = []
    for p in seq:
        if p[0] == "split":
            out.append(split(p[1] - 1, p[2]))
        elif p[0] == "reorder":
            out.append(reorder([q - 1 for q in p[1]]))
        elif p[0] == "fuse":
            dims = list(p[1])
            assert dims == list(range(dims[0], dims[0] + len(dims)))
            out.append(fuse(dims[0] - 1, len(dims)))
        else:
            raise ValueError(p)
    return out


def _pack(seq):
    arr = (_Prim * max(1, len(seq)))()
    for i, p in enumerate(seq):
        if p[0] == "split":
            arr[i].kind, arr[i].k, arr[i].m = 0, p[1], len(p[2])
            for j, f in enumerate(p[2]):
                arr[i].v[j] = f
        elif p[0] == "reorder":
            arr[i].kind, arr[i].k, arr[i].m = 1, 0, len(p[1])
            for j, f in enumerate(p[1]):
                arr[i].v[j] = f
        elif p[0] == "fuse":
            arr[i].kind, arr[i].k, arr[i].m = 2, p[1], p[2]
        else:
            raise ValueError(p)
    return arr, len(seq)


def _i64(a):
    return (ctypes.c_int64 * len(a))(*[int(x) for x in a])


def seq_from_string(name, shape):
    """Primitive sequence for a layout written as dimension letters, e.g.
    logical "NCHW" stored as "NHWC" or "NCHW16c", logical "OIHW" stored as
    "OIHW16i32o", logical "MK" stored as "KM" or "MK64m32k".  `name` is
    "LOGICAL->PHYSICAL".  Built the way Section 4.1.1 builds N(O/o_t)HWo_t:
    one split per blocked dimension, then one reorder."""
    logical, physical = name.split("->")
    toks = []                     # (letter, factor or None), physical order
    num = ""
    for ch in physical:
        if ch.isdigit():
            num += ch
        else:
            toks.append((ch, int(num) if num else None))
            num = ""
    seq = []
    cur = [(c, None) for c in logical]      # dims after the splits so far
    for d, c in enumerate(logical):
        inner = [t for t in toks if t[0] == c.lower() and t[1] is not None]
        if not inner:
            continue
        assert len(inner) == 1, "one blocking level per dimension"
        f = inner[0][1]
        pos = cur.index((c, None))
        assert shape[d] % f == 0
        seq.append(split(pos, [shape[d] // f, f]))
        cur[pos:pos + 1] = [(c, None), (c.lower(), f)]
    perm = []
    for t in toks:
        key = (t[0], None) if t[0].isupper() else (t[0], t[1])
        perm.append(cur.index(key))
    assert sorted(perm) == list(range(len(cur))), (name, perm)
    if perm != list(range(len(cur))):
        seq.append(reorder(perm))
    return seq


def layout_shape(shape, seq):
    arr, n = _pack(seq)
    out = (ctypes.c_int64 * 12)()
    r = lib().orc_layout_shape(len(shape), _i64(shape), arr, n, out)
    if r < 0:
        raise ValueError("bad primitive sequence")
    return tuple(out[i] for i in range(r))


def layout_index(shape, seq, idx):
    """(transformed index tuple, row-major offset) of one logical index."""
    arr, n = _pack(seq)
    out = (ctypes.c_int64 * 12)()
    off = lib().orc_layout_offset(len(shape), _i64(shape), arr, n, _i64(idx), out)
    if off < 0:
        raise ValueError("bad index or primitive sequence")
    r = len(layout_shape(shape, seq))
    return tuple(out[i] for i in range(r)), int(off)


def layout_offsets(shape, seq):
    """int64 array of logical `shape`: physical offset of every element."""
    arr, n = _pack(seq)
    out = np.empty(int(np.prod(shape)), dtype=np.int64)
    rc = lib().orc_layout_offsets_all(len(shape), _i64(shape), arr, n,
                                      out.ctypes.data_as(ctypes.c_void_p))
    if rc != 0:
        raise ValueError("bad primitive sequence")
    return out.reshape(shape)


def layout_transform(src, shape, seq_src, seq_dst):
    """Conversion operator.  `src` is the flat physical buffer (uint16/uint32 or
    any 2/4-byte dtype) of a tensor of logical `shape` stored under seq_src;
    returns the flat physical buffer under seq_dst, same dtype."""
    src = np.ascontiguousarray(src).reshape(-1)
    assert src.size == int(np.prod(shape))
    dst = np.empty_like(src)
    a, na = _pack(seq_src)
    b, nb = _pack(seq_dst)
    rc = lib().orc_layout_transform(src.dtype.itemsize, len(shape), _i64(shape),
                                    a, na, src.ctypes.data_as(ctypes.c_void_p),
                                    b, nb, dst.ctypes.data_as(ctypes.c_void_p))
    if rc != 0:
        raise ValueError("layout_transform failed")
    return dst


def pad_transform(src, src_shape, seq_src, dst_shape, seq_dst):
    """The pad primitive (Section 4.1.2: zeros appended to selected dimensions) and its inverse,
    unpad, carried by the conversion operator (Section 4.2: a padding operator with a propagated
    layout pads and converts in one pass).  `src` is the flat buffer of a tensor of logical
    src_shape under seq_src; the result is the flat buffer of the tensor of logical dst_shape
    under seq_dst whose element at index i is the source's where i lies inside both shapes and
    zero (all bits clear) elsewhere.  Written as its definition: to logical order, copy the
    common box into zeros, to the destination layout."""
    src_shape, dst_shape = tuple(int(v) for v in src_shape), tuple(int(v) for v in dst_shape)
    assert len(src_shape) == len(dst_shape)
    logical = layout_transform(src, src_shape, seq_src, []).reshape(src_shape)
    out = np.zeros(dst_shape, dtype=logical.dtype)
    box = tuple(slice(0, min(a, b)) for a, b in zip(src_shape, dst_shape))
    out[box] = logical[box]
    return layout_transform(out.reshape(-1), dst_shape, [], seq_dst)


# ----------------------------------------------------------------- unfold ----

def unfold_tiles(D, B, S):
    return int(lib().orc_unfold_tiles(D, B, S))


def unfold_1d(src, B, S):
    src = np.ascontiguousarray(src, dtype=np.float64)
    T = unfold_tiles(src.size, B, S)
    dst = np.empty((T, B), dtype=np.float64)
    lib().orc_unfold_1d(src.ctypes.data_as(ctypes.c_void_p), ctypes.c_int64(src.size),
                        ctypes.c_int64(B), ctypes.c_int64(S),
                        dst.ctypes.data_as(ctypes.c_void_p))
    return dst


def unfold(x, dim, B, S):
    """The unfold primitive (Section 4.1.2) on dimension `dim` of an array: every
    1-D line along `dim` goes through unfold_1d.  Values pass through float64
    (exact for float32 and for integers below 2^53); returns float64 of shape
    x.shape[:dim] + (T, B) + x.shape[dim+1:]."""
    x = np.asarray(x)
    moved = np.moveaxis(x, dim, -1)
    lines = moved.reshape(-1, x.shape[dim])
    T = unfold_tiles(x.shape[dim], B, S)
    out = np.empty((lines.shape[0], T, B), dtype=np.float64)
    for j in range(lines.shape[0]):
        out[j] = unfold_1d(lines[j], B, S)
    out = out.reshape(moved.shape[:-1] + (T, B))
    return np.moveaxis(np.moveaxis(out, -2, dim), -1, dim + 1)


def unfold_access(V, i, r, B, S, M):
    t, w = ctypes.c_int64(), ctypes.c_int64()
    lib().orc_unfold_access(ctypes.c_int64(V), ctypes.c_int64(i), ctypes.c_int64(r),
                            ctypes.c_int64(B), ctypes.c_int64(S), ctypes.c_int64(M),
                            ctypes.byref(t), ctypes.byref(w))
    return t.value, w.value


# ------------------------------------------------------------- conv / gemm ----

def f32_to_bf16_bits(x):
    x = np.ascontiguousarray(x, dtype=np.float32)
    f = lib().orc_f32_to_bf16
    return np.array([f(float(v)) for v in x.reshape(-1)], dtype=np.uint16).reshape(x.shape)


def _conv_desc(x, w, stride, pad, dil, out_bf16, bias, relu):
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    assert C2 == C
    sh, sw = (stride, stride) if np.isscalar(stride) else stride
    ph, pw = (pad, pad) if np.isscalar(pad) else pad
    dh, dw = (dil, dil) if np.isscalar(dil) else dil
    in_bf16 = x.dtype == np.uint16
    assert (w.dtype == np.uint16) == in_bf16
    d = _Conv(N, C, H, W, K, R, S, sh, sw, ph, pw, dh, dw,
              int(in_bf16), int(out_bf16), int(bias is not None), int(relu))
    return d


def conv2d(x, w, stride=1, pad=0, dil=1, out_bf16=False, bias=None, relu=False, groups=1):
    """x: (N,C,H,W), w: (K,C/groups,R,S); float32 arrays, or uint16 arrays of bf16
    bits.  Returns (N,K,OH,OW) float32, or uint16 bf16 bits if out_bf16.
    groups > 1 (the group-wise and depth-wise C2D of Section 6.1): output
    channels [g*K/groups, (g+1)*K/groups) are the convolution of input channels
    [g*C/groups, (g+1)*C/groups) with their own filters, i.e. `groups`
    independent convolutions side by side, which is how it is computed here."""
    if groups > 1:
        C, K = x.shape[1], w.shape[0]
        if C % groups or K % groups or w.shape[1] != C // groups:
            raise ValueError("conv2d: groups must divide C and K, w is (K, C/groups, R, S)")
        cg, kg = C // groups, K // groups
        parts = [conv2d(x[:, g * cg:(g + 1) * cg], w[g * kg:(g + 1) * kg], stride, pad, dil, out_bf16,
                        None if bias is None else np.asarray(bias)[g * kg:(g + 1) * kg], relu)
                 for g in range(groups)]
        return np.concatenate(parts, axis=1)
    x = np.ascontiguousarray(x)
    w = np.ascontiguousarray(w)
    d = _conv_desc(x, w, stride, pad, dil, out_bf16, bias, relu)
    OH, OW = int(lib().orc_conv_out_h(ctypes.byref(d))), int(lib().orc_conv_out_w(ctypes.byref(d)))
    y = np.empty((d.N, d.K, OH, OW), dtype=np.uint16 if out_bf16 else np.float32)
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    rc = lib().orc_conv2d(ctypes.byref(d), x.ctypes.data_as(ctypes.c_void_p),
                          w.ctypes.data_as(ctypes.c_void_p),
                          None if b is None else b.ctypes.data_as(ctypes.c_void_p),
                          y.ctypes.data_as(ctypes.c_void_p))
    if rc != 0:
        raise ValueError("conv2d: empty output")
    return y


def conv2d_at(x, w, flat, stride=1, pad=0, dil=1, bias=None, relu=False):
    """Double-precision values of the outputs with flat (N,K,OH,OW) indices
    `flat`."""
    x = np.ascontiguousarray(x)
    w = np.ascontiguousarray(w)
    d = _conv_desc(x, w, stride, pad, dil, False, bias, relu)
    flat = np.ascontiguousarray(flat, dtype=np.int64)
    out = np.empty(flat.size, dtype=np.float64)
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    rc = lib().orc_conv2d_at(ctypes.byref(d), x.ctypes.data_as(ctypes.c_void_p),
                             w.ctypes.data_as(ctypes.c_void_p),
                             None if b is None else b.ctypes.data_as(ctypes.c_void_p),
                             flat.ctypes.data_as(ctypes.c_void_p), ctypes.c_int64(flat.size),
                             out.ctypes.data_as(ctypes.c_void_p))
    if rc != 0:
        raise ValueError("conv2d_at failed")
    return out


def bf16_bits_to_f64(b):
    """uint16 bf16 bit patterns -> float64 values (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def eltwise_add(a, b=None, relu=False):
    """Element-wise operator of a graph (Section 4.2: simple operators take the
    layout of their producer, so this works on arrays of any shape in any one
    layout).  y = a + b (b may be None: y = a), then max(y, 0) if relu.
    float32 arrays: IEEE single-precision addition.  uint16 arrays of bf16
    bits: the exact sum rounded once to bf16, to nearest even."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        s = bf16_bits_to_f64(a)
        if b is not None:
            s = s + bf16_bits_to_f64(b)            # exact: both fit 8 significant bits
        if relu:
            s = np.maximum(s, 0.0)
        # float32 holds the sum exactly unless the exponents are > 16 apart, and then the
        # smaller term is far below half a bf16 step of the larger: one rounding either way
        return f32_to_bf16_bits(s.astype(np.float32))
    s = a.astype(np.float32)
    if b is not None:
        s = (s + np.asarray(b, dtype=np.float32)).astype(np.float32)
    if relu:
        s = np.maximum(s, np.float32(0))
    return s


def conv2d_transpose_out_shape(x_shape, w_shape, stride=1, pad=0, dil=1):
    """(N, K, OH, OW) of the transposed C2D: OH = (H-1)*stride - 2*pad + dil*(R-1) + 1."""
    N, C, H, W = x_shape
    C2, K, R, S = w_shape
    assert C2 == C
    return (N, K, (H - 1) * stride - 2 * pad + dil * (R - 1) + 1, (W - 1) * stride - 2 * pad + dil * (S - 1) + 1)


def conv2d_transpose(x, w, stride=1, pad=0, dil=1, out_bf16=False, bias=None, relu=False):
    """Transposed C2D (the T2D of Section 6.1's operator list): the adjoint of the
    C2D that maps K channels to C with the same filter, written out as a scatter:

        y[n, k, ih*stride - pad + r*dil, iw*stride - pad + s*dil] += x[n, c, ih, iw] * w[c, k, r, s]

    over all (n, c, ih, iw, k, r, s) whose target lies inside the output.  x: (N,C,H,W),
    w: (C,K,R,S), float32 or uint16 bf16 bits; sums in float64, one rounding to float32
    (then bias, ReLU, and a second rounding to bf16 bits if out_bf16).  Pure numpy: one
    channel contraction per filter tap, added into a strided view of the uncropped
    output."""
    x = np.asarray(x)
    w = np.asarray(w)
    xf = bf16_bits_to_f64(x) if x.dtype == np.uint16 else x.astype(np.float64)
    wf = bf16_bits_to_f64(w) if w.dtype == np.uint16 else w.astype(np.float64)
    N, C, H, W = xf.shape
    C2, K, R, S = wf.shape
    if C2 != C:
        raise ValueError("conv2d_transpose: w is (C, K, R, S)")
    _, _, OH, OW = conv2d_transpose_out_shape(xf.shape, wf.shape, stride, pad, dil)
    if OH < 1 or OW < 1:
        raise ValueError("conv2d_transpose: empty output")
    FH, FW = (H - 1) * stride + dil * (R - 1) + 1, (W - 1) * stride + dil * (S - 1) + 1
    full = np.zeros((N, K, FH, FW), dtype=np.float64)
    for r in range(R):
        for s in range(S):
            full[:, :, r * dil:r * dil + (H - 1) * stride + 1:stride,
                 s * dil:s * dil + (W - 1) * stride + 1:stride] += np.einsum("nchw,ck->nkhw", xf, wf[:, :, r, s])
    y = full[:, :, pad:pad + OH, pad:pad + OW].astype(np.float32)
    if bias is not None:
        y = (y + np.asarray(bias, dtype=np.float32).reshape(1, K, 1, 1)).astype(np.float32)
    if relu:
        y = np.maximum(y, np.float32(0))
    return f32_to_bf16_bits(y) if out_bf16 else y


def conv3d(x, w, stride=1, pad=0, dil=1):
    """3-D convolution (the C3D of Section 6.1's operator list) from its definition:

        y[n, k, od, oh, ow] = sum_{c,t,r,s} x[n, c, od*sd - pd + t*dd, oh*sh - ph + r*dh, ow*sw - pw + s*dw] * w[k, c, t, r, s]

    with zeros outside the input.  x: (N,C,D,H,W), w: (K,C,T,R,S), float32 or uint16 bf16
    bits; stride, pad, dil: one number for all three directions or (depth, height, width);
    sums in float64, one rounding to float32.  Pure numpy: one channel contraction per
    filter tap over a strided view of the zero-padded input."""
    x = np.asarray(x)
    w = np.asarray(w)
    xf = bf16_bits_to_f64(x) if x.dtype == np.uint16 else x.astype(np.float64)
    wf = bf16_bits_to_f64(w) if w.dtype == np.uint16 else w.astype(np.float64)
    N, C, D, H, W = xf.shape
    K, C2, T, R, S = wf.shape
    if C2 != C:
        raise ValueError("conv3d: w is (K, C, T, R, S)")
    three = lambda v: tuple(int(e) for e in v) if isinstance(v, (tuple, list)) else (int(v),) * 3
    (sd, sh, sw), (pd, ph, pw), (dd, dh, dw) = three(stride), three(pad), three(dil)
    OD = (D + 2 * pd - dd * (T - 1) - 1) // sd + 1
    OH = (H + 2 * ph - dh * (R - 1) - 1) // sh + 1
    OW = (W + 2 * pw - dw * (S - 1) - 1) // sw + 1
    if min(OD, OH, OW) < 1:
        raise ValueError("conv3d: empty output")
    xp = np.pad(xf, ((0, 0), (0, 0), (pd, pd), (ph, ph), (pw, pw)))
    y = np.zeros((N, K, OD, OH, OW), dtype=np.float64)
    for t in range(T):
        for r in range(R):
            for s_ in range(S):
                win = xp[:, :, t * dd:t * dd + (OD - 1) * sd + 1:sd, r * dh:r * dh + (OH - 1) * sh + 1:sh,
                         s_ * dw:s_ * dw + (OW - 1) * sw + 1:sw]
                y += np.einsum("ncdhw,kc->nkdhw", win, wf[:, :, t, r, s_])
    return y.astype(np.float32)


def conv3d_transpose(x, w, stride=1, pad=0, dil=1):
    """Transposed 3-D convolution (the T3D of Section 6.1's operator list): the adjoint of the
    C3D that maps K channels to C with the same filter, written out as a scatter:

        y[n, k, id*sd - pd + t*dd, ih*sh - ph + r*dh, iw*sw - pw + s*dw] += x[n, c, id, ih, iw] * w[c, k, t, r, s]

    over all terms whose target lies inside the output of extents (D-1)*sd - 2*pd + dd*(T-1) + 1
    (likewise for the other two).  x: (N,C,D,H,W), w: (C,K,T,R,S), float32 or uint16 bf16 bits;
    stride, pad, dil: one number or (depth, height, width); sums in float64, one rounding to
    float32.  Pure numpy: one channel contraction per filter tap, added into a strided view of
    the uncropped output."""
    x = np.asarray(x)
    w = np.asarray(w)
    xf = bf16_bits_to_f64(x) if x.dtype == np.uint16 else x.astype(np.float64)
    wf = bf16_bits_to_f64(w) if w.dtype == np.uint16 else w.astype(np.float64)
    N, C, D, H, W = xf.shape
    C2, K, T, R, S = wf.shape
    if C2 != C:
        raise ValueError("conv3d_transpose: w is (C, K, T, R, S)")
    three = lambda v: tuple(int(e) for e in v) if isinstance(v, (tuple, list)) else (int(v),) * 3
    (sd, sh, sw), (pd, ph, pw), (dd, dh, dw) = three(stride), three(pad), three(dil)
    FD, FH, FW = (D - 1) * sd + dd * (T - 1) + 1, (H - 1) * sh + dh * (R - 1) + 1, (W - 1) * sw + dw * (S - 1) + 1
    OD, OH, OW = FD - 2 * pd, FH - 2 * ph, FW - 2 * pw
    if min(OD, OH, OW) < 1:
        raise ValueError("conv3d_transpose: empty output")
    full = np.zeros((N, K, FD, FH, FW), dtype=np.float64)
    for t in range(T):
        for r in range(R):
            for s_ in range(S):
                full[:, :, t * dd:t * dd + (D - 1) * sd + 1:sd, r * dh:r * dh + (H - 1) * sh + 1:sh,
                     s_ * dw:s_ * dw + (W - 1) * sw + 1:sw] += np.einsum("ncdhw,ck->nkdhw", xf, wf[:, :, t, r, s_])
    return full[:, :, pd:pd + OD, ph:ph + OH, pw:pw + OW].astype(np.float32)


def conv_out_shape(x_shape, w_shape, stride=1, pad=0, dil=1):
    d = _Conv(*x_shape, w_shape[0], w_shape[2], w_shape[3], stride, stride, pad, pad, dil, dil,
              0, 0, 0, 0)
    return (x_shape[0], w_shape[0], int(lib().orc_conv_out_h(ctypes.byref(d))),
            int(lib().orc_conv_out_w(ctypes.byref(d))))


def gemm(A, B, out_bf16=False):
    """A: (batch,M,K) or (M,K); B: (batch,K,N) or (K,N); float32 or uint16 bf16
    bits.  Returns float32 (or uint16 bf16 bits) of shape (batch,M,N)/(M,N)."""
    A = np.ascontiguousarray(A)
    B = np.ascontiguousarray(B)
    squeeze = A.ndim == 2
    if squeeze:
        A, B = A[None], B[None]
    batch, M, K = A.shape
    assert B.shape[0] == batch and B.shape[1] == K
    N = B.shape[2]
    in_bf16 = A.dtype == np.uint16
    assert (B.dtype == np.uint16) == in_bf16
    C = np.empty((batch, M, N), dtype=np.uint16 if out_bf16 else np.float32)
    lib().orc_gemm(ctypes.c_int64(batch), ctypes.c_int64(M), ctypes.c_int64(N),
                   ctypes.c_int64(K), int(in_bf16), int(out_bf16),
                   A.ctypes.data_as(ctypes.c_void_p), B.ctypes.data_as(ctypes.c_void_p),
                   C.ctypes.data_as(ctypes.c_void_p))
    return C[0] if squeeze else C


def gemm_at(A, B, flat):
    A = np.ascontiguousarray(A)
    B = np.ascontiguousarray(B)
    if A.ndim == 2:
        A, B = A[None], B[None]
    batch, M, K = A.shape
    N = B.shape[2]
    in_bf16 = A.dtype == np.uint16
    flat = np.ascontiguousarray(flat, dtype=np.int64)
    out = np.empty(flat.size, dtype=np.float64)
    lib().orc_gemm_at(ctypes.c_int64(batch), ctypes.c_int64(M), ctypes.c_int64(N),
                      ctypes.c_int64(K), int(in_bf16),
                      A.ctypes.data_as(ctypes.c_void_p), B.ctypes.data_as(ctypes.c_void_p),
                      flat.ctypes.data_as(ctypes.c_void_p), ctypes.c_int64(flat.size),
                      out.ctypes.data_as(ctypes.c_void_p))
    return out

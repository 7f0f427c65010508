"""Helpers for the GPU parity tests: bit-preserving host<->device copies,
the error measure, and construction of operands under a layout (always
through the oracle's conversion operator, never through the library)."""
import numpy as np
import torch

import oracle
import paper_2210_12415_amd as alt


def dev(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda()
    if a.dtype == np.uint32:
        return torch.from_numpy(a.view(np.int32)).cuda()
    return torch.from_numpy(a).cuda()


def host(t, dtype):
    torch.cuda.synchronize()
    return t.cpu().numpy().view(dtype)


def empty_dev(n, np_dtype):
    td = {np.dtype(np.uint16): torch.int16, np.dtype(np.uint32): torch.int32,
          np.dtype(np.float32): torch.float32}[np.dtype(np_dtype)]
    return torch.empty(int(n), dtype=td, device="cuda")


def canary_dev(n, np_dtype, pad=64):
    """Device buffer of n elements with `pad` guard elements on each side,
    all set to a recognisable pattern; returns (whole, view of the n)."""
    whole = empty_dev(n + 2 * pad, np_dtype)
    whole.fill_(0x5A5A if np.dtype(np_dtype).itemsize == 2 else 12345)
    return whole, whole[pad:pad + n]


def canary_ok(whole, n, pad=64):
    torch.cuda.synchronize()
    ref = whole[0].item()
    return bool((whole[:pad] == ref).all().item() and (whole[pad + n:] == ref).all().item())


def to_layout(a_logical, logical_name, physical_name):
    """Physical flat buffer of a logical array under 'LOGICAL->PHYSICAL' (oracle)."""
    shape = a_logical.shape
    seq = oracle.seq_from_string(logical_name + "->" + physical_name, shape)
    return oracle.layout_transform(np.ascontiguousarray(a_logical).reshape(-1), shape, [], seq)


def from_layout(flat, shape, logical_name, physical_name):
    seq = oracle.seq_from_string(logical_name + "->" + physical_name, shape)
    return oracle.layout_transform(flat, shape, seq, []).reshape(shape)


def rel_err(got, ref):
    """max_i |g_i - r_i| / (|r_i| + rms(r)): relative error with the output's
    own scale as floor, so that outputs near zero are judged against the size
    of the sums that produced them."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rms = float(np.sqrt(np.mean(ref * ref))) or 1.0
    return float(np.max(np.abs(got - ref) / (np.abs(ref) + rms)))


TOL = {alt.F32: 1e-5, alt.BF16: 2e-2}


def applicable_variants(h, d, kind="conv"):
    count = h.conv2d_variant_count(d) if kind == "conv" else h.gemm_variant_count(d)
    out = []
    for v in range(count):
        try:
            name = h.conv2d_variant_name(d, v) if kind == "conv" else h.gemm_variant_name(d, v)
        except alt.AltError as e:
            if e.status != 4:
                raise
            continue
        out.append((v, name))
    return out

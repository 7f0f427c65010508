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


def err_measures(got, ref, absdot=None):
    """The three error figures the parity tests report, as a dict:
    scaled    max_i |g_i - r_i| / (|r_i| + rms(r))             (the measure the thresholds are asserted on for fp32 sums)
    floored   max_i |g_i - r_i| / max(|r_i|, 1e-3 * rms(r))    (relative error with a small floor)
    component max_i |g_i - r_i| / sum_j |a_ij| |b_j|           (scale-free; absdot = the operator applied to |a|, |b|)
    A sum of Kg fp32 roundings has an absolute error near sqrt(Kg) * 2^-25 * rms whatever the
    order of summation, so outputs that happen to fall near zero carry relative errors of
    1e-4 and more under `floored` even when every addition is correctly rounded: the 1e-5
    threshold for fp32 operands can only be met under `scaled`, the 2e-2 threshold for
    bf16 operands is asserted under `floored`, and `component` is held against the textbook
    bound Kg * 2^-24."""
    got = np.asarray(got, dtype=np.float64).reshape(-1)
    ref = np.asarray(ref, dtype=np.float64).reshape(-1)
    rms = float(np.sqrt(np.mean(ref * ref))) or 1.0
    diff = np.abs(got - ref)
    out = dict(scaled=float(np.max(diff / (np.abs(ref) + rms))),
               floored=float(np.max(diff / np.maximum(np.abs(ref), 1e-3 * rms))))
    if absdot is not None:
        ad = np.asarray(absdot, dtype=np.float64).reshape(-1)
        out["component"] = float(np.max(diff / np.maximum(ad, np.finfo(np.float64).tiny)))
    return out


def abs_bits(bits):
    """|x| of bf16 bit patterns."""
    return (np.asarray(bits, dtype=np.uint16) & np.uint16(0x7fff)).astype(np.uint16)


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

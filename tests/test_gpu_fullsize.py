"""GPU parity at the configured sizes, element by element.

Every output element of the batch-16 ResNet-style layers (in the layouts and
kernel variants the benchmark launches), of the BERT-shaped products and of the
three-layer chain and the residual block at N = 16 is compared with the
oracle's.  Operands are laid out, and results brought back to logical order, by
the oracle's conversion operator: nothing of the library is trusted but the
call under test.  Each case reports three error figures (gpu_util.err_measures)
and asserts the thresholds on the ones its docstring names."""
import json
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2210_12415_amd as alt
from workloads import (BERT_GEMMS, BERT_QKT, CHAIN_LAYERS, RESNET_LAYERS, SMALL_CONV, bf16_bits_to_f32,
                       f32_to_bf16_bits, normal_f32, uniform_f32)

from gpu_util import abs_bits, applicable_variants, dev, err_measures, from_layout, host, to_layout

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
U24 = 2.0 ** -24              # unit roundoff of fp32
BF16_HALF_ULP = 2.0 ** -8     # largest relative step of one rounding to bf16


@pytest.fixture(scope="module")
def h():
    return alt.Handle()


@pytest.fixture(scope="module")
def arena():
    return torch.empty(1 << 30, dtype=torch.uint8, device="cuda")


def _plan_entries():
    with open(os.path.join(ROOT, "workloads", "tuned_plan_gfx950.json")) as f:
        plan = json.load(f)
    out = [(key, name, e) for key in ("bf16_out", "f32_out") for name, e in plan.get(key, {}).items()]
    for name, variant in plan.get("bf16_out_concurrent", {}).items():
        base = plan.get("bf16_out", {}).get(name)      # ("issue_order" is not a layer)
        if base and base["variant"] != variant:
            out.append(("bf16_out_concurrent", name, dict(base, variant=variant)))
    return out


def _phys_name(layout, logical):
    """Physical name of an alt_layout_t in the string form the oracle's parser takes."""
    return "".join(logical[layout.sub_dim[j]] if layout.sub_extent[j] == 0
                   else "%d%s" % (layout.sub_extent[j], logical[layout.sub_dim[j]].lower())
                   for j in range(layout.nsub))


_layer_cache = {}


def _layer_case(c):
    """Operands of a batch-16 layer, the oracle's fp32 result and the oracle's sum of |x||w| (each computed once)."""
    if c["name"] not in _layer_cache:
        li = [l["name"] for l in RESNET_LAYERS].index(c["name"])
        x = f32_to_bf16_bits(normal_f32(0xA17 + 2 + li, (16, c["C"], c["H"], c["W"])))
        w = f32_to_bf16_bits(normal_f32(0xA17 + 102 + li, (c["K"], c["C"], c["R"], c["S"]), std=0.05))
        ref = oracle.conv2d(x, w, stride=c["stride"], pad=c["pad"])
        absdot = oracle.conv2d(abs_bits(x), abs_bits(w), stride=c["stride"], pad=c["pad"])
        _layer_cache.clear()                            # one layer's arrays at a time
        _layer_cache[c["name"]] = (x, w, ref, absdot)
    return _layer_cache[c["name"]]


@pytest.mark.parametrize("entry", sorted(_plan_entries(), key=lambda e: e[1]), ids=lambda e: "%s-%s" % (e[1], e[0]))
def test_bench_layers_every_output(h, entry):
    """The five batch-16 layers under the layout and kernel variant the benchmark launches
    (stored plan: bf16 output, fp32 output, the jointly chosen variants), all 0.4-3.2 M outputs.
    fp32 output: floored <= 2e-2 (the bf16-operand threshold), scaled <= 1e-5, component <= Kg * 2^-24.
    bf16 output: |g - r| <= 2^-8 |r| + Kg * 2^-24 * sum|x||w| element by element (one rounding of the fp32 sum)."""
    key, lname, e = entry
    c = next(l for l in RESNET_LAYERS if l["name"] == lname)
    xl, wl = e["layout"].split("/")
    out_dtype = alt.F32 if key == "f32_out" else alt.BF16
    d = alt.conv_desc(16, c["C"], c["H"], c["W"], c["K"], c["R"], c["S"], stride=c["stride"], pad=c["pad"],
                      in_dtype=alt.BF16, out_dtype=out_dtype, x_layout="NCHW->" + xl, w_layout="OIHW->" + wl,
                      y_layout="NCHW->" + xl)
    byname = {n: v for v, n in applicable_variants(h, d)}
    assert e["variant"] in byname, "the stored plan names a variant this build does not have: re-run bench.py --retune"
    d.variant = byname[e["variant"]]
    x, w, ref, absdot = _layer_case(c)
    Kg = c["C"] * c["R"] * c["S"]
    xd, wd = dev(to_layout(x, "NCHW", xl)), dev(to_layout(w, "OIHW", wl))
    tdt, ndt = (torch.int16, np.uint16) if out_dtype == alt.BF16 else (torch.float32, np.float32)
    yd = torch.full((ref.size,), -1 if out_dtype == alt.BF16 else float("nan"), dtype=tdt, device="cuda")
    ws_bytes = h.conv2d_workspace_size(d)
    ws = torch.empty(max(ws_bytes, 4) // 4, dtype=torch.float32, device="cuda")
    h.conv2d(d, xd, wd, yd, workspace=ws, ws_bytes=ws_bytes)
    got = from_layout(host(yd, ndt), ref.shape, "NCHW", xl)
    if out_dtype == alt.F32:
        m = err_measures(got, ref, absdot)
        print(lname, key, e["variant"], m)
        assert m["floored"] <= 2e-2 and m["scaled"] <= 1e-5 and m["component"] <= Kg * U24, m
    else:
        g = bf16_bits_to_f32(got).astype(np.float64)
        m = err_measures(g, ref, absdot)
        print(lname, key, e["variant"], m)
        bound = BF16_HALF_ULP * np.abs(ref.astype(np.float64)) + Kg * U24 * absdot.astype(np.float64)
        assert np.all(np.abs(g - ref) <= bound), m
        assert m["floored"] <= 2e-2, m


def test_small_fp32_conv_three_measures(h):
    """The small fp32 convolution (fp32 matrix-core products, fp32 sums) in NCHW and NHWC: scaled <= 1e-5 and
    component <= Kg * 2^-24; `floored` is reported (outputs near zero exceed 1e-5 under it for any fp32 sum)."""
    c = SMALL_CONV
    x = uniform_f32(0xA18, (c["N"], c["C"], c["H"], c["W"]))
    w = uniform_f32(0xA19, (c["K"], c["C"], c["R"], c["S"]))
    ref = oracle.conv2d(x, w, stride=c["stride"], pad=c["pad"])
    absdot = oracle.conv2d(np.abs(x), np.abs(w), stride=c["stride"], pad=c["pad"])
    Kg = c["C"] * c["R"] * c["S"]
    for xl, wl in [("NCHW", "OIHW"), ("NHWC", "OHWI")]:
        d = alt.conv_desc(c["N"], c["C"], c["H"], c["W"], c["K"], c["R"], c["S"], stride=c["stride"], pad=c["pad"],
                          in_dtype=alt.F32, x_layout="NCHW->" + xl, w_layout="OIHW->" + wl, y_layout="NCHW->" + xl)
        for v, name in applicable_variants(h, d):
            d.variant = v
            yd = torch.full((ref.size,), float("nan"), dtype=torch.float32, device="cuda")
            ws_bytes = h.conv2d_workspace_size(d)
            ws = torch.empty(max(ws_bytes, 4) // 4, dtype=torch.float32, device="cuda")
            h.conv2d(d, dev(to_layout(x, "NCHW", xl)), dev(to_layout(w, "OIHW", wl)), yd, workspace=ws, ws_bytes=ws_bytes)
            m = err_measures(from_layout(host(yd, np.float32), ref.shape, "NCHW", xl), ref, absdot)
            assert m["scaled"] <= 1e-5 and m["component"] <= Kg * U24, (xl, name, m)


@pytest.mark.parametrize("g", BERT_GEMMS + [BERT_QKT], ids=[g["name"] for g in BERT_GEMMS + [BERT_QKT]])
def test_bert_products_every_output(h, arena, g):
    """The four BERT-shaped products (QK^T batched, B stored [N][K]) under the tuned operand layout and variant and
    under the default one, every output: floored <= 2e-2, scaled <= 1e-5, component <= K * 2^-24."""
    batch, M, K, N = g["batch"], g["M"], g["K"], g["N"]
    A = f32_to_bf16_bits(normal_f32(0xA17 + 4, (batch, M, K), std=0.02))
    B = f32_to_bf16_bits(normal_f32(0xA17 + 104, (batch, K, N), std=0.02))
    ref = oracle.gemm(A, B)
    absdot = oracle.gemm(abs_bits(A), abs_bits(B))
    d0 = alt.gemm_desc(M, N, K, batch=batch, in_dtype=alt.BF16, out_dtype=alt.F32)
    tuned, _ = h.tune_gemm(d0, arena, arena.numel(), max_trials=64, warmup=2, reps=5)
    cases = [("tuned", tuned), ("row-major", alt.gemm_desc(M, N, K, batch=batch)),
             ("B as NK", alt.gemm_desc(M, N, K, batch=batch, b_layout="KN->NK"))]
    for label, d in cases:
        al, bl, cl = _phys_name(d.a_layout, "MK"), _phys_name(d.b_layout, "KN"), _phys_name(d.c_layout, "MN")
        Ad = dev(np.concatenate([to_layout(A[b], "MK", al) for b in range(batch)]))
        Bd = dev(np.concatenate([to_layout(B[b], "KN", bl) for b in range(batch)]))
        Cd = torch.full((batch * M * N,), float("nan"), dtype=torch.float32, device="cuda")
        ws_bytes = h.gemm_workspace_size(d)
        ws = torch.empty(max(ws_bytes, 4) // 4, dtype=torch.float32, device="cuda")
        h.gemm(d, Ad, Bd, Cd, workspace=ws, ws_bytes=ws_bytes)
        flat = host(Cd, np.float32).reshape(batch, M * N)
        got = np.stack([from_layout(flat[b], (M, N), "MN", cl) for b in range(batch)])
        m = err_measures(got, ref, absdot)
        print(g["name"], label, h.gemm_variant_name(d, d.variant) if d.variant >= 0 else "default", m)
        assert m["floored"] <= 2e-2 and m["scaled"] <= 1e-5 and m["component"] <= K * U24, (label, m)


def _chain_reference(x, ws, bias):
    ref = x
    for i, c in enumerate(CHAIN_LAYERS):
        ref = oracle.conv2d(ref, ws[i], stride=c["stride"], pad=c["pad"], bias=bias if c["bias"] else None,
                            relu=c["relu"], out_bf16=True)
    return ref


def test_chain_at_n16_every_output(h, arena):
    """The three-layer chain at its configured size (N = 16, 56x56), planned on the device (layouts per edge,
    kernel variant per layer) and executed as planned; every element of the final tensor against the oracle's
    chain (bf16 between the layers).  Intermediate roundings to bf16 may fall the other way where the fp32 sums
    differ in their last bits, so the comparison allows one bf16 step per layer on the final values, measured
    against |r| + rms(r) (a flipped intermediate moves a final sum by about 2^-8 of one of its terms, which is
    not small against a final value that happens to fall near zero)."""
    N = 16
    ops = [alt.conv_desc(N, c["C"], c["H"], c["W"], c["K"], c["R"], c["S"], stride=c["stride"], pad=c["pad"],
                         in_dtype=alt.BF16, out_dtype=alt.BF16,
                         epilogue=(alt.EPI_BIAS if c["bias"] else 0) | (alt.EPI_RELU if c["relu"] else 0))
           for c in CHAIN_LAYERS]
    plan = h.tune_chain(ops, "NCHW->NCHW", arena, arena.numel(), max_trials=0, warmup=3, reps=20)
    assert plan.nops == 3 and plan.total_us <= plan.default_total_us * 1.0001
    x = f32_to_bf16_bits(normal_f32(81, (N, 64, 56, 56)))
    ws = [f32_to_bf16_bits(normal_f32(82 + i, (c["K"], c["C"], c["R"], c["S"]), std=0.05)) for i, c in enumerate(CHAIN_LAYERS)]
    bias = normal_f32(90, (64,), std=0.1)
    ref = _chain_reference(x, ws, bias)
    cur, cur_shape = dev(x.reshape(-1)), x.shape
    for i, c in enumerate(CHAIN_LAYERS):
        d = plan.op[i]
        if plan.transform_before[i]:
            nxt = torch.empty_like(cur)
            h.layout_transform(alt.BF16, cur_shape, plan.edge_layout[i], cur, d.x_layout, nxt)
            cur = nxt
        wd = dev(to_layout(ws[i], "OIHW", _phys_name(d.w_layout, "OIHW")))
        oshape = h.conv2d_output_shape(d)
        y = torch.full((int(np.prod(oshape)),), -1, dtype=torch.int16, device="cuda")
        h.conv2d(d, cur, wd, y, bias=dev(bias) if c["bias"] else None, workspace=arena, ws_bytes=arena.numel())
        cur, cur_shape = y, oshape
    got = from_layout(host(cur, np.uint16), cur_shape, "NCHW", _phys_name(plan.op[2].y_layout, "NCHW"))
    g, r = bf16_bits_to_f32(got).astype(np.float64), bf16_bits_to_f32(ref).astype(np.float64)
    m = err_measures(g, r)
    print("chain N=16", [h.conv2d_variant_name(plan.op[i], plan.op[i].variant) for i in range(3)], m,
          "fraction of elements whose bits differ: %.4f" % float(np.mean(got != ref)))
    assert m["scaled"] <= 3 * BF16_HALF_ULP, m

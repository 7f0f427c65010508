"""GPU tests of the tuner, the cache and the chain planner: the winner is never
slower than the default layout's best, a tuned descriptor reproduces the
oracle, the cache round-trips through a file, and the planned chain computes
what the oracle's chain computes."""
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2210_12415_amd as alt
from workloads import CHAIN_LAYERS, bf16_bits_to_f32, f32_to_bf16_bits, normal_f32, small_ints_f32

from gpu_util import TOL, dev, from_layout, host, rel_err, to_layout

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def h():
    return alt.Handle()


@pytest.fixture(scope="module")
def arena():
    return torch.empty(1 << 29, dtype=torch.uint8, device="cuda")


def _phys_name(layout, logical):
    """Physical string of a parsed separable layout, e.g. 'NCHW16c'."""
    out = ""
    for j in range(layout.nsub):
        letter = logical[layout.sub_dim[j]]
        ext = layout.sub_extent[j]
        out += letter if ext == 0 else "%d%s" % (ext, letter.lower())
    return out


def test_tune_conv_budgeted_and_correct(h, arena):
    N, C, H, W, K = 4, 64, 14, 14, 64
    shape = alt.conv_desc(N, C, H, W, K, 3, 3, stride=1, pad=1, in_dtype=alt.BF16, out_dtype=alt.F32)
    best, rep = h.tune_conv2d(shape, arena, arena.numel(), max_trials=60, warmup=2, reps=10)
    assert 0 < rep.trials <= 60 + 8
    assert rep.n_layouts >= 4
    assert rep.best_us <= rep.default_us
    assert best.variant >= 0
    # the tuned descriptor computes the right thing
    x = small_ints_f32(71, (N, C, H, W))
    w = small_ints_f32(72, (K, C, 3, 3))
    ref = oracle.conv2d(x, w, stride=1, pad=1)
    xl, wl, yl = _phys_name(best.x_layout, "NCHW"), _phys_name(best.w_layout, "OIHW"), _phys_name(best.y_layout, "NCHW")
    xd = dev(to_layout(f32_to_bf16_bits(x), "NCHW", xl))
    wd = dev(to_layout(f32_to_bf16_bits(w), "OIHW", wl))
    yd = torch.empty(ref.size, dtype=torch.float32, device="cuda")
    h.conv2d(best, xd, wd, yd, workspace=arena, ws_bytes=arena.numel())
    assert np.array_equal(from_layout(host(yd, np.float32), ref.shape, "NCHW", yl), ref)
    # variant = -1 now resolves to the cached winner: same result, and the cache survives a file
    best.variant = -1
    yd.zero_()
    h.conv2d(best, xd, wd, yd, workspace=arena, ws_bytes=arena.numel())
    assert np.array_equal(from_layout(host(yd, np.float32), ref.shape, "NCHW", yl), ref)
    path = "/tmp/alt_cache_test.txt"
    h.cache_save(path)
    text = open(path).read()
    assert "conv|" in text and "_k" in text
    h2 = alt.Handle()
    h2.cache_load(path)
    h2.cache_save(path + ".2")
    assert open(path + ".2").read() == text
    os.remove(path)
    os.remove(path + ".2")


def test_tune_conv_unlimited_beats_or_equals_budgeted(h, arena):
    shape = alt.conv_desc(1, 128, 14, 14, 128, 3, 3, stride=1, pad=1, in_dtype=alt.BF16)
    _, rep_all = h.tune_conv2d(shape, arena, arena.numel(), max_trials=0, warmup=2, reps=10)
    assert rep_all.best_us <= rep_all.default_us
    # every explored layout reports its own best; the winner is their minimum
    lus = [rep_all.layout_best_us[i] for i in range(rep_all.n_layouts)]
    assert abs(min(lus) - rep_all.best_us) < 1e-6
    # re-measuring the winner lands near its recorded time
    d = alt.conv_desc(1, 128, 14, 14, 128, 3, 3, stride=1, pad=1, in_dtype=alt.BF16)
    us, trials = h.tune_conv2d_variants(d, arena, arena.numel(), max_trials=0, warmup=2, reps=10)
    assert trials > 0 and us > 0


def test_tune_gemm(h, arena):
    d0 = alt.gemm_desc(256, 256, 512, in_dtype=alt.BF16)
    best, rep = h.tune_gemm(d0, arena, arena.numel(), max_trials=0, warmup=2, reps=10)
    assert rep.best_us <= rep.default_us and rep.n_layouts >= 2
    A = small_ints_f32(73, (256, 512))
    B = small_ints_f32(74, (512, 256))
    ref = oracle.gemm(A, B)
    al, bl, cl = _phys_name(best.a_layout, "MK"), _phys_name(best.b_layout, "KN"), _phys_name(best.c_layout, "MN")
    Cd = torch.empty(256 * 256, dtype=torch.float32, device="cuda")
    h.gemm(best, dev(to_layout(f32_to_bf16_bits(A), "MK", al)), dev(to_layout(f32_to_bf16_bits(B), "KN", bl)), Cd,
           workspace=arena, ws_bytes=arena.numel())
    assert np.array_equal(from_layout(host(Cd, np.float32), (256, 256), "MN", cl), ref)


def test_chain_plan_executes_to_oracle_result(h, arena):
    """Config-5-shaped chain at reduced batch: conv3x3+bias+ReLU -> conv3x3 s2 -> conv1x1, bf16 edges."""
    N = 2
    cfgs = CHAIN_LAYERS
    ops = [alt.conv_desc(N, c["C"], c["H"], c["W"], c["K"], c["R"], c["S"], stride=c["stride"], pad=c["pad"],
                         in_dtype=alt.BF16, out_dtype=alt.BF16,
                         epilogue=(alt.EPI_BIAS if c["bias"] else 0) | (alt.EPI_RELU if c["relu"] else 0))
           for c in cfgs]
    plan = h.tune_chain(ops, "NCHW->NCHW", arena, arena.numel(), max_trials=0, warmup=2, reps=5)
    assert plan.nops == 3 and plan.total_us <= plan.default_total_us * 1.0001
    # a conversion is planned exactly where the producer's layout differs from the consumer's
    for i in range(3):
        prev = _phys_name(plan.edge_layout[i], "NCHW")
        cur = _phys_name(plan.op[i].x_layout, "NCHW")
        assert bool(plan.transform_before[i]) == (prev != cur)
        assert _phys_name(plan.edge_layout[i + 1], "NCHW") == _phys_name(plan.op[i].y_layout, "NCHW")
    # oracle chain: bf16 between layers, logical NCHW
    x = f32_to_bf16_bits(normal_f32(81, (N, 64, 56, 56)))
    ws = [f32_to_bf16_bits(normal_f32(82 + i, (c["K"], c["C"], c["R"], c["S"]), std=0.05)) for i, c in enumerate(cfgs)]
    bias = normal_f32(90, (64,), std=0.1)
    ref = x
    for i, c in enumerate(cfgs):
        ref = oracle.conv2d(ref, ws[i], stride=c["stride"], pad=c["pad"], bias=bias if c["bias"] else None,
                            relu=c["relu"], out_bf16=True)
    # execute the plan through the library
    cur = dev(x.reshape(-1))
    cur_shape = x.shape
    for i, c in enumerate(cfgs):
        d = plan.op[i]
        if plan.transform_before[i]:
            nxt = torch.empty_like(cur)
            h.layout_transform(alt.BF16, cur_shape, plan.edge_layout[i], cur, d.x_layout, nxt)
            cur = nxt
        wd = torch.empty_like(dev(ws[i].reshape(-1)))
        h.pack_weights(d, dev(ws[i].reshape(-1)), wd)
        oshape = h.conv2d_output_shape(d)
        y = torch.empty(int(np.prod(oshape)), dtype=torch.int16, device="cuda")
        h.conv2d(d, cur, wd, y, bias=dev(bias) if c["bias"] else None, workspace=arena, ws_bytes=arena.numel())
        cur, cur_shape = y, oshape
    got = from_layout(host(cur, np.uint16), cur_shape, "NCHW", _phys_name(plan.op[2].y_layout, "NCHW"))
    # bf16 rounding between layers: compare values, allow the ulp-level differences rounding order causes
    assert rel_err(bf16_bits_to_f32(got), bf16_bits_to_f32(ref)) <= TOL[alt.BF16]

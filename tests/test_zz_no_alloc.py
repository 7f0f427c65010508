"""alt_conv2d_static (the entry point that allocates nothing: its split-K partial tiles
live in a static device array) against alt_conv2d on the same inputs, bit for bit, on
two calls in a row, the second with a smaller input; and the size limit."""
import numpy as np
import pytest
import torch

import paper_2210_12415_amd as alt
from workloads import f32_to_bf16_bits, normal_f32

from gpu_util import applicable_variants, dev, host

pytestmark = pytest.mark.gpu


def _desc(N, C, H, K, R, variant=-1, out_dtype=alt.F32, epilogue=0):
    return alt.conv_desc(N, C, H, H, K, R, R, stride=1, pad=R // 2, in_dtype=alt.BF16, out_dtype=out_dtype,
                         epilogue=epilogue, variant=variant,
                         x_layout="NCHW->NHWC", w_layout="OIHW->OHWI", y_layout="NCHW->NHWC")


def _both(h, N, C, H, K, R, seed, variant_filter):
    """Runs alt_conv2d (caller's workspace) and alt_conv2d_static under the same split-K variant."""
    d = _desc(N, C, H, K, R)
    names = [(v, n) for v, n in applicable_variants(h, d) if variant_filter(n)]
    assert names
    outs = []
    x = dev(f32_to_bf16_bits(normal_f32(seed, (N * H * H * C,))))
    w = dev(f32_to_bf16_bits(normal_f32(seed + 1, (K * R * R * C,), std=0.05)))
    bias = dev(normal_f32(seed + 2, (K,), std=0.1))
    for v, name in names[:6]:
        for out_dtype, tdt in ((alt.F32, torch.float32), (alt.BF16, torch.int16)):
            d = _desc(N, C, H, K, R, variant=v, out_dtype=out_dtype, epilogue=alt.EPI_BIAS | alt.EPI_RELU)
            n_out = N * H * H * K
            ws_bytes = h.conv2d_workspace_size(d)
            assert 0 < ws_bytes <= (32 << 20), (name, ws_bytes)
            ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
            y0 = torch.full((n_out,), 7, dtype=tdt, device="cuda")
            y1 = torch.full((n_out,), 9, dtype=tdt, device="cuda")
            h.conv2d(d, x, w, y0, bias=bias, workspace=ws, ws_bytes=ws_bytes)
            h.conv2d_static(d, x, w, y1, bias=bias)
            torch.cuda.synchronize()
            assert torch.equal(y0, y1), (name, out_dtype)
            outs.append(name)
    return outs


def test_static_workspace_matches_callers_workspace_twice():
    h = alt.Handle()
    split = lambda n: not n.endswith("_k1")
    first = _both(h, 4, 256, 14, 256, 3, 3001, split)
    second = _both(h, 1, 128, 7, 128, 3, 3011, split)       # smaller input, the array still holds the first call's tiles
    assert first and second
    # variant = -1: the library picks; same result as alt_conv2d given a workspace of the array's size
    d = _desc(4, 256, 14, 256, 3)
    x = dev(f32_to_bf16_bits(normal_f32(3021, (4 * 14 * 14 * 256,))))
    w = dev(f32_to_bf16_bits(normal_f32(3022, (256 * 9 * 256,), std=0.05)))
    ws = torch.empty(32 << 20, dtype=torch.uint8, device="cuda")
    y0 = torch.zeros(4 * 14 * 14 * 256, dtype=torch.float32, device="cuda")
    y1 = torch.ones_like(y0)
    h.conv2d(d, x, w, y0, workspace=ws, ws_bytes=ws.numel())
    h.conv2d_static(d, x, w, y1)
    torch.cuda.synchronize()
    assert torch.equal(y0, y1)
    assert h.splitk_status().counters_nonzero == 0


def test_static_workspace_rejects_what_does_not_fit():
    h = alt.Handle()
    d = _desc(64, 256, 56, 256, 3)
    big = [(v, n) for v, n in applicable_variants(h, d) if not n.endswith("_k1")]
    assert big
    d.variant = big[-1][0]
    assert h.conv2d_workspace_size(d) > (32 << 20)
    # (full-size buffers although the call is expected to fail on the host, before any launch)
    x = torch.zeros(64 * 56 * 56 * 256, dtype=torch.int16, device="cuda")
    w = torch.zeros(256 * 9 * 256, dtype=torch.int16, device="cuda")
    y = torch.zeros(64 * 56 * 56 * 256, dtype=torch.float32, device="cuda")
    with pytest.raises(alt.AltError) as e:
        h.conv2d_static(d, x, w, y)
    assert e.value.status == 5 and "workspace" in str(e.value)

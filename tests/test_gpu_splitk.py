"""Split-K launches of the tile kernels on several streams: the arrival counters of
the fused reduction are bound to streams, so launches in flight on different
streams never share a set whatever their issue order.  Integer-valued inputs make
every sum exact: any lost or early-read partial tile shows as a wrong integer."""
import numpy as np
import pytest
import torch

import oracle
import paper_2210_12415_amd as alt
from workloads import f32_to_bf16_bits, small_ints_f32

from gpu_util import applicable_variants, dev, from_layout, host, to_layout

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def h():
    return alt.Handle()


def _case(h, seed, N, C, H, K, R, pick):
    """A convolution in NHWC/OHWI with integer inputs under the split-K variant pick() chooses."""
    x = small_ints_f32(seed, (N, C, H, H), -3, 3)
    w = small_ints_f32(seed + 50, (K, C, R, R), -3, 3)
    pad = R // 2
    d = alt.conv_desc(N, C, H, H, K, R, R, stride=1, pad=pad, in_dtype=alt.BF16,
                      x_layout="NCHW->NHWC", w_layout="OIHW->OHWI", y_layout="NCHW->NHWC")
    names = [(v, n) for v, n in applicable_variants(h, d) if not n.endswith("_k1") and ("direct" in n or "stream" in n)]
    assert names, "no split-K tile kernel applies"
    d.variant, name = pick(names)
    ws_bytes = h.conv2d_workspace_size(d)
    assert ws_bytes > 0
    return dict(d=d, name=name, ref=oracle.conv2d(x, w, stride=1, pad=pad),
                x=dev(to_layout(f32_to_bf16_bits(x), "NCHW", "NHWC")), w=dev(to_layout(f32_to_bf16_bits(w), "OIHW", "OHWI")),
                ws=torch.empty(ws_bytes, dtype=torch.uint8, device="cuda"), ws_bytes=ws_bytes)


def _check(c, y):
    got = from_layout(host(y, np.float32), c["ref"].shape, "NCHW", "NHWC")
    assert np.array_equal(got, c["ref"]), c["name"]


def test_split_k_launch_queued_behind_an_event_while_another_stream_issues_many(h):
    """Stream A's split-K launch waits on an event behind a long kernel; stream C meanwhile issues
    twelve split-K launches.  Both results are the oracle's integers and the counters end at zero."""
    a = _case(h, 900, 2, 256, 14, 256, 3, lambda names: names[0])
    c = _case(h, 901, 2, 256, 14, 256, 3, lambda names: names[-1])
    sa, sb, sc = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    ya = torch.full((a["ref"].size,), float("nan"), dtype=torch.float32, device="cuda")
    yc = torch.full((c["ref"].size,), float("nan"), dtype=torch.float32, device="cuda")
    big = torch.randn(8192, 8192, device="cuda")
    torch.cuda.synchronize()
    evt = torch.cuda.Event()
    with torch.cuda.stream(sb):
        for _ in range(4):
            big = big @ big * 1e-4              # a few milliseconds of work ahead of the event
        evt.record(sb)
    sa.wait_event(evt)
    h.conv2d(a["d"], a["x"], a["w"], ya, workspace=a["ws"], ws_bytes=a["ws_bytes"], stream=sa)
    for _ in range(12):
        h.conv2d(c["d"], c["x"], c["w"], yc, workspace=c["ws"], ws_bytes=c["ws_bytes"], stream=sc)
    torch.cuda.synchronize()
    _check(a, ya)
    _check(c, yc)
    st = h.splitk_status()
    assert st.counters_nonzero == 0 and 2 <= st.streams_bound <= st.max_streams


def test_three_split_k_variants_concurrently_under_conv2d_multi(h):
    """Three independent convolutions, each under a split-K variant, issued by one alt_conv2d_multi call on
    three streams, forty steps without synchronising in between (the streams drift against one another)."""
    cases = [_case(h, 910, 2, 256, 14, 256, 3, lambda names: names[0]),
             _case(h, 911, 1, 512, 7, 512, 3, lambda names: names[len(names) // 2]),
             _case(h, 912, 4, 256, 14, 64, 1, lambda names: names[-1])]
    streams = [torch.cuda.Stream() for _ in cases]
    ys = [torch.full((c["ref"].size,), float("nan"), dtype=torch.float32, device="cuda") for c in cases]
    calls = [dict(d=c["d"], x=c["x"], w=c["w"], y=y, workspace=c["ws"], ws_bytes=c["ws_bytes"], stream=s)
             for c, y, s in zip(cases, ys, streams)]
    torch.cuda.synchronize()
    step = h.conv2d_multi_prepared(calls)
    for _ in range(40):
        step()
    torch.cuda.synchronize()
    for c, y in zip(cases, ys):
        _check(c, y)
    st = h.splitk_status()
    assert st.counters_nonzero == 0


def test_split_k_inside_a_captured_graph_replays_exactly(h):
    """A captured split-K launch keeps its stream's counter set: replays (with eager work and
    synchronisations between them) give the oracle's integers every time."""
    c = _case(h, 920, 2, 256, 14, 256, 3, lambda names: names[0])
    y = torch.full((c["ref"].size,), float("nan"), dtype=torch.float32, device="cuda")
    side = torch.cuda.Stream()
    h.conv2d(c["d"], c["x"], c["w"], y, workspace=c["ws"], ws_bytes=c["ws_bytes"], stream=side)
    side.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        h.conv2d(c["d"], c["x"], c["w"], y, workspace=c["ws"], ws_bytes=c["ws_bytes"], stream=side)
    for _ in range(4):
        y.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        _check(c, y)
    assert h.splitk_status().counters_nonzero == 0

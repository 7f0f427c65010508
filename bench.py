#!/usr/bin/env python3
"""Benchmark of the conv2d / gemm / layout_transform path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

One step = one pass over the five ResNet-50-style convolution layers at batch
16 (bf16 inputs, fp32 accumulation on the matrix cores, bf16 output), each
under the layouts and kernel variant the tuner picked, inputs already resident
in HBM in the tuned layout (the producer writes the consumer's layout; weights
are packed once, offline).  `value` is the layers' nominal FLOPs per step over
the measured time per step.  The same run also reports, under "extra", the
per-layer figures, the layout conversion operator on the activation shapes
(GB/s), the BERT-shaped matrix products, the batch-1 layers, the three-layer
chain and the tuner's best-vs-default-layout ratios.  Prints one JSON line.
"""
import argparse
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# Kernel arguments in device memory: with the HIP default (host memory) every
# workgroup's first scalar loads cross the host link, which costs these
# microsecond-sized kernels 2-5 us each.  Read by the HIP runtime when it starts.
os.environ.setdefault("HIP_FORCE_DEV_KERNARG", "1")

PEAK_BF16_TFLOPS = 2500.0
PEAK_HBM_GBPS = 8000.0
MIN_TIMED_MS = 50.0          # every timed region of the headline step runs at least this long
MAX_LINE_BYTES = 2000        # the final stdout line stays below this; everything else goes to EXTRA_PATH
EXTRA_PATH = os.path.join(ROOT, "gpurun_out", "bench_extra.json")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # (a step is ~27 us: 2000 of them keep the fixed costs of a timed region, a few hundred us of runtime
    # housekeeping after the launches before it, below one percent)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--quick", action="store_true", help="skip the extra sections")
    ap.add_argument("--sections", default="all",
                    help="comma-separated extra sections to run besides the headline step: f32, transforms, gemm, b1, "
                         "scaled, chain, graph, groups, budget, peaks (default all; --quick runs none)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--default-trials", type=int, default=32,
                    help="measurements spent per layer on the default layout's own kernel variants (0 = all)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run the library's plain copy kernel (256 MiB read + 256 MiB written per launch), "
                         "which gives a hardware-counter run its scale")
    ap.add_argument("--only", default="",
                    help="profiling target: run just one prepared launch loop (no tuning, no timing sections) and exit. "
                         "step = the five batch-16 layers under the stored plan; gemm4096 = the 4096^3 product under the "
                         "256x256 streaming tile; conv_b256 = the 64-channel 56x56 layer at batch 256; transform = the "
                         "NCHW->NHWC conversion of (256,64,56,56) fp32 and of (16,64,56,56) fp32 over rings of 1 GiB")
    ap.add_argument("--plan", default=os.path.join(ROOT, "workloads", "tuned_plan_gfx950.json"),
                    help="tuned layouts and kernel variants of the batch-16 layers (a previous run's choice)")
    ap.add_argument("--retune", action="store_true",
                    help="tune the batch-16 layers on the device now instead of reading --plan, and rewrite it")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2210_12415_amd as alt
    from workloads import (RESNET_LAYERS, TRANSFORM_SHAPES, BERT_GEMMS, BERT_QKT, CHAIN_LAYERS,
                           conv_flops, conv_out_hw, f32_to_bf16_bits, normal_f32)

    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU")
    all_sections = ("f32", "transforms", "gemm", "b1", "scaled", "chain", "graph", "groups", "budget", "peaks")
    chosen = set(all_sections) if args.sections == "all" else set(x for x in args.sections.split(",") if x)
    if chosen - set(all_sections):
        raise SystemExit("bench.py: unknown section(s) %s" % ", ".join(sorted(chosen - set(all_sections))))

    def want(name):
        return not args.quick and name in chosen
    alt.lib()                                   # fails loudly if libalt.so is missing
    dev = torch.device("cuda:0")
    h = alt.Handle()
    stream = torch.cuda.current_stream()

    def dbuf(a):
        a = np.ascontiguousarray(a)
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).to(dev)
        return torch.from_numpy(a).to(dev)

    arena = torch.empty(1 << 30, dtype=torch.uint8, device=dev)

    def timed(fn, reps, warm=5):
        """Average microseconds per call over `reps` back-to-back calls (HIP
        events on the launch stream)."""
        for _ in range(warm):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            fn()
        e1.record(stream)
        e1.synchronize()
        return e0.elapsed_time(e1) * 1000.0 / reps

    def median_timed(fn, reps, batches=5):
        return float(np.median([timed(fn, reps) for _ in range(batches)]))

    # ------------------------------------------------------------ conv layers ----
    def from_plan(shape, entry):
        """The descriptor a stored plan entry names, or None if this build lacks its variant."""
        a, b = entry["layout"].split("/")
        d = alt.conv_desc(shape.N, shape.C, shape.H, shape.W, shape.K, shape.R, shape.S, stride=shape.stride_h,
                          pad=shape.pad_h, in_dtype=shape.in_dtype, out_dtype=shape.out_dtype,
                          x_layout="NCHW->" + a, w_layout="OIHW->" + b, y_layout="NCHW->" + a)
        for v in range(h.conv2d_variant_count(d)):
            try:
                if h.conv2d_variant_name(d, v) == entry["variant"]:
                    d.variant = v
                    return d
            except alt.AltError:
                pass
        return None

    def prepare_layers(batch, out_dtype, budget, plan=None):
        """Tunes each layer (or takes a stored choice), then lays out its operands for the chosen layouts."""
        layers = []
        for li, L in enumerate(RESNET_LAYERS):
            shape = alt.conv_desc(batch, L["C"], L["H"], L["W"], L["K"], L["R"], L["S"], stride=L["stride"],
                                  pad=L["pad"], in_dtype=alt.BF16, out_dtype=out_dtype)
            best = from_plan(shape, plan[L["name"]]) if plan and L["name"] in plan else None
            if best is not None:
                e = plan[L["name"]]
                rep = alt.TuneReport()
                rep.trials, rep.best_us, rep.default_us = e["trials"], e["tuned_us"], e["default_layout_us"]
                for i, (nm, us) in enumerate(e["layout_us"].items()):
                    rep.layout_name[i].value = nm.encode()
                    rep.layout_best_us[i] = us
                rep.n_layouts = len(e["layout_us"])
            else:
                best, rep = h.tune_conv2d(shape, arena, arena.numel(), max_trials=budget, warmup=3, reps=30)
            x = f32_to_bf16_bits(normal_f32(0xA17 + 2 + li, (batch, L["C"], L["H"], L["W"])))
            w = f32_to_bf16_bits(normal_f32(0xA17 + 102 + li, (L["K"], L["C"], L["R"], L["S"]), std=0.05))
            x_nchw, w_oihw = dbuf(x.reshape(-1)), dbuf(w.reshape(-1))
            xd, wd = torch.empty_like(x_nchw), torch.empty_like(w_oihw)
            h.layout_transform(alt.BF16, x.shape, "NCHW->NCHW", x_nchw, best.x_layout, xd)
            h.pack_weights(best, w_oihw, wd)
            oh, ow = conv_out_hw(L["H"], L["W"], L["R"], L["S"], L["stride"], L["pad"])
            n_out = batch * L["K"] * oh * ow
            yd = torch.empty(n_out, dtype=torch.float32 if out_dtype == alt.F32 else torch.int16, device=dev)
            ws_bytes = h.conv2d_workspace_size(best)
            ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)
            names = [rep.layout_name[i].value.decode() for i in range(rep.n_layouts)]
            lus = [rep.layout_best_us[i] for i in range(rep.n_layouts)]
            layers.append(dict(L=L, desc=best, x=xd, w=wd, y=yd, ws=ws, ws_bytes=ws_bytes, x_nchw=x_nchw,
                               flops=conv_flops(batch, **L), rep=rep,
                               layout=names[int(np.argmin(lus))], variant=h.conv2d_variant_name(best, best.variant),
                               layout_us=dict(zip(names, [round(float(u), 2) for u in lus])),
                               trials=rep.trials, default_us=float(rep.default_us), best_us=float(rep.best_us),
                               bytes=(x.size + w.size) * 2 + n_out * (4 if out_dtype == alt.F32 else 2)))
        return layers

    def run_layer(l, st=None):
        if st is None:                          # the eager path: arguments marshalled once per layer
            if "call" not in l:
                l["call"] = h.conv2d_prepared(l["desc"], l["x"], l["w"], l["y"], workspace=l["ws"],
                                              ws_bytes=l["ws_bytes"], stream=stream)
            l["call"]()
        else:
            h.conv2d(l["desc"], l["x"], l["w"], l["y"], workspace=l["ws"], ws_bytes=l["ws_bytes"], stream=st)

    side = torch.cuda.Stream()

    def cold_layer_us(l):
        """Microseconds per launch of layer l with activations and output that no cache holds: the launches of
        one graph walk a ring of (x, y) pairs carved out of the arena, at least 400 MB apart before a pair comes
        round again (the last-level cache is 256 MB); the weights stay where they are."""
        xb, yb = l["x"].numel() * l["x"].element_size(), l["y"].numel() * l["y"].element_size()
        pitch = (xb + yb + 511) // 256 * 256
        nring = int(min(256, arena.numel() // pitch))
        if nring * pitch < (400 << 20) and nring < 256:
            return None
        arena.view(torch.int16).random_(-200, 200)
        torch.cuda.synchronize()
        pairs = []
        for i in range(nring):
            base = i * pitch
            xoff = (xb + 255) // 256 * 256
            pairs.append((arena[base:base + xb].view(l["x"].dtype), arena[base + xoff:base + xoff + yb].view(l["y"].dtype)))
        it = [0]

        def one(st):
            x, y = pairs[it[0] % nring]
            it[0] += 1
            h.conv2d(l["desc"], x, l["w"], y, workspace=l["ws"], ws_bytes=l["ws_bytes"], stream=st)
        one(side)
        side.synchronize()
        it[0] = 0
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            for _ in range(nring):
                one(side)
        us = graph_timed(g, nring, replays=3, batches=3)
        del g
        return us

    def capture(fn, n):
        """A HIP graph of n back-to-back calls of fn(stream), recorded on a side stream."""
        fn(side)                                # first use of a kernel (module load, attributes) stays outside the capture
        side.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            for _ in range(n):
                fn(side)
        return g

    def graph_timed(g, launches_per_replay, replays=10, batches=5):
        """Median microseconds per launch over `replays` replays of graph g."""
        out = []
        for _ in range(batches):
            g.replay()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(replays):
                g.replay()
            e1.record(stream)
            e1.synchronize()
            out.append(e0.elapsed_time(e1) * 1000.0 / (replays * launches_per_replay))
        return float(np.median(out))

    if args.only:
        # ---------------------------------------------------- profiling targets ----
        def named(d, name, kind="conv"):
            count = h.conv2d_variant_count(d) if kind == "conv" else h.gemm_variant_count(d)
            for v in range(count):
                try:
                    if (h.conv2d_variant_name(d, v) if kind == "conv" else h.gemm_variant_name(d, v)) == name:
                        d.variant = v
                        return d
                except alt.AltError:
                    pass
            raise SystemExit("bench.py: this build has no variant %s" % name)

        reps = max(args.steps, 1)
        if args.only == "gemm4096":
            d = named(alt.gemm_desc(4096, 4096, 4096, in_dtype=alt.BF16, out_dtype=alt.BF16, b_layout="KN->NK"),
                      "bf16_256x256x32_stream_w2x4x1_s4_k1", "gemm")
            A = torch.randint(-200, 200, (4096 * 4096,), dtype=torch.int16, device=dev)
            B = torch.randint(-200, 200, (4096 * 4096,), dtype=torch.int16, device=dev)
            Cd = torch.empty(4096 * 4096, dtype=torch.int16, device=dev)
            us = timed(lambda: h.gemm(d, A, B, Cd, stream=stream), reps)
            print(json.dumps(dict(target=args.only, variant=h.gemm_variant_name(d, d.variant), us=round(us, 2),
                                  tflops=round(2.0 * 4096 ** 3 / us / 1e6, 1))))
        elif args.only == "conv_b256":
            d = named(alt.conv_desc(256, 64, 56, 56, 64, 3, 3, stride=1, pad=1, in_dtype=alt.BF16, out_dtype=alt.BF16,
                                    x_layout="NCHW->NHWC", w_layout="OIHW->OHWI", y_layout="NCHW->NHWC"),
                      "bf16_256x64x64_direct_w4x1_s3_k1")
            xs = torch.randint(-200, 200, (256 * 64 * 56 * 56,), dtype=torch.int16, device=dev)
            wsd = torch.randint(-200, 200, (64 * 64 * 9,), dtype=torch.int16, device=dev)
            ys = torch.empty(256 * 64 * 56 * 56, dtype=torch.int16, device=dev)
            us = timed(lambda: h.conv2d(d, xs, wsd, ys, stream=stream), reps)
            print(json.dumps(dict(target=args.only, variant=h.conv2d_variant_name(d, d.variant), us=round(us, 2),
                                  tflops=round(conv_flops(256, **RESNET_LAYERS[0]) / us / 1e6, 1))))
        elif args.only == "transform":
            out = {}
            for shp in [(256, 64, 56, 56), (16, 64, 56, 56)]:
                numel = int(np.prod(shp))
                nring = max(2, int(math.ceil((1 << 30) / (numel * 8))))
                srcs = [torch.randint(-30000, 30000, (numel,), dtype=torch.int32, device=dev).view(torch.float32) for _ in range(nring)]
                dsts = [torch.empty(numel, dtype=torch.float32, device=dev) for _ in range(nring)]
                la, lb = alt.layout_parse("NCHW->NCHW"), alt.layout_parse("NCHW->NHWC")
                k = [0]

                def one():
                    h.layout_transform(alt.F32, shp, la, srcs[k[0] % nring], lb, dsts[k[0] % nring], stream=stream)
                    k[0] += 1
                us = timed(one, max(reps, 2 * nring), warm=nring)
                out["x".join(map(str, shp))] = dict(us=round(us, 2), GBps=round(2.0 * numel * 4 / 1e3 / us, 1), ring_buffers=2 * nring)
                del srcs, dsts
            print(json.dumps(dict(target=args.only, fp32_nchw_to_nhwc=out)))
        elif args.only == "step":
            with open(args.plan) as f:
                plan = json.load(f)["bf16_out"]
            layers = prepare_layers(16, alt.BF16, 0, plan)
            torch.cuda.synchronize()

            def step():
                for l in layers:
                    run_layer(l)
            us = timed(step, reps)
            print(json.dumps(dict(target=args.only, us_per_step_one_stream=round(us, 2),
                                  variants=[l["variant"] for l in layers])))
        elif args.only == "step_nchw":
            # the five layers in the default layouts (NCHW activations and output, OIHW weights): the
            # channel-planar kernels, each layer under the library's own choice of tile
            ls = []
            for L in RESNET_LAYERS:
                d = alt.conv_desc(16, L["C"], L["H"], L["W"], L["K"], L["R"], L["S"], stride=L["stride"], pad=L["pad"],
                                  in_dtype=alt.BF16, out_dtype=alt.BF16)
                oh, ow = conv_out_hw(L["H"], L["W"], L["R"], L["S"], L["stride"], L["pad"])
                ls.append((d, torch.randint(-200, 200, (16 * L["C"] * L["H"] * L["W"],), dtype=torch.int16, device=dev),
                           torch.randint(-200, 200, (L["K"] * L["C"] * L["R"] * L["S"],), dtype=torch.int16, device=dev),
                           torch.empty(16 * L["K"] * oh * ow, dtype=torch.int16, device=dev)))

            def step():
                for d, x, w, y in ls:
                    h.conv2d(d, x, w, y, stream=stream)
            us = timed(step, reps)
            print(json.dumps(dict(target=args.only, us_per_step_one_stream=round(us, 2),
                                  variants=[h.conv2d_variant_name(d, -1) for d, _, _, _ in ls])))
        else:
            raise SystemExit("bench.py: unknown --only target %s" % args.only)
        if args.calib_copy:
            h.get_peak(arena[:512 << 20], 512 << 20)
        torch.cuda.synchronize()
        return

    all_plans = {}
    if not args.retune and os.path.exists(args.plan):
        with open(args.plan) as f:
            all_plans = json.load(f)
    tuned_now = []

    def load_layers(out_dtype, key):
        """The five batch-16 layers with output type `out_dtype`, under the stored choice or tuned now."""
        plan = all_plans.get(key)
        layers = prepare_layers(16, out_dtype, 0, plan)
        torch.cuda.synchronize()
        if plan is None or any(l["L"]["name"] not in plan for l in layers):
            tuned_now.append(key)
            all_plans[key] = {l["L"]["name"]: dict(layout=l["layout"], variant=l["variant"], trials=l["trials"],
                                                   tuned_us=round(l["best_us"], 2),
                                                   default_layout_us=round(l["default_us"], 2),
                                                   layout_us=l["layout_us"]) for l in layers}
        return layers

    lanes = [torch.cuda.Stream() for _ in RESNET_LAYERS]

    def multi_step(layers, descs, order=None):
        """One alt_conv2d_multi call that issues `layers` under `descs`, each on a stream of its own,
        in the given order (which kernels meet on the chip depends on it)."""
        calls = [dict(d=d, x=l["x"], w=l["w"], y=l["y"], workspace=l["ws"], ws_bytes=l["ws_bytes"], stream=lanes[i])
                 for i, (l, d) in enumerate(zip(layers, descs))]
        return h.conv2d_multi_prepared([calls[i] for i in (order or range(len(calls)))])

    def co_tune(layers):
        """Kernel variants and issue order for the five-stream launch, chosen jointly by
        alt_tune_conv2d_multi (coordinate descent on the measured time of the whole step)."""
        import copy
        calls = [dict(d=l["desc"], x=l["x"], w=l["w"], y=l["y"], workspace=l["ws"], ws_bytes=l["ws_bytes"], stream=lanes[i])
                 for i, l in enumerate(layers)]
        variants, order, _, measurements = h.tune_conv2d_multi(calls)
        descs = []
        for l, v in zip(layers, variants):
            d = copy.copy(l["desc"])
            d.variant = v
            descs.append(d)
        return descs, order, measurements

    def measure_step(layers, co_descs=None, co_order=None):
        """Times the step over `layers` as one HIP graph replayed args.steps times, then each layer on its own."""
        def step(st=None):
            for l in layers:
                run_layer(l, st)

        # The step is recorded once into a HIP graph and replayed: the five launches
        # then cost the GPU's own dispatch time, not the host's call path.  Every
        # replay runs the same kernels on the same buffers as the eager step; the
        # outputs of the two are compared bit for bit below.
        step()
        torch.cuda.synchronize()
        eager_y = [l["y"].clone() for l in layers]
        for l in layers:
            l["y"].fill_(0)
        g_step = capture(step, 1)
        for _ in range(args.warmup):
            g_step.replay()
        torch.cuda.synchronize()
        for l, ye in zip(layers, eager_y):
            if not torch.equal(l["y"], ye):
                raise SystemExit("bench.py: graph replay of %s differs from the eager launch" % l["L"]["name"])
        def timed_steps(one_step):
            # --steps is a floor: a step is tens of microseconds and a timed region carries a fixed
            # cost of a few hundred, so every way is timed for at least MIN_TIMED_MS of device work.
            # A short probe region sizes the count; the steps actually timed are reported.
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(20):
                one_step()
            torch.cuda.synchronize()
            probe_ms = (time.perf_counter() - t0) * 1000.0 / 20
            n = max(args.steps, int(math.ceil(MIN_TIMED_MS / max(probe_ms, 1e-3))))
            for attempt in range(4):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                e0.record(stream)
                for _ in range(n):
                    one_step()
                e1.record(stream)
                torch.cuda.synchronize()
                total_ms = (time.perf_counter() - t0) * 1000.0
                if total_ms >= MIN_TIMED_MS or attempt == 3:
                    break
                # (the probe ran slower than the steady state: time again with enough steps)
                n = int(math.ceil(n * 1.15 * MIN_TIMED_MS / max(total_ms, 1e-3)))
            return total_ms / n, e0.elapsed_time(e1) / n, n

        # Three ways to issue the same five launches: one graph replay per step, five
        # launches on one stream through calls marshalled once, or one alt_conv2d_multi
        # call that spreads them over five streams.  The layers do not depend on one
        # another, so on separate streams one layer's start-up and tail overlap its
        # neighbours' main loops and a kernel with fewer workgroups than the chip has
        # compute units shares it.  The step is timed all three ways (host clock around
        # args.steps steps, device idle before and after); the best is `value`, and all
        # three figures are kept.
        for _ in range(args.warmup):
            step()
        g_ms, g_dev, g_n = timed_steps(g_step.replay)
        s_ms, s_dev, s_n = timed_steps(step)
        def timed_multi(descs, order=None):
            # reference: the same kernels launched one after the other on the default stream
            # (another variant may sum in another order and round a bf16 output differently)
            for l, d in zip(layers, descs):
                h.conv2d(d, l["x"], l["w"], l["y"], workspace=l["ws"], ws_bytes=l["ws_bytes"], stream=stream)
            torch.cuda.synchronize()
            serial_y = [l["y"].clone() for l in layers]
            multi = multi_step(layers, descs, order)
            for l in layers:
                l["y"].fill_(0)
            torch.cuda.synchronize()                # the fills run on the default stream, the step on streams of its own
            for _ in range(args.warmup):
                multi()
            torch.cuda.synchronize()
            for l, ye in zip(layers, serial_y):
                if not torch.equal(l["y"], ye):
                    raise SystemExit("bench.py: multi-stream launch of %s differs from the same kernel launched alone" % l["L"]["name"])
            r = timed_steps(multi)
            return r[0], r[2]
        m_ms, m_n = timed_multi([l["desc"] for l in layers])
        ways = [(g_ms, g_dev, "one HIP graph replay per step (5 kernel nodes, one stream)", g_n),
                (s_ms, s_dev, "5 launches per step on one stream (arguments marshalled once)", s_n),
                (m_ms, m_ms, "one alt_conv2d_multi call per step: the 5 independent layers on 5 streams", m_n)]
        res = dict(graph_ms_per_step=g_ms, stream_ms_per_step=s_ms, multi_stream_ms_per_step=m_ms)
        if co_descs is not None:
            # the same launch with the kernel variants chosen jointly for it (see co_tune)
            c_ms, c_n = timed_multi(co_descs, co_order)
            res["multi_stream_cotuned_ms_per_step"] = c_ms
            res["cotuned_variants"] = [h.conv2d_variant_name(d, d.variant) for d in co_descs]
            res["cotuned_issue_order"] = [layers[i]["L"]["name"] for i in (co_order or range(len(layers)))]
            ways.append((c_ms, c_ms, "one alt_conv2d_multi call per step: the 5 independent layers on 5 streams, "
                                     "kernel variants chosen jointly under that launch", c_n))
        best = min(ways, key=lambda t: t[0])
        res.update(ms_per_step=best[0], dev_ms_per_step=best[1], launch=best[2], steps_timed=best[3])
        del eager_y
        del g_step
        # per-layer kernel durations, live: 20 launches of the layer per graph replay; the default
        # layout (NCHW activations, OIHW weights) is measured in the same run, under the best of its own
        # kernel variants (a short search on the device); what comes from the stored plan says so
        per_layer = []
        for l in layers:
            g = capture(lambda st, l=l: run_layer(l, st), 20)
            us = graph_timed(g, 20)
            del g
            l["us"] = us
            cold_us = cold_layer_us(l)
            L = l["L"]
            d0 = alt.conv_desc(16, L["C"], L["H"], L["W"], L["K"], L["R"], L["S"], stride=L["stride"], pad=L["pad"],
                               in_dtype=alt.BF16, out_dtype=l["desc"].out_dtype)
            try:
                def_us, def_trials = h.tune_conv2d_variants(d0, arena, arena.numel(), max_trials=args.default_trials,
                                                            warmup=3, reps=20)
                def_us = float(def_us)
            except alt.AltError:
                def_us, def_trials = float("nan"), 0
            stored = not tuned_now
            per_layer.append(dict(layer=L["name"], layout=l["layout"], variant=l["variant"], us=round(us, 3),
                                  us_cold_inputs=None if cold_us is None else round(cold_us, 3),
                                  tflops=round(l["flops"] / us / 1e6, 1),
                                  frac_mfma_peak=round(l["flops"] / us / 1e6 / PEAK_BF16_TFLOPS, 4),
                                  frac_own_ceiling=round(l["flops"] / us / 1e6 / own_ceiling_tflops(l), 4),
                                  compulsory_GBps=round(l["bytes"] / us / 1e3, 1),
                                  default_layout_us_live=round(def_us, 2), default_layout_trials_live=int(def_trials),
                                  speedup_vs_default_layout_live=round(def_us / us, 2),
                                  plan_is_stored=stored,
                                  plan=dict(tuner_trials=l["trials"], default_layout_us=round(l["default_us"], 2),
                                            tuned_us=round(l["best_us"], 2), layout_us=l["layout_us"])))
        res["per_layer"] = per_layer
        return res

    def own_ceiling_tflops(l):
        """min(MFMA peak, arithmetic intensity x HBM peak) of a layer, from its compulsory bytes."""
        return min(PEAK_BF16_TFLOPS, l["flops"] / l["bytes"] * PEAK_HBM_GBPS / 1e3)

    def load_traffic():
        """HBM bytes per launch from a stored pair of hardware-counter runs (FETCH_SIZE and
        WRITE_SIZE averages per dispatch, scaled by the plain copy kernel's reading), or None."""
        path = os.path.join(ROOT, "workloads", "measured_traffic_gfx950.json")
        if not os.path.exists(path):
            return None
        with open(path) as f:
            return json.load(f)

    def kernel_traffic(doc, layer, batch):
        """The stored traffic of the kernel instantiation and grid this layer launches."""
        import re
        if not doc:
            return None
        L, name = layer["L"], layer["variant"]
        m = re.match(r"bf16_(\d+)x(\d+)x(\d+)_(direct|stream)_w(\d+)x(\d+)(?:x(\d+))?_s(\d+)_k(\d+)$", name)
        if not m:
            return None
        BM, BN, BK, kind, wgm, wgn, kw, ns, sk = (int(g) if g and g.isdigit() else g for g in m.groups())
        kw = kw or 1
        oh, ow = conv_out_hw(L["H"], L["W"], L["R"], L["S"], L["stride"], L["pad"])
        tiles = -(-(batch * oh * ow) // BM) * -(-L["K"] // BN)
        if sk > 1:
            tiles = -(-tiles // 8) * 8
        grid = tiles * sk * 64 * wgm * wgn * kw
        ncc = L["C"] // sk // kw // BK
        if kind == "direct":
            kr = L["R"] if (L["R"] == L["S"] and ((L["R"] == 3 and ncc in (1, 2)) or (L["R"] == 1 and ncc in (1, 2, 4, 8)))) else 0
            key = "dconv_kernel<%d, %d, %d, %d, %d, %d, %d, %d, %d>|%d" % (BM, BN, wgm, wgn, kw, ns, BK, kr, ncc if kr else 0, grid)
        else:
            key = "dstream_kernel<%d, %d, %d, %d, %d, %d, %d, false>|%d" % (BM, BN, wgm, wgn, kw, ns, BK, grid)
        e = doc["kernels"].get(key)
        if not e or "fetch_bytes" not in e or "write_bytes" not in e:
            return None
        return dict(fetch_bytes=e["fetch_bytes"], write_bytes=e["write_bytes"])

    # headline: bf16 in, fp32 accumulate, bf16 out (the layer's output feeds a bf16 layer)
    layers = load_layers(alt.BF16, "bf16_out")
    co_plan = all_plans.get("bf16_out_concurrent")
    co_descs, co_order = None, None
    if co_plan is not None:
        co_descs = [from_plan(l["desc"], dict(layout=l["layout"], variant=co_plan.get(l["L"]["name"], ""))) for l in layers]
        names = [l["L"]["name"] for l in layers]
        if any(d is None for d in co_descs):
            co_descs = None
        elif sorted(co_plan.get("issue_order", [])) == sorted(names):
            co_order = [names.index(n) for n in co_plan["issue_order"]]
    if co_descs is None and (args.retune or "bf16_out" in tuned_now):
        co_descs, co_order, co_trials = co_tune(layers)
        all_plans["bf16_out_concurrent"] = {l["L"]["name"]: h.conv2d_variant_name(d, d.variant)
                                            for l, d in zip(layers, co_descs)}
        all_plans["bf16_out_concurrent"]["issue_order"] = [layers[i]["L"]["name"] for i in co_order]
        tuned_now.append("bf16_out_concurrent (%d step measurements)" % co_trials)
    head = measure_step(layers, co_descs, co_order)
    ms_per_step, dev_ms_per_step = head["ms_per_step"], head["dev_ms_per_step"]
    step_flops = sum(l["flops"] for l in layers)
    value = step_flops / (ms_per_step * 1e-3) / 1e12
    per_layer = head["per_layer"]
    dom = max(layers, key=lambda l: l["us"])
    achieved = dom["flops"] / dom["us"] / 1e6
    attainable = None
    if want("peaks"):
        pk = h.get_peak(arena, arena.numel())
        attainable = dict(copy_GBps=round(float(pk.copy_gbps), 1), read_GBps=round(float(pk.read_gbps), 1),
                          write_GBps=round(float(pk.write_gbps), 1),
                          mfma_bf16_TFLOPs=round(float(pk.mfma_bf16_tflops), 1),
                          compute_units=pk.compute_units, clock_mhz=pk.clock_mhz, arch=pk.arch.decode(),
                          note="streams over a 1 GiB arena (copy: 512 MiB read + 512 MiB written per launch); "
                               "register-resident bf16 MFMA loop")
    traffic_doc = load_traffic()
    for l, pl in zip(layers, per_layer):
        tr = kernel_traffic(traffic_doc, l, 16)
        if tr:
            pl["hbm_bytes_per_launch"] = tr
    dom_tr = kernel_traffic(traffic_doc, dom, 16)
    roofline = dict(bound="mfma", achieved=round(achieved, 2), peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                    frac=round(achieved / PEAK_BF16_TFLOPS, 4),
                    traffic=(dom_tr["fetch_bytes"] + dom_tr["write_bytes"]) if dom_tr else None,
                    traffic_source="stored rocprofv3 --pmc runs of this kernel and grid" if dom_tr else None,
                    kernel=dom["variant"], layer=dom["L"]["name"],
                    us_per_launch=round(dom["us"], 3), flops_per_launch=dom["flops"],
                    frac_vs_attainable=round(achieved / attainable["mfma_bf16_TFLOPs"], 4) if attainable else None,
                    frac_own_ceiling=round(achieved / own_ceiling_tflops(dom), 4))

    extra = dict(per_layer_b16=per_layer, device_ms_per_step=round(dev_ms_per_step, 4), launch=head["launch"],
                 graph_replay_ms_per_step=round(head["graph_ms_per_step"], 5),
                 stream_launch_ms_per_step=round(head["stream_ms_per_step"], 5),
                 multi_stream_ms_per_step=round(head["multi_stream_ms_per_step"], 5))
    if "multi_stream_cotuned_ms_per_step" in head:
        extra["multi_stream_cotuned_ms_per_step"] = round(head["multi_stream_cotuned_ms_per_step"], 5)
        extra["multi_stream_cotuned_variants"] = head["cotuned_variants"]
        extra["multi_stream_cotuned_issue_order"] = head["cotuned_issue_order"]

    if want("f32"):
        # the same step with fp32 output (twice the output bytes)
        l32 = load_layers(alt.F32, "f32_out")
        r32 = measure_step(l32)
        extra["step_f32_out"] = dict(ms_per_step=round(r32["ms_per_step"], 5), launch=r32["launch"],
                                     tflops=round(step_flops / (r32["ms_per_step"] * 1e-3) / 1e12, 2),
                                     per_layer_b16=r32["per_layer"])
        del l32
    extra["layer_choice"] = ("tuned in this run: " + ", ".join(tuned_now)) if tuned_now else \
        "read from " + os.path.relpath(args.plan, ROOT)
    if tuned_now:
        out_path = args.plan if args.retune else os.path.join(ROOT, "gpurun_out", "tuned_plan.json")
        try:
            os.makedirs(os.path.dirname(out_path), exist_ok=True)
            with open(out_path, "w") as f:
                json.dump(all_plans, f, indent=1)
        except OSError:
            pass

    if args.calib_copy:
        h.get_peak(arena[:512 << 20], 512 << 20)

    if want("transforms"):
        # -------------------------------------------------- conversion operator ----
        # Cold figures: a ring of distinct source and destination buffers of at least 1 GiB in total,
        # four times the 256 MB last-level cache, so every launch reads from and writes to HBM.  Warm
        # figures: the same pair of buffers again and again (cache-resident at the configured sizes).
        # Both are per launch inside a HIP graph on one stream, i.e. they include the gap between
        # consecutive kernels of a stream.
        RING_BYTES = 1 << 30
        pairs = [("NCHW->NCHW", "NCHW->NHWC"), ("NCHW->NHWC", "NCHW->NCHW"),
                 ("NCHW->NCHW", "NCHW->NCHW16c"), ("NCHW->NCHW", "NCHW->NCHW32c")]

        def transform_rows(shapes, warm):
            rows = []
            for shp in shapes:
                numel = int(np.prod(shp))
                for dt, tdt, es in [(alt.F32, torch.float32, 4), (alt.BF16, torch.int16, 2)]:
                    nring = max(2, int(math.ceil(RING_BYTES / (numel * es * 2))))
                    srcs = [torch.randint(-30000, 30000, (numel,), dtype=torch.int16 if es == 2 else torch.int32,
                                          device=dev).view(tdt) for _ in range(nring)]
                    dsts = [torch.empty(numel, dtype=tdt, device=dev) for _ in range(nring)]
                    for a, b in pairs:
                        la, lb = alt.layout_parse(a), alt.layout_parse(b)
                        def ring(st):
                            for i in range(nring):
                                h.layout_transform(dt, shp, la, srcs[i], lb, dsts[i], stream=st)

                        g = capture(ring, 1)
                        us_cold = graph_timed(g, nring, replays=4, batches=3)
                        gb = 2.0 * numel * es / 1e9
                        row = dict(shape=list(shp), dtype="f32" if dt == alt.F32 else "bf16",
                                   src=a.split(">")[1], dst=b.split(">")[1], ring_buffers=2 * nring,
                                   ring_MB=round(2 * nring * numel * es / 1e6), us_hbm=round(us_cold, 2),
                                   GBps_hbm=round(gb / (us_cold * 1e-6), 1),
                                   frac_hbm_peak=round(gb / (us_cold * 1e-6) / PEAK_HBM_GBPS, 4))
                        if warm:
                            g = capture(lambda st: h.layout_transform(dt, shp, la, srcs[0], lb, dsts[0], stream=st), 20)
                            us_warm = graph_timed(g, 20, replays=5, batches=3)
                            row.update(us_cache_resident=round(us_warm, 2),
                                       GBps_cache_resident=round(gb / (us_warm * 1e-6), 1))
                        del g
                        rows.append(row)
                    del srcs, dsts
            return rows

        extra["layout_transform"] = transform_rows(TRANSFORM_SHAPES, warm=True)
        # scaled beyond the configs: 16x the batch of each shape, cold, to show the kernels away from launch overhead
        extra["layout_transform_scaled"] = transform_rows([(16 * s[0],) + tuple(s[1:]) for s in TRANSFORM_SHAPES], warm=False)
        # the unfold primitive (overlapped tiles of 14 + 2 rows along H of an NHWC tensor, Section 4.1.2): expands the data
        ushape = (16, 56, 56, 64)
        oshape = alt.unfold_shape(ushape, 1, 16, 14)
        u0 = torch.randint(-30000, 30000, (int(np.prod(ushape)),), dtype=torch.int16, device=dev)
        u1 = torch.empty(int(np.prod(oshape)), dtype=torch.int16, device=dev)
        gr = capture(lambda st: h.unfold(alt.BF16, ushape, 1, 16, 14, u0, u1, stream=st), 20)
        us = graph_timed(gr, 20)
        del gr
        moved = (u0.numel() + u1.numel()) * 2
        extra["unfold_16x56x56x64_bf16_H_tiles_of_16_every_14"] = dict(
            out_shape=list(oshape), us=round(us, 2), GBps=round(moved / 1e9 / (us * 1e-6), 1),
            frac_hbm_peak=round(moved / 1e9 / (us * 1e-6) / PEAK_HBM_GBPS, 4), note="cache-resident buffers")
        del u0, u1
        # the spatially tiled C2D template (Section 5.1) with the tiles materialised: a 58x58x64 input unfolded
        # into 16x16-pixel tiles (14 + 2 along H and W), convolved tile by tile without padding, against the direct
        # kernel, which keeps the same overlapped tile in LDS and never writes it out
        N_, C_, H_, K_, ht = 16, 64, 58, 64, 14
        TH, BH = (H_ - 2) // ht, ht + 2
        xs = torch.randint(-200, 200, (N_ * H_ * H_ * C_,), dtype=torch.int16, device=dev)
        wsd2 = torch.randint(-200, 200, (K_ * C_ * 9,), dtype=torch.int16, device=dev)
        s1 = alt.unfold_shape((N_, H_, H_, C_), 1, BH, ht)
        s2 = alt.unfold_shape(s1, 3, BH, ht)
        t1 = torch.empty(int(np.prod(s1)), dtype=torch.int16, device=dev)
        t2 = torch.empty(int(np.prod(s2)), dtype=torch.int16, device=dev)
        t3 = torch.empty_like(t2)
        ident, swap = alt.layout_from_prims(s2, []), alt.layout_from_prims(s2, [alt.reorder([0, 1, 3, 2, 4, 5])])
        dt = alt.conv_desc(N_ * TH * TH, C_, BH, BH, K_, 3, 3, stride=1, pad=0, in_dtype=alt.BF16, out_dtype=alt.BF16,
                           x_layout="NCHW->NHWC", w_layout="OIHW->OHWI", y_layout="NCHW->NHWC")
        yt = torch.empty(N_ * TH * TH * ht * ht * K_, dtype=torch.int16, device=dev)

        def tiled(st):
            h.unfold(alt.BF16, (N_, H_, H_, C_), 1, BH, ht, xs, t1, stream=st)
            h.unfold(alt.BF16, s1, 3, BH, ht, t1, t2, stream=st)
            h.layout_transform(alt.BF16, s2, ident, t2, swap, t3, stream=st)
            h.conv2d(dt, t3, wsd2, yt, stream=st)
        gr = capture(tiled, 5)
        us_all = graph_timed(gr, 5)
        del gr
        gr = capture(lambda st: h.conv2d(dt, t3, wsd2, yt, stream=st), 20)
        us_conv = graph_timed(gr, 20)
        del gr
        direct = next(l for l in layers if l["L"]["name"] == "c64_56_3x3")
        extra["conv_on_unfolded_tiles_c64_56x56_b16"] = dict(
            tiles=[N_ * TH * TH, BH, BH, C_], unfold_reorder_and_conv_us=round(us_all, 2), tile_conv_alone_us=round(us_conv, 2),
            direct_kernel_us=round(direct["us"], 2),
            note="the tile convolution has no padding and runs on the direct kernel too (default variant); "
                 "direct_kernel_us is the un-tiled layer with same-size padding under its tuned variant")
        del xs, wsd2, t1, t2, t3, yt

    if want("gemm"):
        # ------------------------------------------------------------------ gemm ----
        gm = []
        for g in BERT_GEMMS + [BERT_QKT]:
            d0 = alt.gemm_desc(g["M"], g["N"], g["K"], batch=g["batch"], in_dtype=alt.BF16, out_dtype=alt.F32)
            best, rep = h.tune_gemm(d0, arena, arena.numel(), max_trials=0, warmup=3, reps=30)
            A = torch.randint(-200, 200, (g["batch"] * g["M"] * g["K"],), dtype=torch.int16, device=dev)
            B = torch.randint(-200, 200, (g["batch"] * g["K"] * g["N"],), dtype=torch.int16, device=dev)
            Cd = torch.empty(g["batch"] * g["M"] * g["N"], dtype=torch.float32, device=dev)
            wsb = h.gemm_workspace_size(best)
            ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device=dev)
            gr = capture(lambda st: h.gemm(best, A, B, Cd, workspace=ws, ws_bytes=wsb, stream=st), 20)
            us = graph_timed(gr, 20)
            del gr
            fl = 2.0 * g["batch"] * g["M"] * g["N"] * g["K"]
            names = [rep.layout_name[i].value.decode() for i in range(rep.n_layouts)]
            lus = [float(rep.layout_best_us[i]) for i in range(rep.n_layouts)]
            gm.append(dict(gemm=g["name"], M=g["M"], N=g["N"], K=g["K"], batch=g["batch"],
                           layout=names[int(np.argmin(lus))], variant=h.gemm_variant_name(best, best.variant),
                           us=round(us, 3), tflops=round(fl / us / 1e6, 1),
                           frac_mfma_peak=round(fl / us / 1e6 / PEAK_BF16_TFLOPS, 4),
                           default_layout_us=round(float(rep.default_us), 2), tuned_us=round(float(rep.best_us), 2),
                           speedup_vs_default_layout=round(float(rep.default_us) / float(rep.best_us), 2),
                           tuner_trials=rep.trials, layout_us=dict(zip(names, [round(u, 2) for u in lus]))))
        extra["gemm_bert"] = gm
        # scaled beyond the configs: one 4096^3 product, bf16 output, tuned with a budget
        d0 = alt.gemm_desc(4096, 4096, 4096, in_dtype=alt.BF16, out_dtype=alt.BF16, b_layout="KN->NK")
        us_best, trials = None, 0
        A = torch.randint(-200, 200, (4096 * 4096,), dtype=torch.int16, device=dev)
        B = torch.randint(-200, 200, (4096 * 4096,), dtype=torch.int16, device=dev)
        Cd = torch.empty(4096 * 4096, dtype=torch.int16, device=dev)
        best, rep = h.tune_gemm(d0, arena, arena.numel(), max_trials=64, warmup=2, reps=5, layout_mask=0)
        wsb = h.gemm_workspace_size(best)
        ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device=dev)
        us = median_timed(lambda: h.gemm(best, A, B, Cd, workspace=ws, ws_bytes=wsb, stream=stream), 20, 3)
        fl = 2.0 * 4096 ** 3
        extra["gemm_4096"] = dict(variant=h.gemm_variant_name(best, best.variant), us=round(us, 1),
                                  tflops=round(fl / us / 1e6, 1), frac_mfma_peak=round(fl / us / 1e6 / PEAK_BF16_TFLOPS, 4),
                                  tuner_trials=rep.trials)
        # the same product with B row-major ([K][N], the default layout), under the library's own choice of tile
        dk = alt.gemm_desc(4096, 4096, 4096, in_dtype=alt.BF16, out_dtype=alt.BF16)
        us_kn = median_timed(lambda: h.gemm(dk, A, B, Cd, stream=stream), 20, 3)
        extra["gemm_4096"]["row_major_b"] = dict(variant=h.gemm_variant_name(dk, -1), us=round(us_kn, 1),
                                                 tflops=round(fl / us_kn / 1e6, 1))
        del A, B, Cd

    if want("b1"):
        # ------------------------------------------------------- batch-1 layers ----
        l1 = prepare_layers(1, alt.F32, 0)
        b1 = []
        for l in l1:
            g = capture(lambda st, l=l: run_layer(l, st), 20)
            us = graph_timed(g, 20)
            del g
            b1.append(dict(layer=l["L"]["name"], layout=l["layout"], variant=l["variant"], us=round(us, 3),
                           tflops=round(l["flops"] / us / 1e6, 2),
                           speedup_vs_default_layout=round(l["default_us"] / l["best_us"], 2)))
        extra["per_layer_b1"] = b1
        del l1

    if want("scaled"):
        # ---------------------------------------- scaled: 16x batch, bf16 output ----
        scaled = []
        for L in RESNET_LAYERS[:1] + RESNET_LAYERS[2:3]:
            batch = 256
            shape = alt.conv_desc(batch, L["C"], L["H"], L["W"], L["K"], L["R"], L["S"], stride=L["stride"],
                                  pad=L["pad"], in_dtype=alt.BF16, out_dtype=alt.BF16,
                                  x_layout="NCHW->NHWC", w_layout="OIHW->OHWI", y_layout="NCHW->NHWC")
            xs = torch.randint(-200, 200, (batch * L["C"] * L["H"] * L["W"],), dtype=torch.int16, device=dev)
            wsd = torch.randint(-200, 200, (L["K"] * L["C"] * L["R"] * L["S"],), dtype=torch.int16, device=dev)
            oh, ow = conv_out_hw(L["H"], L["W"], L["R"], L["S"], L["stride"], L["pad"])
            ys = torch.empty(batch * L["K"] * oh * ow, dtype=torch.int16, device=dev)
            us_best, _ = h.tune_conv2d_variants(shape, arena, arena.numel(), max_trials=96, warmup=2, reps=10)
            us = median_timed(lambda: h.conv2d(shape, xs, wsd, ys, workspace=arena, ws_bytes=arena.numel(), stream=stream), 20, 3)
            fl = conv_flops(batch, **L)
            scaled.append(dict(layer=L["name"], batch=batch, variant=h.conv2d_variant_name(shape, shape.variant),
                               us=round(us, 1), tflops=round(fl / us / 1e6, 1),
                               frac_mfma_peak=round(fl / us / 1e6 / PEAK_BF16_TFLOPS, 4)))
            del xs, wsd, ys
        extra["conv_scaled_batch256_nhwc_bf16out"] = scaled

    if want("chain"):
        # ------------------------------------------------------------------ chain ----
        ops = [alt.conv_desc(16, c["C"], c["H"], c["W"], c["K"], c["R"], c["S"], stride=c["stride"], pad=c["pad"],
                             in_dtype=alt.BF16, out_dtype=alt.BF16,
                             epilogue=(alt.EPI_BIAS if c["bias"] else 0) | (alt.EPI_RELU if c["relu"] else 0))
               for c in CHAIN_LAYERS]
        plan = h.tune_chain(ops, "NCHW->NCHW", arena, arena.numel(), max_trials=0, warmup=3, reps=20)
        extra["chain"] = dict(planned_total_us=round(float(plan.total_us), 2),
                              all_nchw_total_us=round(float(plan.default_total_us), 2),
                              speedup_vs_all_nchw=round(float(plan.default_total_us) / float(plan.total_us), 2),
                              transforms_inserted=[int(plan.transform_before[i]) for i in range(plan.nops)],
                              op_us=[round(float(plan.op_us[i]), 2) for i in range(plan.nops)],
                              transform_us=[round(float(plan.transform_us[i]), 2) for i in range(plan.nops)],
                              variants=[h.conv2d_variant_name(plan.op[i], plan.op[i].variant) for i in range(plan.nops)],
                              measurements=plan.trials)

    if want("graph"):
        # ------------------------------------------------- residual block (graph) ----
        # conv3x3+bias+ReLU -> conv3x3+bias -> + block input -> ReLU, 64 channels, 56x56, batch 16, bf16 tensors:
        # layouts propagate through the sum, the block input has two consumers
        def phys(l):
            return "".join("NCHW"[l.sub_dim[j]] if l.sub_extent[j] == 0 else "%d%s" % (l.sub_extent[j], "nchw"[l.sub_dim[j]])
                           for j in range(l.nsub))
        mk = lambda relu: alt.conv_desc(16, 64, 56, 56, 64, 3, 3, stride=1, pad=1, in_dtype=alt.BF16, out_dtype=alt.BF16,
                                        epilogue=alt.EPI_BIAS | (alt.EPI_RELU if relu else 0))
        blk = [alt.graph_node(alt.NODE_CONV, 0, conv=mk(True)), alt.graph_node(alt.NODE_CONV, 1, conv=mk(False)),
               alt.graph_node(alt.NODE_ADD, 2, 0, relu=1)]
        gp = h.tune_graph(blk, "NCHW->NCHW", arena, arena.numel(), max_trials=0, warmup=3, reps=20)
        numel = 16 * 64 * 56 * 56
        ea = torch.randint(-30000, 30000, (numel,), dtype=torch.int16, device=dev)
        eb = torch.randint(-30000, 30000, (numel,), dtype=torch.int16, device=dev)
        ey = torch.empty_like(ea)
        gr = capture(lambda st: h.eltwise_add(alt.BF16, numel, ea, eb, ey, relu=True, stream=st), 20)
        add_us = graph_timed(gr, 20)
        del gr
        # the same block with the join fused into the second convolution's epilogue (alt_conv2d_add), under the
        # planned layout of that convolution when the tile kernels take it
        import copy
        fused = None
        fd = copy.copy(gp.conv[1])
        fd.epilogue = alt.EPI_BIAS | alt.EPI_RELU
        fw = torch.randint(-200, 200, (64 * 64 * 9,), dtype=torch.int16, device=dev)
        fb = torch.zeros(64, dtype=torch.float32, device=dev)
        try:
            gr = capture(lambda st: h.conv2d_add(fd, ea, fw, eb, ey, bias=fb, stream=st), 20)
            fused = graph_timed(gr, 20)
            del gr
        except alt.AltError:
            pass
        del ea, eb, ey, fw, fb
        extra["residual_block"] = dict(
            planned_total_us=round(float(gp.total_us), 2), all_nchw_total_us=round(float(gp.default_total_us), 2),
            speedup_vs_all_nchw=round(float(gp.default_total_us) / float(gp.total_us), 2),
            tensor_layouts=[phys(gp.tensor_layout[t]) for t in range(4)],
            conversions=[[int(gp.convert[i][j]) for j in range(2)] for i in range(3)],
            conversion_us=[[round(float(gp.convert_us[i][j]), 2) for j in range(2)] for i in range(3)],
            node_us=[round(float(gp.node_us[i]), 2) for i in range(3)],
            variants=[h.conv2d_variant_name(gp.conv[i], gp.conv[i].variant) for i in range(2)],
            measurements=gp.trials,
            add_relu_us=round(add_us, 2), add_relu_GBps=round(3.0 * numel * 2 / 1e9 / (add_us * 1e-6), 1),
            add_relu_frac_hbm_peak=round(3.0 * numel * 2 / 1e9 / (add_us * 1e-6) / PEAK_HBM_GBPS, 4))
        rb = extra["residual_block"]
        rb["sum_fused_into_node"] = int(gp.fused_into[2])        # -1: the planner kept the sum as a launch of its own
        if fused is not None:
            rb["conv_with_fused_sum_us"] = round(fused, 2)

    if want("groups"):
        # --------------------------- depth-wise and group-wise convolution ----
        # MobileNet-V2-shaped depth-wise 3x3 layers, bf16 in and out, under three layout choices: memory-bound, so the
        # figure is GB/s over the compulsory bytes (activations in, activations out, weights)
        dw = []
        for (C, HW, stride) in [(144, 56, 1), (384, 28, 1), (96, 112, 2)]:
            per = {}
            for xl, wl in [("NCHW", "OIHW"), ("NHWC", "HWIO"), ("NCHW16c", "OIHW16o")]:
                d = alt.conv_desc(16, C, HW, HW, C, 3, 3, stride=stride, pad=1, in_dtype=alt.BF16, out_dtype=alt.BF16,
                                  epilogue=alt.EPI_BIAS | alt.EPI_RELU, x_layout="NCHW->" + xl, w_layout="OIHW->" + wl,
                                  y_layout="NCHW->" + xl, groups=C)
                osh = h.conv2d_output_shape(d)
                xb = torch.randint(-30000, 30000, (16 * C * HW * HW,), dtype=torch.int16, device=dev)
                wb = torch.randint(-30000, 30000, (C * 9,), dtype=torch.int16, device=dev)
                bb = torch.zeros(C, dtype=torch.float32, device=dev)
                yb = torch.empty(int(np.prod(osh)), dtype=torch.int16, device=dev)
                gr = capture(lambda st: h.conv2d(d, xb, wb, yb, bias=bb, stream=st), 20)
                us = graph_timed(gr, 20)
                del gr
                nbytes = (xb.numel() + yb.numel() + wb.numel()) * 2
                per[xl] = dict(us=round(us, 2), GBps=round(nbytes / 1e9 / (us * 1e-6), 1),
                               frac_hbm_peak=round(nbytes / 1e9 / (us * 1e-6) / PEAK_HBM_GBPS, 4))
                del xb, wb, yb
            best = min(per, key=lambda k: per[k]["us"])
            dw.append(dict(layer="dw3x3_c%d_%dx%d_s%d" % (C, HW, HW, stride), batch=16, per_layout=per, best_layout=best,
                           speedup_vs_nchw=round(per["NCHW"]["us"] / per[best]["us"], 2)))
        extra["depthwise_b16"] = dw
        # a ResNeXt-shaped grouped 3x3 layer (128 channels in 4 groups, 28x28), tuned like the other layers
        gshape = alt.conv_desc(16, 128, 28, 28, 128, 3, 3, stride=1, pad=1, in_dtype=alt.BF16, out_dtype=alt.BF16, groups=4)
        gbest, grep_ = h.tune_conv2d(gshape, arena, arena.numel(), max_trials=0, warmup=3, reps=20)
        gfl = 2.0 * 16 * 128 * 28 * 28 * 32 * 9
        gnames = [grep_.layout_name[i].value.decode() for i in range(grep_.n_layouts)]
        extra["grouped_c128_g4_28x28_b16"] = dict(
            variant=h.conv2d_variant_name(gbest, gbest.variant), layout=gnames[int(np.argmin([grep_.layout_best_us[i] for i in range(grep_.n_layouts)]))],
            tuned_us=round(float(grep_.best_us), 2), default_layout_us=round(float(grep_.default_us), 2),
            tflops=round(gfl / float(grep_.best_us) / 1e6, 1), trials=grep_.trials,
            layout_us=dict(zip(gnames, [round(float(grep_.layout_best_us[i]), 2) for i in range(grep_.n_layouts)])))

        # a segmentation-style dilated 3x3 layer (256 channels, 28x28, taps two pixels apart), tuned like the others
        dshape = alt.conv_desc(16, 256, 28, 28, 256, 3, 3, stride=1, pad=2, dil=2, in_dtype=alt.BF16, out_dtype=alt.BF16)
        dbest, drep = h.tune_conv2d(dshape, arena, arena.numel(), max_trials=0, warmup=3, reps=20)
        dfl = 2.0 * 16 * 256 * 28 * 28 * 256 * 9
        dnames = [drep.layout_name[i].value.decode() for i in range(drep.n_layouts)]
        extra["dilated_c256_3x3_d2_28x28_b16"] = dict(
            variant=h.conv2d_variant_name(dbest, dbest.variant), layout=dnames[int(np.argmin([drep.layout_best_us[i] for i in range(drep.n_layouts)]))],
            tuned_us=round(float(drep.best_us), 2), default_layout_us=round(float(drep.default_us), 2),
            tflops=round(dfl / float(drep.best_us) / 1e6, 1), trials=drep.trials,
            layout_us=dict(zip(dnames, [round(float(drep.layout_best_us[i]), 2) for i in range(drep.n_layouts)])))

        # a decoder-style transposed convolution (128 -> 64 channels, 4x4, stride 2, 28x28 -> 56x56, batch 16):
        # zero insertion + the forward kernels, per activation layout
        t2d = {}
        tfl = 2.0 * 16 * 128 * 64 * 16 * 28 * 28              # nominal: every input pixel meets every filter tap
        for xl, wl in [("NCHW", "OIHW"), ("NHWC", "OHWI"), ("NCHW32c", "OIHW32o32i")]:
            d = alt.conv_desc(16, 128, 28, 28, 64, 4, 4, stride=2, pad=1, in_dtype=alt.BF16, out_dtype=alt.BF16,
                              x_layout="NCHW->" + xl, w_layout="OIHW->" + wl, y_layout="NCHW->" + xl)
            osh = h.conv2d_transpose_output_shape(d)
            # tune(op, shape) for the transposed operator: the variants of the forward problem it runs as
            h.tune_conv2d_variants(h.conv2d_transpose_problem(d), arena, arena.numel(), max_trials=0, warmup=3, reps=20)
            xb = torch.randint(-200, 200, (16 * 128 * 28 * 28,), dtype=torch.int16, device=dev)
            wsrc = torch.randint(-200, 200, (128 * 64 * 16,), dtype=torch.int16, device=dev)
            wb = torch.empty(int(np.prod(h.conv2d_transpose_weight_shape(d))), dtype=torch.int16, device=dev)
            h.pack_weights_transpose(d, wsrc, wb, stream=stream)
            yb = torch.empty(int(np.prod(osh)), dtype=torch.int16, device=dev)
            wsb = h.conv2d_transpose_workspace_size(d)
            wsd = torch.empty(wsb + 16, dtype=torch.uint8, device=dev)
            gr = capture(lambda st: h.conv2d_transpose(d, xb, wb, yb, workspace=wsd, ws_bytes=wsb, stream=st), 20)
            us = graph_timed(gr, 20)
            del gr, xb, wb, yb, wsd
            t2d[xl] = dict(us=round(us, 2), nominal_tflops=round(tfl / us / 1e6, 1))
        extra["conv_transpose_c128_k64_4x4_s2_28x28_b16"] = dict(
            per_layout=t2d, speedup_vs_nchw=round(t2d["NCHW"]["us"] / min(v["us"] for v in t2d.values()), 2),
            form="sub-pixel" if h.conv2d_transpose_weight_shape(d)[0] != 64 else "zero insertion",
            note="sub-pixel form: one stride-1 convolution of x with 4*K output channels into the workspace, then the kernel that "
                 "moves the four phases into place (and one that replicates the bias when there is one); tuned forward kernel")

        # a ResNet3D-18-shaped layer (the C3D of the operator list): 128 -> 128 channels, 3x3x3, 8 slices of 28x28,
        # batch 2; depth unfolded into the channels per call, then the 2-D kernels on 16 images of 384 channels
        c3d = {}
        c3fl = 2.0 * 2 * 8 * 28 * 28 * 128 * 128 * 27         # nominal: padding taps counted
        for xl, wl in [("NCHW", "OIHW"), ("NHWC", "OHWI"), ("NCHW32c", "OIHW32o32i")]:
            d = alt.conv3d_desc(2, 128, 8, 28, 28, 128, 3, 3, 3, stride=1, pad=1, in_dtype=alt.BF16, out_dtype=alt.BF16,
                                x_layout="NCHW->" + xl, w_layout="OIHW->" + wl, y_layout="NCHW->" + xl)
            osh = h.conv3d_output_shape(d)
            # tune(op, shape) for the 3-D operator: the variants of the 2-D problem it runs as
            h.tune_conv2d_variants(h.conv3d_problem(d), arena, arena.numel(), max_trials=0, warmup=3, reps=20)
            xb = torch.randint(-200, 200, (2 * 8 * 128 * 28 * 28,), dtype=torch.int16, device=dev)
            wb = torch.randint(-200, 200, (128 * 128 * 27,), dtype=torch.int16, device=dev)
            yb = torch.empty(int(np.prod(osh)), dtype=torch.int16, device=dev)
            wsb = h.conv3d_workspace_size(d)
            wsd = torch.empty(wsb + 16, dtype=torch.uint8, device=dev)
            gr = capture(lambda st: h.conv3d(d, xb, wb, yb, workspace=wsd, ws_bytes=wsb, stream=st), 20)
            us = graph_timed(gr, 20)
            del gr, xb, wb, yb, wsd
            c3d[xl] = dict(us=round(us, 2), nominal_tflops=round(c3fl / us / 1e6, 1))
        extra["conv3d_c128_3x3x3_8x28x28_b2"] = dict(
            per_layout=c3d, speedup_vs_nchw=round(c3d["NCHW"]["us"] / min(v["us"] for v in c3d.values()), 2),
            note="two launches per call (depth unfolding into the workspace, tuned forward kernel)")

        # the transposed 3-D operator (T3D): a decoder-shaped 4x4x4 stride-2 layer, 128 -> 64 channels,
        # 4 slices of 14x14 -> 8 slices of 28x28, batch 2
        t3d = {}
        t3fl = 2.0 * 2 * 128 * 64 * 64 * 4 * 14 * 14          # nominal: every input element meets every filter tap
        for xl, wl in [("NCHW", "OIHW"), ("NHWC", "OHWI"), ("NCHW32c", "OIHW32o32i")]:
            d = alt.conv3d_desc(2, 128, 4, 14, 14, 64, 4, 4, 4, stride=2, pad=1, in_dtype=alt.BF16, out_dtype=alt.BF16,
                                x_layout="NCHW->" + xl, w_layout="OIHW->" + wl, y_layout="NCHW->" + xl)
            osh = h.conv3d_transpose_output_shape(d)
            h.tune_conv2d_variants(h.conv3d_transpose_problem(d), arena, arena.numel(), max_trials=0, warmup=3, reps=20)
            xb = torch.randint(-200, 200, (2 * 4 * 128 * 14 * 14,), dtype=torch.int16, device=dev)
            wsrc = torch.randint(-200, 200, (128 * 64 * 64,), dtype=torch.int16, device=dev)
            wb = torch.empty(int(np.prod(h.conv3d_transpose_weight_shape(d))), dtype=torch.int16, device=dev)
            h.pack_weights3d_transpose(d, wsrc, wb, stream=stream)
            yb = torch.empty(int(np.prod(osh)), dtype=torch.int16, device=dev)
            wsb = h.conv3d_transpose_workspace_size(d)
            wsd = torch.empty(wsb + 16, dtype=torch.uint8, device=dev)
            gr = capture(lambda st: h.conv3d_transpose(d, xb, wb, yb, workspace=wsd, ws_bytes=wsb, stream=st), 20)
            us = graph_timed(gr, 20)
            del gr, xb, wb, yb, wsd
            t3d[xl] = dict(us=round(us, 2), nominal_tflops=round(t3fl / us / 1e6, 1))
        extra["conv3d_transpose_c128_k64_4x4x4_s2_4x14x14_b2"] = dict(
            per_layout=t3d, speedup_vs_nchw=round(t3d["NCHW"]["us"] / min(v["us"] for v in t3d.values()), 2),
            form="sub-pixel" if h.conv3d_transpose_weight_shape(d)[0] != 64 else "zero insertion",
            note="sub-pixel form: one forward 3-D convolution of x with 8*K output channels over the merged 3x3x3 window, then the "
                 "kernel that moves the eight phases into place")

        # a 1-D convolution (C1D: the C2D with H = R = 1): 256 channels, 9 taps, 2048 samples, batch 16, tuned like the others
        c1shape = alt.conv_desc(16, 256, 1, 2048, 256, 1, 9, in_dtype=alt.BF16, out_dtype=alt.BF16)
        c1shape.pad_h, c1shape.pad_w = 0, 4
        c1best, c1rep = h.tune_conv2d(c1shape, arena, arena.numel(), max_trials=0, warmup=3, reps=20)
        c1fl = 2.0 * 16 * 2048 * 256 * 256 * 9
        c1names = [c1rep.layout_name[i].value.decode() for i in range(c1rep.n_layouts)]
        extra["conv1d_c256_k9_l2048_b16"] = dict(
            variant=h.conv2d_variant_name(c1best, c1best.variant), layout=c1names[int(np.argmin([c1rep.layout_best_us[i] for i in range(c1rep.n_layouts)]))],
            tuned_us=round(float(c1rep.best_us), 2), default_layout_us=round(float(c1rep.default_us), 2),
            tflops=round(c1fl / float(c1rep.best_us) / 1e6, 1), trials=c1rep.trials,
            layout_us=dict(zip(c1names, [round(float(c1rep.layout_best_us[i]), 2) for i in range(c1rep.n_layouts)])))

    if want("budget"):
        # ------------------------------- budgeted search against the full one ----
        # the tuner with 48 measurements per layer (variants ranked by the cost estimate, measured best first)
        # against the exhaustive search over the same space
        bud = []
        for L in RESNET_LAYERS:
            shape = alt.conv_desc(16, L["C"], L["H"], L["W"], L["K"], L["R"], L["S"], stride=L["stride"], pad=L["pad"],
                                  in_dtype=alt.BF16, out_dtype=alt.BF16)
            res = {}
            for name, budget in (("48", 48), ("all", 0)):
                h.cache_clear()
                bbest, brep = h.tune_conv2d(shape, arena, arena.numel(), max_trials=budget, warmup=3, reps=20)
                res[name] = dict(us=round(float(brep.best_us), 2), trials=brep.trials,
                                 variant=h.conv2d_variant_name(bbest, bbest.variant))
            bud.append(dict(layer=L["name"], budget_48=res["48"], exhaustive=res["all"],
                            ratio=round(res["48"]["us"] / res["all"]["us"], 3)))
        h.cache_clear()
        extra["budgeted_search_b16"] = bud

    if attainable:
        extra["attainable"] = attainable

    # ------------------------------------------------------------ cpu baseline ----
    cpu = None
    if not args.no_cpu:
        import oracle
        oracle.build()
        # the whole step (the five layers at batch 16), passes repeated until about ten seconds of CPU work
        ops = []
        for li, L in enumerate(RESNET_LAYERS):
            x = f32_to_bf16_bits(normal_f32(0xA17 + 2 + li, (16, L["C"], L["H"], L["W"])))
            w = f32_to_bf16_bits(normal_f32(0xA17 + 102 + li, (L["K"], L["C"], L["R"], L["S"]), std=0.05))
            ops.append((L, x, w))
        t_total, f_total, passes = 0.0, 0.0, 0
        while t_total < 10.0 and passes < 40:
            for L, x, w in ops:
                t0 = time.perf_counter()
                oracle.conv2d(x, w, stride=L["stride"], pad=L["pad"])
                t_total += time.perf_counter() - t0
                f_total += conv_flops(16, **L)
            passes += 1
        cpu = dict(value=round(f_total / t_total / 1e12, 6), unit="TFLOP/s", cores=oracle.num_threads(),
                   kind="oracle", sample="the whole step (five layers, batch 16), %d passes, %.1f s" % (passes, t_total))

    out = dict(metric="conv2d/GEMM TFLOP/s (% bf16 MFMA peak); layout_transform GB/s (% HBM)",
               value=round(value, 2), unit="TFLOP/s", n_gpus=1, steps=int(head["steps_timed"]), warmup=args.warmup,
               ms_per_step=round(ms_per_step, 5), higher_is_better=True, scaling="weak", vs_baseline=None,
               dtype="bf16", data="synthetic",
               config=dict(workload="ResNet-50-style conv layers C64/56x56/3x3, C128/28x28/3x3, C256/14x14/3x3, "
                                    "C512/7x7/3x3, C256->64/56x56/1x1 at batch 16, bf16 in, fp32 accumulate, bf16 out, "
                                    "tuned layout per layer, inputs resident in HBM",
                           flops_per_step=step_flops, frac_bf16_mfma_peak=round(value / PEAK_BF16_TFLOPS, 4),
                           steps_requested=args.steps, launch=head["launch"][:60],
                           plan="tuned in this run" if tuned_now else "stored: " + os.path.relpath(args.plan, ROOT)),
               roofline=roofline, cpu_baseline=cpu, summary=summarise(extra))
    emit(out, extra)


def summarise(extra):
    """A few figures of each section for the final line (the sections themselves go to EXTRA_PATH)."""
    s = dict(layer_us=[p["us"] for p in extra["per_layer_b16"]],
             layer_us_cold_inputs=[p.get("us_cold_inputs") for p in extra["per_layer_b16"]],
             layer_frac_mfma=[p["frac_mfma_peak"] for p in extra["per_layer_b16"]],
             layer_speedup_vs_default_layout=[p["speedup_vs_default_layout_live"] for p in extra["per_layer_b16"]],
             one_stream_ms_per_step=extra["graph_replay_ms_per_step"])
    tr = extra.get("layout_transform")
    if tr:
        s["transform_cold_GBps_min_max"] = [min(t["GBps_hbm"] for t in tr), max(t["GBps_hbm"] for t in tr)]
    sc = extra.get("layout_transform_scaled")
    if sc:
        s["transform_16x_cold_GBps_min_max"] = [min(t["GBps_hbm"] for t in sc), max(t["GBps_hbm"] for t in sc)]
        s["transform_16x_cold_GBps_56x56"] = [t["GBps_hbm"] for t in sc if tuple(t.get("shape", ())[2:]) == (56, 56)][:4]
    gm = extra.get("gemm_bert")
    if gm:
        s["gemm_frac_mfma"] = [g["frac_mfma_peak"] for g in gm]
    big = extra.get("gemm_4096")
    if big:
        s["gemm_4096_frac_mfma"] = big["frac_mfma_peak"]
    cs = extra.get("conv_scaled_batch256_nhwc_bf16out")
    if cs:
        s["conv_b256_frac_mfma"] = [c["frac_mfma_peak"] for c in cs]
    ch = extra.get("chain")
    if ch:
        s["chain_us"] = ch["planned_total_us"]
    at = extra.get("attainable")
    if at:
        s["attainable"] = {k: at[k] for k in at if k.endswith("GBps") or k.endswith("TFLOPs")}
    s["extra_file"] = os.path.relpath(EXTRA_PATH, ROOT)
    return s


def final_line(out):
    """The one JSON line that ends the run: compact separators, below MAX_LINE_BYTES (whatever a
    summary list grows to, the headline fields survive: the summary is what gets dropped)."""
    line = json.dumps(out, separators=(",", ":"))
    if len(line) >= MAX_LINE_BYTES:
        out = dict(out)
        out["summary"] = dict(extra_file=out.get("summary", {}).get("extra_file"), dropped="line too long")
        line = json.dumps(out, separators=(",", ":"))
    if len(line) >= MAX_LINE_BYTES:
        raise SystemExit("bench.py: final line is %d bytes" % len(line))
    return line


def emit(out, extra):
    """Writes the sections to EXTRA_PATH (and to stdout, each on a line of its own, before the final line)."""
    try:
        os.makedirs(os.path.dirname(EXTRA_PATH), exist_ok=True)
        with open(EXTRA_PATH, "w") as f:
            json.dump(dict(headline=out, extra=extra), f, indent=1)
    except OSError:
        pass
    for k, v in extra.items():
        print("# extra.%s %s" % (k, json.dumps(v, separators=(",", ":"))))
    sys.stdout.flush()
    print(final_line(out))


if __name__ == "__main__":
    main()

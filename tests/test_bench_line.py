"""The benchmark's last stdout line is what the build driver parses: one JSON
object with the headline, `roofline` and `cpu_baseline`, short enough to survive
a bounded tail of the output whatever the other sections grow to."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def _headline():
    return dict(metric="conv2d/GEMM TFLOP/s (% bf16 MFMA peak); layout_transform GB/s (% HBM)", value=612.34,
                unit="TFLOP/s", n_gpus=1, steps=2000, warmup=20, ms_per_step=0.02685, higher_is_better=True,
                scaling="weak", vs_baseline=None, dtype="bf16", data="synthetic",
                config=dict(workload="w" * 260, flops_per_step=16441671680, frac_bf16_mfma_peak=0.2449,
                            steps_requested=20, launch="l" * 60, plan="stored: workloads/tuned_plan_gfx950.json"),
                roofline=dict(bound="mfma", achieved=499.7, peak=2500.0, unit="TFLOP/s", frac=0.1999, traffic=12079104,
                              traffic_source="stored rocprofv3 --pmc runs of this kernel and grid",
                              kernel="bf16_64x32x32_direct_w1x1x8_s4_k1", layer="c512_7_3x3", us_per_launch=7.404,
                              flops_per_launch=3699376128, frac_vs_attainable=0.2213, frac_own_ceiling=0.1999),
                cpu_baseline=dict(value=0.034, unit="TFLOP/s", cores=16, kind="oracle",
                                  sample="the whole step (five layers, batch 16), 22 passes, 10.3 s"))


def test_final_line_parses_and_is_short():
    out = _headline()
    extra = dict(per_layer_b16=[dict(us=6.7, frac_mfma_peak=0.22, speedup_vs_default_layout_live=9.1)] * 5,
                 graph_replay_ms_per_step=0.0401,
                 layout_transform=[dict(GBps_hbm=3000.0 + i) for i in range(24)],
                 layout_transform_scaled=[dict(GBps_hbm=5500.0 + i) for i in range(24)],
                 gemm_bert=[dict(frac_mfma_peak=0.25)] * 4, gemm_4096=dict(frac_mfma_peak=0.46),
                 conv_scaled_batch256_nhwc_bf16out=[dict(frac_mfma_peak=0.37)] * 2, chain=dict(planned_total_us=23.0),
                 attainable=dict(copy_GBps=4970.0, read_GBps=5000.0, write_GBps=5000.0, mfma_bf16_TFLOPs=2250.0,
                                 compute_units=256))
    out["summary"] = bench.summarise(extra)
    line = bench.final_line(out)
    assert "\n" not in line and len(line) < bench.MAX_LINE_BYTES
    back = json.loads(line)
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "dtype", "config", "roofline",
                "cpu_baseline"):
        assert key in back
    assert back["roofline"]["frac"] == 0.1999 and back["cpu_baseline"]["cores"] == 16


def test_final_line_drops_the_summary_before_the_headline():
    out = _headline()
    out["summary"] = dict(extra_file="gpurun_out/bench_extra.json", junk=list(range(2000)))
    line = bench.final_line(out)
    back = json.loads(line)
    assert len(line) < bench.MAX_LINE_BYTES and "junk" not in back["summary"] and back["roofline"] and back["cpu_baseline"]


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr


@pytest.mark.gpu
def test_bench_quick_run_ends_in_a_parsable_line():
    """The driver's own command line (20 steps, 5 warm-up), without the extra sections and the CPU leg."""
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "20", "--warmup", "5", "--quick",
                        "--no-cpu"], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    last = r.stdout.strip().splitlines()[-1]
    back = json.loads(last)
    assert len(last) < bench.MAX_LINE_BYTES
    assert back["steps"] >= 20 and back["ms_per_step"] * back["steps"] >= 45.0      # timed for at least ~50 ms
    assert back["roofline"]["bound"] == "mfma" and 0 < back["roofline"]["frac"] < 1

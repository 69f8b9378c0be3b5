"""CPU-only checks of the benchmark's output line: whatever the tables hold, the last stdout line stays a
single JSON object below 2 KB that carries the headline, the roofline of the dominant kernel and the CPU figure."""
import json

import bench
import workloads as wl


def _fake_launches(steps=20):
    names = ["f32_64x64_w32x32_dma", "f32_128x64_w64x32_dma", "f32_128x128_w64x64_dma", "f32_128x128_w64x64_dma"]
    ms = [0.0231, 0.129, 0.958, 7.4]
    return [(names[i], n, 2.0 * n ** 3, ms[i]) for _ in range(steps) for i, n in enumerate(wl.FP32_SQUARES)]


def _fake_result():
    return {"metric": "GEMM TFLOP/s (TOPS for int8) and % of MFMA peak per dtype, 1 MI355X", "value": 147.173,
            "unit": "TFLOP/s", "n_gpus": 1, "steps": 20, "warmup": 3, "ms_per_step": 8.5361, "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
            "config": {"workload": "fp32 square GEMM sweep M=N=K in {1024,2048,4096,8192}, column-major, "
                                   "alpha=1.5, beta=0.5, A/B/C i.i.d. U[-1,1)", "wall_s": 0.171},
            "pct_of_peak": 93.56, "roofline": bench.roofline_of_dominant_kernel(_fake_launches()),
            "cpu_baseline": {"value": 0.006562, "unit": "TFLOP/s", "cores": 16, "kind": "oracle",
                             "sample": "first 2048 columns of the 4096^3 fp32 case (alpha=1.5, beta=0.5), 10.5 s"},
            "detail_file": "gpurun_out/bench_detail.json"}


def _fake_detail():
    rows = []
    for cfg, dt, lay, sizes in (("c2 fp32 square", "f32", "col", wl.FP32_SQUARES), ("c3 fp16 square", "f16", "row", wl.FP16_SQUARES),
                                ("bf16 square (beyond the configurations)", "bf16", "row", wl.FP16_SQUARES[1:])):
        for n in sizes:
            rows.append({"config": cfg, "dtype": dt, "layout": lay, "M": n, "N": n, "K": n, "kernel": "x" * 30, "split": 1,
                         "us": 123456.78, "tflops": 1234.56, "pct_peak": 49.04})
    for (M, N, K) in wl.IM2ROW_HEADLINE:
        for lay in ("col", "row"):
            rows.append({"config": "c4 im2row", "dtype": "f32", "layout": lay, "M": M, "N": N, "K": K, "kernel": "k", "split": 6,
                         "us": 11.16, "tflops": 20.72, "pct_peak": 13.17})
    for (M, N, K) in wl.INT8_SHAPES:
        for lay in ("col", "row"):
            rows.append({"config": "c5 int8", "dtype": "i8", "layout": lay, "M": M, "N": N, "K": K, "kernel": "k", "split": 1,
                         "us": 64.09, "tflops": 2144.56, "pct_peak": 42.61})
    models = {name: {"dtype": "f32", "sum_us": 12345.6, "tflops": 123.45, "pct_peak": 50.12, "layers": [{"M": 1}] * 20}
              for name in ("resnet50_v1.5", "vgg16", "resnet50_v1.5_f16", "vgg16_f16", "resnet50_v1.5_i8", "vgg16_i8")}
    solo = {d: {"kernel": "k" * 30, "solo_tflops": 1657.3, "pct_peak": 65.9,
                "registers_only": {"kernel": "r", "solo_tflops": 1721.9, "pct_peak": 68.4}} for d in ("f32", "f16", "i8", "bf16")}
    return {"per_shape": rows, "im2row_models": models, "conv_im2row": [{"M": 1}] * 15, "solo_mode": solo}


def test_line_is_short_and_complete():
    text = bench.compact_line(_fake_result(), _fake_detail())
    assert "\n" not in text and len(text) < 2048
    line = json.loads(text)
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline", "summary"):
        assert key in line
    assert line["config"]["workload"].startswith("fp32 square GEMM sweep")
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic", "kernel", "launches", "avg_launch_ms"):
        assert key in line["roofline"]
    for key in ("f16_8192", "i8_4096", "im2row_headline_us", "model_resnet50_v1.5", "model_vgg16", "solo_pct_peak"):
        assert key in line["summary"]
    assert len(line["summary"]["im2row_headline_us"]) == 6
    # the tables themselves stay out of the line
    assert "per_shape" not in line and "im2row_models" not in line and "conv_im2row" not in line


def test_line_without_tables():
    line = json.loads(bench.compact_line(_fake_result(), {}))
    assert "summary" not in line and line["value"] == 147.173


def test_roofline_is_the_dominant_kernels_own_rate():
    r = bench.roofline_of_dominant_kernel(_fake_launches(steps=3))
    assert r["kernel"] == "f32_128x128_w64x64_dma" and r["launches"] == 6 and r["sizes"] == [4096, 8192]
    flop = 2.0 * 4096 ** 3 + 2.0 * 8192 ** 3
    assert abs(r["achieved"] - flop / ((0.958 + 7.4) * 1e-3) / 1e12) < 1e-3
    assert abs(r["frac"] - r["achieved"] / 157.3) < 1e-4
    assert abs(r["avg_launch_ms"] - (0.958 + 7.4) / 2) < 1e-4
    # counter figure: the mean over that kernel's launches, null as soon as an unprofiled kernel is selected
    assert abs(r["traffic"] - (844.2e6 + 67.1e6 + 6684.6e6 + 268.4e6) / 2) < 1.0
    other = [("f32_new_kernel", n, f, ms) for (_, n, f, ms) in _fake_launches(steps=1)]
    assert bench.roofline_of_dominant_kernel(other)["traffic"] is None

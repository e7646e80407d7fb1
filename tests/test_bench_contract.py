"""bench.py's command line and output contract: one JSON line with the agreed keys, one GPU only, and the
algorithmic work it prices the kernels with (checked on the host against numbers worked out by hand)."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2", "--steps", "1", "--warmup", "0"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_algorithmic_work_of_the_headline_stage():
    import bench
    from synth_inputs import workloads as W
    w = W.mlp_wide(width=4096, mb=256, n=8)
    P = 2 * (4096 * 4096 + 4096)
    assert bench.kernel_work("update", w, 1, True) == (8.0 * P, 28.0 * P)            # 28 bytes per parameter
    fl, by = bench.kernel_work("fprop", w, 1, True)                                  # 8 micro-batches x 2 layers
    assert fl == 16 * 2.0 * 256 * 4096 * 4096
    assert by == 16 * 2.0 * (256 * 4096 + 4096 * 4096 + 2 * 256 * 4096)              # x, W in; a, act' out (bf16)
    fl, by = bench.kernel_work("dgrad", w, 1, True)
    assert fl == 2 * 2.0 * 2048 * 4096 * 4096
    assert bench.kernel_work("dgrad", w, 0, False)[0] == fl / 2                       # no input gradient at stage 0's first layer
    fl, by = bench.kernel_work("wgrad", w, 1, True)
    assert fl == 2 * 2.0 * 2048 * 4096 * 4096 and by == 2 * (2.0 * 2 * 2048 * 4096 + 4.0 * 4096 * 4096)


def test_algorithmic_work_of_a_strided_convolution():
    import bench
    from synth_inputs import workloads as W
    l = W.Conv2d(256, 256, 8, 8, "none", stride=2)
    fl, by = bench.layer_work("fprop", l, rows=512, mb=128)
    assert fl == 2.0 * 128 * 16 * (9 * 256) * 256                                    # 16 output pixels per image
    assert by == 2.0 * (128 * 64 * 256 + 9 * 256 * 256 + 2 * 128 * 16 * 256)         # 64 input pixels per image read
    assert bench.layer_work("wgrad", W.Subsample2(256, 8, 8), 512, 128) == (0.0, 0.0)


def test_algorithmic_work_of_the_stem_and_head_layers():
    import bench
    from synth_inputs import workloads as W
    stem = W.Conv2d(3, 64, 64, 64, "none", k=7, stride=2, pad=3)
    fl, by = bench.layer_work("fprop", stem, rows=512, mb=128)
    assert fl == 2.0 * 128 * 1024 * (49 * 3) * 64                                    # 32 x 32 output pixels, 49 taps
    assert by == 2.0 * (128 * 4096 * 3 + 49 * 3 * 64 + 2 * 128 * 1024 * 64)
    fl, _ = bench.layer_work("wgrad", stem, rows=512, mb=128)
    assert fl == 2.0 * 512 * 1024 * 147 * 64
    assert bench.layer_work("fprop", W.AvgPool(2048, 4), 512, 128) == (0.0, 0.0)
    w = W.resnet_stages()
    _, by = bench.kernel_work("pool", w, 3, True)                                    # stage 3: one subsampling, the average pooling
    sub = 2.0 * 512 * (1024 * 16 / 2) + 2.0 * 512 * (1024 * 16 / 4 + 1024 * 16)
    avg = 2 * 2.0 * 512 * (2048 * 4 + 2048)
    assert by == sub + avg
    assert bench.kernel_work("dgrad", w, 0, False)[0] < bench.kernel_work("dgrad", w, 0, True)[0]   # no input gradient of the stem


@pytest.mark.gpu
def test_bench_prints_one_json_line_with_the_contract_keys():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "3", "--warmup", "1", "--width", "512",
                        "--mb", "64", "--n", "2", "--cpu-minibatches", "1"], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    out = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in out, key
    assert out["n_gpus"] == 1 and out["steps"] == 3 and out["warmup"] == 1 and out["vs_baseline"] is None
    assert out["unit"] == "samples/s" and out["higher_is_better"] is True and out["data"] == "synthetic"
    assert "workload" in out["config"] and "model" not in out["config"]
    assert abs(out["value"] - 64 * 2 / (out["ms_per_step"] * 1e-3)) <= 1e-3 * out["value"]
    rf = out["roofline"]
    assert rf["bound"] in ("hbm", "mfma", "alu") and rf["unit"] in ("GB/s", "TFLOP/s")
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-3 and rf["traffic"] is None   # measured for the default workload only
    cb = out["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["cores"] >= 1 and cb["value"] > 0 and cb["sample"]

"""The benchmark's output line: one JSON object with the fields the driver reads, the roofline
of the dominant kernel and the oracle's timing; more than one GPU is refused with a message."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*flags):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *flags], cwd=ROOT,
                          capture_output=True, text=True, timeout=300)


@pytest.mark.gpu
def test_bench_line_has_the_contract_fields():
    r = run_bench("--steps", "3", "--warmup", "1", "--no-large-quantize", "--no-square", "--no-conv",
                  "--no-sweep", "--no-others", "--no-requant", "--no-resnet18", "--no-fallbacks", "--dist-steps", "20", "--cpu-rows",
                  "2048")
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1, "exactly one line on stdout"
    d = json.loads(lines[0])
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1
    assert d["higher_is_better"] is True and d["scaling"] == "weak" and d["vs_baseline"] is None
    assert d["data"] == "synthetic" and d["unit"] == "TOPS" and isinstance(d["dtype"], str)
    assert d["value"] > 0 and d["ms_per_step"] > 0
    M, K, N = 65536, 1152, 128
    assert abs(d["value"] - 3 * 2.0 * M * K * N / (d["ms_per_step"] * 1e-3) / 1e12) < 1e-6 * d["value"]
    assert "workload" in d["config"] and "model" not in d["config"]
    roof = d["roofline"]
    assert roof["bound"] in ("hbm", "mfma", "alu") and roof["unit"] in ("GB/s", "TFLOP/s", "TOP/s")
    assert roof["peak"] == 8000.0 and 0 < roof["frac"] < 1
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-9
    assert "traffic" in roof and ("traffic_source" in roof or roof["traffic"] is None)
    dist = d["step_time_distribution"]
    for leg in ("warm", "cold"):
        assert dist[leg]["steps"] == 20
        assert 0 < dist[leg]["min_ms"] <= dist[leg]["median_ms"] <= dist[leg]["max_ms"]
    assert dist["cold"]["median_ms"] >= dist["warm"]["min_ms"]
    cpu = d["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["value"] > 0 and cpu["cores"] >= 1 and cpu["sample"]


def test_more_than_one_gpu_is_refused():
    r = run_bench("--gpus", "2")
    assert r.returncode != 0
    assert "one GPU" in r.stderr


@pytest.mark.gpu
def test_bench_line_has_the_extra_legs():
    """The standalone quantizer legs (both axes, block orders 64 and 256) and the step lines of
    the other layer workloads."""
    r = run_bench("--steps", "2", "--warmup", "1", "--no-square", "--no-conv", "--no-sweep",
                  "--dist-steps", "0", "--no-cpu-baseline")
    assert r.returncode == 0, r.stderr[-2000:]
    d = json.loads([ln for ln in r.stdout.splitlines() if ln.strip()][0])
    assert d["step_time_distribution"] is None
    q = d["quantize_1GiB"]
    for leg in ("axis1_n64", "axis0_n64", "axis1_n256", "axis0_n256"):
        assert 0 < q[leg]["pass1_frac_of_hbm_peak"] < 1 and 0 < q[leg]["pass2_frac_of_hbm_peak"] < 1
    assert q["pass1_GBps"] == q["axis1_n64"]["pass1_GBps"]
    others = d["other_workloads"]
    assert set(others) == {"har", "resnet_k576"}
    for o in others.values():
        assert o["ms_per_step"] > 0 and o["TOPS"] > 0 and o["kernels_us"]
    # the 21 layer shapes of a ResNet-18 training step
    r18 = d["resnet18_batch128"]
    assert r18["layers"] == 21 and len(r18["per_shape"]) == 12 and r18["matmul_ms_per_training_step"] > 0
    assert 420 < r18["GOP_per_training_step"] < 430
    # the paths behind the fast kernels' shape limits carry a figure each
    fb = d["fallback_paths"]
    assert set(fb) == {"fwd_K_multiple_of_8_not_32", "fwd_K_not_multiple_of_8", "fwd_mixed_4bit_8bit",
                       "quantize_axis0_cols_not_multiple_of_4", "step_had_block_128"}
    assert all(v["ms"] > 0 and v["kernels_us"] for v in fb.values())
    assert "gemm_i4_fwd" in fb["fwd_K_multiple_of_8_not_32"]["kernels_us"]
    assert any(k.startswith("gemm_tiled") for k in fb["fwd_K_not_multiple_of_8"]["kernels_us"])
    # the matmul's test of its tiles: one figure where nearly every tile passes, one where none does
    tt = d["tile_test"]
    assert tt["fwd_layer_codes_us"] > 0 and tt["fwd_codes_uniform_over_the_range_us"] > 0
    # the forward product under the second reading of the accumulator: two passes, no tile sums stored
    rq = d["requant_fwd"]
    assert rq["tile_sums_materialised_bytes"] == 0 and rq["workspace_bytes"] < 64 << 20
    assert 0 < rq["matmul_us"] < 1000 and {"requant_tile_sums", "requant_quantize_sum"} <= set(rq["kernels_us"])

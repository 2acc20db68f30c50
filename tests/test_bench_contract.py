"""The benchmark's contract: one GPU only, one JSON line with the agreed keys, and the derived peaks it prices against."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert p.returncode != 0
    assert "one GPU" in p.stderr and p.stdout.strip() == ""


def test_peaks_and_algorithmic_units():
    sys.path.insert(0, ROOT)
    import bench
    assert bench.HBM_PEAK_GBS == 8000.0 and bench.FP64_VECTOR_PEAK_TFLOPS == 78.6
    # point-cloud pass, d = 3: 6 plain vector instructions (4 issue cycles) and one v_exp_f32 (8) per pair and wave64
    pairs, flop = bench.points_alu_peak(3)
    assert abs(pairs - 1024 * 2.4e9 * 64 / 32) < 1.0 and flop == 9
    assert abs(bench.EXP_PEAK_PER_S - 1024 * 64 * 2.4e9 / 8) < 1.0
    # the fp64 vector peak is the chip's unit counts: 256 compute units x 4 SIMDs x 16 lanes x 2 flop x 2.4 GHz
    assert abs(256 * 4 * 16 * 2 * 2.4e9 / 1e12 - bench.FP64_VECTOR_PEAK_TFLOPS) < 0.1


@pytest.mark.gpu
@pytest.mark.parametrize("workload,extra", [("c1", []), ("c2", ["--steps", "20", "--warmup", "5"])])
def test_bench_prints_one_json_line_with_the_contract_keys(workload, extra):
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", workload, *extra], capture_output=True,
                       text=True, timeout=600, cwd=ROOT)
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [l for l in p.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["higher_is_better"] is True and d["vs_baseline"] is None and d["data"] == "synthetic"
    assert "workload" in d["config"] and "model" not in d["config"]
    assert abs(d["value"] - d["steps"] / (d["ms_per_step"] * 1e-3 * d["steps"])) <= 1e-6 * d["value"]
    r = d["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in r, key
    assert r["bound"] == "hbm" and r["peak"] == 8000.0 and r["unit"] == "GB/s"
    if workload == "c2":
        assert d["steps"] == 20 and r["kernel"] in ("k_resident", "k_persist") and 0.3 < r["frac"] < 1.0
        assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-9
        assert 0.3 < d["iteration"]["frac_iteration"] <= r["frac"] + 0.05
    b = d["cpu_baseline"]
    assert b["kind"] == "oracle" and b["cores"] >= 1 and b["value"] > 0 and "sample" in b


@pytest.mark.gpu
def test_read_rate_calibration():
    """The measurement aid behind `bench.py --calibrate-read`: a plain streaming read of a device buffer reaches a
    plausible fraction of the published peak (a few TB/s on an MI355X; anything above 0.2 TB/s and below the peak passes,
    so that the test holds on smaller devices), and invalid arguments are refused."""
    import torch
    from paper_2605_00837_amd import binding as fs
    buf = torch.zeros(128 << 20, dtype=torch.uint8, device="cuda")
    us = min(fs.fs_read_rate(buf, 10) for _ in range(3))
    rate = buf.numel() / (us * 1e-6) / 1e12
    assert 0.2 < rate < 8.0, rate
    with pytest.raises(fs.FsError):
        fs.fs_read_rate(buf[:8], 10)
    with pytest.raises(fs.FsError):
        fs.fs_read_rate(buf, 0)

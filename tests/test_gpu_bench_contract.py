"""The benchmark's output contract, on a small instance: one JSON line with the metric, the roofline
object of the dominant kernel and the oracle's CPU baseline; more than one GPU is refused."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench(*args):
    proc = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")] + list(args), cwd=ROOT,
                          stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=600)
    return proc


@pytest.mark.parametrize("mode", ["sym", "mat", "otf"])
def test_bench_prints_one_json_line_with_roofline_and_cpu_baseline(mode):
    proc = _bench("--mode", mode, "--n", "3000", "--steps", "2", "--warmup", "1", "--cpu-sample", "600")
    assert proc.returncode == 0, proc.stderr[-2000:]
    lines = [l for l in proc.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    out = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
                "scaling", "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in out, key
    assert out["n_gpus"] == 1 and out["steps"] == 2 and out["warmup"] == 1
    assert out["unit"] == "ms" and out["higher_is_better"] is False and out["vs_baseline"] is None
    assert out["value"] > 0 and out["value"] == pytest.approx(out["ms_per_step"])
    assert "workload" in out["config"] and out["config"]["iters_run"] == 50
    roof = out["roofline"]
    assert roof["bound"] in ("hbm", "mfma") and roof["unit"] in ("GB/s", "TFLOP/s")
    assert roof["frac"] == pytest.approx(roof["achieved"] / roof["peak"])
    assert roof["traffic"] is None                     # the measured byte counts belong to n = 50000 only
    cpu = out["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["cores"] >= 1 and cpu["value"] > 0 and cpu["unit"] == "ms"
    # the oracle timed by stage at the benchmark's own n, the small-n extrapolation beside it
    assert set(cpu["stages"]) == {"build_s", "product_s_per_iteration", "vector_s_per_iteration", "derivative_s"}
    assert cpu["extrapolated_from_small_n"]["value"] > 0
    if mode == "sym":
        # the default line also carries the other two product modes, measured in the same run
        mat, otf = out["roofline_mat"], out["roofline_otf"]
        assert mat["bound"] == "hbm" and mat["unit"] == "GB/s" and mat["peak"] == 8000.0
        assert otf["bound"] == "mfma" and otf["unit"] == "TFLOP/s"
        for leg in (mat, otf):
            assert leg["frac"] == pytest.approx(leg["achieved"] / leg["peak"]) and leg["ms_per_call"] > 0
            assert leg["launches"] == 3 * 50
            assert leg["logdet"] == pytest.approx(out["config"]["logdet"], rel=1e-3)
    else:
        assert "roofline_mat" not in out and "roofline_otf" not in out


def test_bench_refuses_more_than_one_gpu():
    proc = _bench("--gpus", "2")
    assert proc.returncode != 0
    assert "one GPU" in (proc.stderr + proc.stdout)

"""The measurement script's contract: one GPU only, the byte counts it prices the kernels with, and (on a GPU)
the one JSON line with its `roofline` and `cpu_baseline` objects."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402  (imports neither torch nor the library at module level)


def run_bench(*flags, timeout=300):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *flags], cwd=ROOT, capture_output=True,
                          text=True, timeout=timeout)


def test_more_than_one_gpu_is_refused_with_a_message():
    res = run_bench("--gpus", "2")
    assert res.returncode != 0 and "ONE GPU" in res.stderr and res.stdout.strip() == ""


def test_algorithmic_bytes_per_pair_coordinate():
    """Per pair-coordinate: the gossip pass reads X and W of both nodes (16 B) and writes both X (8 B); the one-pass
    round reads X, a, c of both (24 B); a b-bit code is b/8 B per node, written always and read when the read is stale."""
    f = bench.algorithmic_bytes_per_pair_coordinate
    assert f("gossip", 4, 1.0) == 16 + 8 + 1 + 1
    assert f("gossip", 8, 0.0) == 16 + 8 + 2
    assert f("round", 4, 1.0) == 24 + 8 + 1 + 1
    assert f("round", 8, 1.0) == 24 + 8 + 2 + 2
    assert f("round", 8, 0.5) == 24 + 8 + 2 + 1
    # in place: one matrix, nothing pending to read in the gossip pass
    assert f("gossip", 4, 1.0, inplace=True) == 8 + 8 + 1 + 1


def test_vector_alu_peak_is_the_chips_issue_rate():
    assert bench.VALU_PEAK_TLANEOPS == pytest.approx(256 * 4 * 16 * 2.4e9 / 1e12)
    fixed, per_step = bench.VALU_PER_NODE_TILE_8BIT
    assert fixed > 0 and per_step > 0


@pytest.mark.gpu
def test_the_json_line():
    res = run_bench("--gpus", "1", "--steps", "3", "--warmup", "2", "--no-configs", "--config-steps", "2")
    assert res.returncode == 0, res.stderr[-2000:]
    lines = [ln for ln in res.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1                                    # ONE JSON line
    out = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in out, key
    assert out["n_gpus"] == 1 and out["steps"] == 3 and out["warmup"] == 2 and out["vs_baseline"] is None
    assert out["data"] == "synthetic" and "config 4" in out["config"]["workload"] and "model" not in out["config"]
    roof = out["roofline"]
    assert roof["bound"] == "hbm" and roof["peak"] == 8000.0 and roof["unit"] == "GB/s"
    assert roof["frac"] == pytest.approx(roof["achieved"] / roof["peak"]) and 0.3 < roof["frac"] < 1.0
    # whole-step throughput cannot beat what the kernel alone moves
    assert out["ms_per_step"] >= roof["ms_per_launch"]
    cpu = out["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["value"] > 0 and cpu["cores"] >= 1 and cpu["sample"]

"""bench.py's command-line contract: the one JSON line with its required keys, and the refusal of more than one GPU."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, BENCH, "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "--gpus 1" in r.stderr and not r.stdout.strip()


def test_algorithmic_flops_of_the_benchmarked_shard():
    """3 x (2 M (h 3h_l + h_l h + h f_l + f_l h) + 2 b n_l s^2 d) for the GPT-3 13B TP=8 shard."""
    sys.path.insert(0, ROOT)
    import bench
    from paper_2409_15241_amd import synth
    sc = synth.WORKLOADS["gpt3-13b"]
    M, h, hl, fl, b, nl, s, d = 8192, 5120, 640, 2560, 4, 5, 2048, 128
    want = 3 * (2 * M * (h * 3 * hl + hl * h + h * fl + fl * h) + 2 * b * nl * s * s * d)
    assert bench.algorithmic_flops(sc) == want
    assert abs(want / 1e9 - 1997.16) < 0.01


@pytest.mark.gpu
def test_bench_prints_one_json_line_with_the_contract_keys():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    r = subprocess.run([sys.executable, BENCH, "--workload", "tiny", "--steps", "3", "--warmup", "1", "--stack-layers", "2",
                        "--no-other-workloads"], capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
              "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["higher_is_better"] is True
    assert d["unit"] == "TFLOP/s" and d["dtype"] == "bf16" and d["data"] == "synthetic" and d["vs_baseline"] is None
    assert d["config"]["workload"] == "tiny" and "model" not in d["config"]
    assert d["value"] > 0 and d["ms_per_step"] > 0
    rf = d["roofline"]
    for k in ("bound", "achieved", "peak", "unit", "frac", "traffic", "traffic_source"):
        assert k in rf, k
    assert d["other_workloads"] is None
    assert d["measured_mfma_ceiling"]["value"] > 500.0 and 0.0 < d["pct_of_measured_mfma_ceiling"] < 100.0
    assert rf["bound"] == "mfma" and rf["peak"] == 2500.0 and abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-9
    cb = d["cpu_baseline"]
    for k in ("value", "unit", "cores", "kind", "sample"):
        assert k in cb, k
    assert cb["kind"] == "oracle" and cb["value"] > 0 and cb["cores"] >= 1


@pytest.mark.gpu
def test_bench_graph_replay_mode_prints_its_line_with_a_roofline():
    """--graph times replays of the captured step; the per-launch roofline pass runs the eager step beside it."""
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    r = subprocess.run([sys.executable, BENCH, "--workload", "tiny", "--steps", "3", "--warmup", "1", "--graph",
                        "--no-other-workloads", "--no-cpu-baseline", "--no-ceiling"],
                       capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    d = json.loads([l for l in r.stdout.splitlines() if l.strip()][-1])
    assert d["value"] > 0 and d["roofline"]["achieved"] > 0 and d["roofline"]["launches_per_step"] >= 1


def test_bench_refuses_graph_capture_with_a_pool_the_library_does_not_capture():
    r = subprocess.run([sys.executable, BENCH, "--workload", "tiny", "--graph", "--streams", "3"],
                       capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert r.returncode == 2 and "--graph is limited" in r.stderr and not r.stdout.strip()

"""Host-side checks of bench.py's output contract (no GPU): the line it prints carries the
required keys, stays short, and a multi-GPU request is refused with a message."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _fake_record():
    roof = {"kernel": "pass1_dots_gram", "bound": "hbm", "achieved": 6186.387312, "peak": 8000.0, "unit": "GB/s",
            "frac": 0.773298414, "traffic": 2960200000.0, "traffic_source": "profiles/x.txt " * 8,
            "avg_launch_ms": 0.477953, "algorithmic_bytes_per_launch": 2956800000.0}
    cpu = {"value": 148.29072, "unit": "examples/s", "cores": 1, "kind": "oracle", "sample": "first 960 pairs",
           "seconds": 12.9, "host_cores_available": 16, "signs_agree_with_gpu_on_sample": True,
           "in_margin_flips_on_sample": 0}
    others = []
    for k in range(8):
        others.append({"workload": "w%d" % k, "m": 32, "n": 1024, "d": 1 << 20, "examples": 32768, "steps": 3,
                       "warmup": 1, "value": 615037.123456, "unit": "examples/s", "ms_per_step": 53.2781234,
                       "balancer_hbm_frac": 0.665067, "roofline": dict(roof), "cpu_baseline": dict(cpu),
                       "kernels": {"a": {"avg_launch_ms": 0.1, "achieved_GBs": 5000.0}},
                       "inputs_flushed_to_hbm": {"value": 1.0, "ms_per_step": 2.0, "steps": 2,
                                                 "balancer_hbm_frac": 0.62, "generator_ms_per_step": 3.0},
                       "note": "short rows: bound by the chain of dependent launches"})
    return {"metric": "examples balanced/sec per epoch at m workers x d params", "value": 68675.3123, "unit": "examples/s",
            "n_gpus": 1, "steps": 20, "warmup": 5, "ms_per_step": 238.5721, "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
            "config": {"workload": "c4_resnet18", "m": 32, "n": 512, "d": 11200000},
            "bytes_per_example": 93800000.0, "balancer_achieved_GBs": 6441.7, "balancer_hbm_frac": 0.805,
            "roofline": roof, "kernels": {"pass1_dots_gram": {"avg_launch_ms": 0.478, "achieved_GBs": 6186.0}},
            "cpu_baseline": cpu, "workloads": others}


def test_compact_line_keeps_the_contract_and_stays_short():
    sys.path.insert(0, ROOT)
    import bench
    line = bench.compact_line(_fake_record())
    text = json.dumps(line)
    assert len(text) < 6000
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
                "scaling", "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline", "workloads"):
        assert key in line
    assert line["config"]["workload"] == "c4_resnet18" and "model" not in line["config"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in line["roofline"]
    assert abs(line["roofline"]["frac"] - line["roofline"]["achieved"] / line["roofline"]["peak"]) < 1e-5
    for key in ("value", "unit", "cores", "kind", "sample"):
        assert key in line["cpu_baseline"]
    assert line["cpu_baseline"]["kind"] == "oracle"
    assert len(line["workloads"]) == 8
    for w in line["workloads"]:
        for key in ("workload", "value", "ms_per_step", "kernel", "frac", "cpu_baseline"):
            assert key in w
    assert json.loads(text) == line          # plain JSON types only


def test_more_than_one_gpu_is_refused_with_a_message():
    proc = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                          capture_output=True, text=True, timeout=120)
    assert proc.returncode != 0
    assert "ONE GPU" in proc.stderr and proc.stdout.strip() == ""
    env = dict(os.environ, WORLD_SIZE="2")
    proc = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True,
                          timeout=120, env=env)
    assert proc.returncode != 0 and "ONE GPU" in proc.stderr

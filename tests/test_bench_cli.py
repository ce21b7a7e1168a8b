"""Host-side checks of bench.py that need no GPU: the multi-GPU refusal and the shape of the CPU-baseline leg."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, cwd=ROOT)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_cpu_baseline_leg_runs_the_oracle_on_a_bounded_sample():
    sys.path.insert(0, ROOT)
    import bench
    b = bench.cpu_baseline_layer("short")
    assert b["kind"] == "oracle" and b["unit"] == "tokens/s" and b["value"] > 0 and b["cores"] >= 1
    assert "512 tokens" in b["sample"]

"""Host-side behaviour of bench.py that needs no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_cpu_baseline_sample_is_bounded():
    """The CPU leg takes every tree of a small workload and a sample of whole trees of a large one."""
    sys.path.insert(0, ROOT)
    import bench
    from paper_1809_00832_amd import synth
    small = bench.cpu_baseline(synth.workload("tiny"))
    assert small["kind"] == "oracle" and small["unit"] == "trees/s" and small["value"] > 0 and "all 4 trees" in small["sample"]
    big = bench.cpu_baseline(synth.workload("sentence"), max_nodes=300)
    assert "of the 25 trees" in big["sample"] and big["cores"] >= 1

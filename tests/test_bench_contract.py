"""The benchmark's command line contract that can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr or "1 GPU" in r.stderr or "single" in r.stderr.lower()
    assert r.stdout.strip() == ""                      # no JSON line


def test_backward_of_other_layer_kinds_over_deduplicated_frontiers_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--model", "gat", "--backward", "--dedup"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "backward" in r.stderr

"""Command-line contract of bench.py that needs no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                         stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert res.returncode != 0
    assert "single-GPU" in res.stdout and "--gpus 1" in res.stdout
    assert "{" not in res.stdout                      # no result line


def test_help_lists_the_experiments():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--help"],
                         stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert res.returncode == 0
    for flag in ("--steps", "--warmup", "--gpus", "--block-sizes", "--table1", "--sgemm", "--minibatch",
                 "--rotating", "--bprop-data", "--bprop-filter", "--vgg16", "--variant-sweep", "--tail-cuts", "--tail-map"):
        assert flag in res.stdout, flag

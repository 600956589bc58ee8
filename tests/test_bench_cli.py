"""bench.py's command line, as far as it can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    """The hot path is a single-GPU kernel path: --gpus N > 1 exits with a message that says so,
    before anything touches a device."""
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert p.returncode != 0
    assert "one GPU" in (p.stdout + p.stderr)
    assert "{" not in p.stdout  # no result line


def test_help_lists_the_workloads():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--help"], capture_output=True, text=True, timeout=120)
    assert p.returncode == 0
    for w in ("c3_prefill", "c4_decode", "c2_ffn", "c5_block", "--decode-only", "--no-sub"):
        assert w in p.stdout

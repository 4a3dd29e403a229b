"""bench.py's command line on a machine without a GPU: more than one GPU is refused with a message
(this build runs on one GPU: no sharding, no collectives)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2", "--steps", "1", "--warmup", "0"],
                       capture_output=True, text=True, timeout=120)
    assert p.returncode != 0
    assert "ONE GPU" in p.stderr and p.stdout.strip() == ""

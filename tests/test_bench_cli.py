"""bench.py's command line where no GPU is needed: more than one GPU is refused with a message that says why
(one process drives one GPU here; nothing in this build uses a second)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=300)
    assert res.returncode != 0
    assert "ONE GPU" in (res.stderr + res.stdout)

"""bench.py's command line, as far as it can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    """This build measures one GPU; asking for more exits with a message that says so (and no JSON line)."""
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    text = r.stdout + r.stderr
    assert "one GPU" in text or "1 GPU" in text or "single GPU" in text, text
    assert not any(l.startswith("{") for l in r.stdout.splitlines())

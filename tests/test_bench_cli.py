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


def test_recorded_traffic_of_the_dominant_kernel_comes_from_the_profile_summary():
    """roofline.traffic is read from profiles/hbm_traffic_bench_c5.md: the row of the kernel behind the dominant
    call must be there, and its scaled read + write bytes must be what that kernel has to move, within 2 %."""
    sys.path.insert(0, ROOT)
    import bench
    n, nb = 61100840, (61100840 + 4095) // 4096
    got = bench.recorded_traffic("decode_accumulate_avg")
    assert got is not None, "no row for the decode-and-average kernel in " + bench.TRAFFIC_PROFILE
    want = bench.algorithmic_bytes(n, nb)["decode_accumulate_avg"]
    assert want == 8 * (n + 4 * nb) + 4 * n
    assert 0.99 * want <= got <= 1.02 * want, (got, want)
    assert bench.recorded_traffic("no_such_call") is None

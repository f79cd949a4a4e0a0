"""Host-side behaviour of bench.py that needs no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    # this build runs on one GPU: any other count must end before anything touches a device
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""


def test_workloads_cover_every_baseline_configuration():
    sys.path.insert(0, ROOT)
    import bench
    names = set(bench.WORKLOADS)
    assert bench.HEADLINE in names
    for name, steps, warmup in bench.SUITE:
        assert name in names and steps >= 1 and warmup >= 0
    # C2, C3 (prefill and the three decode batches), C4, C5 of the configuration list, plus the next-row 4-bit stack
    assert {"c2", "c3_prefill", "c3_decode_b1", "c3_decode_b4", "c3_decode_b16", "c4", "c5", "c6"} <= names

"""Host-side behaviour of bench.py that needs no GPU: it measures one GPU only and says so."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2", "--steps", "1", "--warmup", "0"],
                       capture_output=True, text=True, timeout=300)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""


def test_bench_options_parse():
    sys.path.insert(0, ROOT)
    import bench
    argv = sys.argv
    try:
        sys.argv = ["bench.py"]
        a = bench.parse()
        assert (a.gpus, a.steps, a.warmup, a.layers, a.batch) == (1, 20, 100, 32, 16)
        assert a.recovery == "next-step" and a.groups is None and not a.no_verify
        sys.argv = ["bench.py", "--gpus", "1", "--steps", "5", "--warmup", "2", "--recovery", "same-step", "--groups", "4"]
        a = bench.parse()
        assert (a.steps, a.warmup, a.recovery, a.groups) == (5, 2, "same-step", 4)
    finally:
        sys.argv = argv

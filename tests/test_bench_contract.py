"""bench.py on the host: more than one GPU is refused with a message (this build is single-GPU),
and the defaults are the metric's workload."""
import pathlib
import subprocess
import sys

ROOT = pathlib.Path(__file__).resolve().parents[1]


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, str(ROOT / "bench.py"), "--gpus", "2"], capture_output=True, text=True, cwd=ROOT)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_defaults():
    sys.path.insert(0, str(ROOT))
    import bench

    old = sys.argv
    try:
        sys.argv = ["bench.py"]
        a = bench.parse()
    finally:
        sys.argv = old
    assert (a.gpus, a.config, a.overlap, a.share_heads, a.qkv_linear) == (1, 4, "none", 0, False)
    assert a.steps >= 5 and a.warmup >= 1

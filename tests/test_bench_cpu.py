"""bench.py's command line without a GPU: more than one GPU is refused with a message, and the measurement legs that
--leg names exist."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in r.stderr


def test_every_leg_has_its_function():
    sys.path.insert(0, ROOT)
    import bench
    for leg in ("mlp_block", "indexed", "decoder_layer", "scheduler", "attention", "nano"):
        assert callable(getattr(bench, "measure_" + leg))
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--leg", "no_such_leg"], capture_output=True, text=True)
    assert r.returncode != 0

"""Host-side pieces of bench.py that need no GPU: the one-GPU refusal, and the HBM-traffic figure read from the tracked
rocprofv3 summary (never a constant of the script)."""
import importlib.util
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and not r.stdout.strip()
    env = dict(os.environ, WORLD_SIZE="2")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True, timeout=120, env=env)
    assert r.returncode != 0 and "ONE GPU" in r.stderr


def test_traffic_comes_from_the_tracked_counter_summary():
    b = _bench()
    t = b.counter_traffic("c3_8b_b16", 1, 97)
    # the gate|up projection moves its 234.9 MB of weights once, plus activations and its output: a few per cent more
    assert t is not None and 234.9e6 < t < 1.10 * 234.9e6
    # any other workload, seed or row count: no figure rather than a stale one
    assert b.counter_traffic("c5_8b_b128", 1, 883) is None
    assert b.counter_traffic("c3_8b_b16", 2, 97) is None
    assert b.counter_traffic("c3_8b_b16", 1, 96) is None
    with open(b.TRAFFIC_PROFILE) as f:
        assert sum(1 for line in f if line.startswith("# bench:")) == 1

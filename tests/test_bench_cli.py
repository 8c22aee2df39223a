"""Host-side checks of bench.py that need no GPU: the one-GPU rule and the traffic lookup."""

import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)
    assert not any(line.startswith("{") for line in r.stdout.splitlines())     # no result line


def test_traffic_is_reported_only_for_the_recorded_kernel_source(monkeypatch):
    sys.path.insert(0, ROOT)
    import importlib
    bench = importlib.import_module("bench")
    # a figure only while the recorded source hash is the current one (then for every workload), else none at all
    got = [bench.measured_traffic(w) for w in ("c2_mid", "c3_large", "c4_stream", "c5_merge", "c3_large_fp8", "c4_stream_fp8")]
    assert all(t is None for t in got) or all(t is not None and t > 1e8 for t in got)
    assert bench.measured_traffic("no_such_workload") is None
    # a changed source: no figure
    import hashlib
    real = hashlib.sha256

    class Other:
        def __init__(self):
            self.h = real(b"something else")

        def update(self, b):
            self.h.update(b)

        def hexdigest(self):
            return self.h.hexdigest()

    monkeypatch.setattr(hashlib, "sha256", Other)
    assert bench.measured_traffic("c3_large") is None

"""Host-side checks of the repository contract: bench.py refuses more than one GPU with a message,
fails loudly without a GPU (no CPU fallback), and the entry-point module has build() and smoke()."""
import importlib
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)


def test_bench_without_gpu_does_not_fall_back_to_the_cpu():
    import torch
    if torch.cuda.is_available():
        return
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "1", "--warmup", "0"],
                       capture_output=True, text=True)
    assert r.returncode != 0 and "GPU" in (r.stdout + r.stderr)
    assert "metric" not in r.stdout          # no result line was produced


def test_entry_module_has_build_and_smoke():
    sys.path.insert(0, ROOT)
    m = importlib.import_module("__graft_entry__")
    assert callable(m.build) and callable(m.smoke)

"""The driver-facing contract of bench.py and __graft_entry__.py that can be checked without a GPU."""
import importlib
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU; asking for more must end with a message, not a run."""
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                         text=True, timeout=120, cwd=ROOT)
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr and res.stdout.strip() == ""
    env = dict(os.environ, WORLD_SIZE="4")
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True,
                         timeout=120, cwd=ROOT, env=env)
    assert res.returncode != 0 and "ONE GPU" in res.stderr


def test_algorithmic_byte_formulas():
    """(7R-6) N e for an all-reduce, (4R-3) N e for a reduce-scatter: summed from the per-step units the
    bench uses for its per-kernel figures (send 2, sum 4, last sum 3, copy 3, last copy 2)."""
    sys.path.insert(0, ROOT)
    bench = importlib.import_module("bench")
    wl = importlib.import_module("workloads")
    for w in (wl.cfg1(), wl.cfg2(), wl.cfg3(), wl.cfg4(), wl.cfg5(16)):
        units = sum(bench._step_units(w, j)[1] for j in range(w.steps_per_slab))
        assert units == (7 * w.R - 6 if w.phases == "ar" else 4 * w.R - 3)
        assert w.algorithmic_bytes == units * w.N * w.elem_bytes


def test_graft_entry_has_build_and_smoke():
    sys.path.insert(0, ROOT)
    entry = importlib.import_module("__graft_entry__")
    assert callable(entry.build) and callable(entry.smoke)

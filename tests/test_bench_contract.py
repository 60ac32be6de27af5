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


def test_stream_probe_is_a_library_of_its_own():
    """The bare kernels `bench.py --stream-mix` times are measurement aids: they sit in libr2probe.so, which
    exports its two calls and refuses arguments that do not fit them before any launch; nothing of them is in
    the product library, and the package never loads them."""
    import ctypes

    pkg = os.path.join(ROOT, "paper_2512_25059_amd")
    probe = os.path.join(pkg, "libr2probe.so")
    if not os.path.exists(probe):
        from paper_2512_25059_amd import build

        build.build_probe()
    lib = ctypes.CDLL(probe)
    lib.r2probe_cold_mix.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_uint64), ctypes.c_int,
                                     ctypes.c_uint64, ctypes.c_int, ctypes.c_void_p]
    lib.r2probe_ring_pattern.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_uint64), ctypes.c_int, ctypes.c_uint64,
                                         ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int, ctypes.c_void_p]
    four = (ctypes.c_uint64 * 4)(4096, 8192, 12288, 16384)
    assert lib.r2probe_cold_mix(1, 1, four, 4, 8191, 1, None) == -1  # not a whole number of tiles
    assert lib.r2probe_cold_mix(3, 0, four, 4, 8192, 1, None) == -1  # at most two streams each way
    assert lib.r2probe_cold_mix(0, 0, four, 4, 8192, 1, None) == -1
    assert lib.r2probe_cold_mix(1, 1, four, 3, 8192, 1, None) == -1  # four buffers at least
    assert lib.r2probe_cold_mix(1, 1, None, 4, 8192, 1, None) == -1
    assert lib.r2probe_ring_pattern(4, four, 4, 4096, 8192, 8192, 1, None) == -1
    assert lib.r2probe_ring_pattern(0, four, 4, 0, 8192, 8192, 1, None) == -1
    assert lib.r2probe_ring_pattern(0, four, 4, 4096, 8200, 8192, 1, None) == -1  # stage not 16-byte aligned
    product = ctypes.CDLL(os.path.join(pkg, "libr2ccl.so"))
    assert not hasattr(product, "r2probe_cold_mix") and not hasattr(product, "r2probe_ring_pattern")
    for name in os.listdir(pkg):
        if name.endswith(".py"):
            assert "r2probe" not in open(os.path.join(pkg, name)).read() or name == "build.py"

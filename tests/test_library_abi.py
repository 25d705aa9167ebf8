"""The C-ABI library loads and exports every symbol include/qes.h declares (no GPU needed)."""
import ctypes
import os
import re

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "qes.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qes_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    import paper_2602_03120_amd.binding as b
    lib = ctypes.CDLL(b.library_path())
    names = _declared()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(b.EXPORTS) == names


def test_host_only_entry_points():
    import paper_2602_03120_amd as qes
    assert qes.abi_version() == 1
    assert qes.status_string(0) == "ok" and "invalid" in qes.status_string(-1)
    f = qes.normalize_fitness(np.array([1, 2, 3, 4, 5], dtype=np.float32))
    assert abs(f.mean()) < 1e-7 and abs(f.std() - 1) < 1e-6
    assert (qes.normalize_fitness(np.full(7, 2.0, dtype=np.float32)) == 0).all()


def test_normalize_fitness_against_numpy():
    """The library's own normalisation (a one-pass running mean / squared-deviation update) against
    numpy's fp64 z-score with the population standard deviation."""
    import paper_2602_03120_amd as qes
    rng = np.random.default_rng(11)
    for N in (2, 3, 8, 30, 64, 1000, 1024):
        for shift, scale in ((0.0, 1.0), (100.0, 1.0), (-3.0, 1e-3), (1e4, 50.0)):
            r = (rng.standard_normal(N) * scale + shift).astype(np.float32)
            r64 = r.astype(np.float64)
            ref = ((r64 - r64.mean()) / r64.std()).astype(np.float32)
            got = qes.normalize_fitness(r)
            assert (np.abs(got - ref) <= 2 * np.spacing(np.abs(ref)) + 1e-12).all(), (N, shift, scale)
            assert abs(got.astype(np.float64).mean()) < 1e-6 and abs(got.astype(np.float64).std() - 1) < 1e-6
    assert (qes.normalize_fitness(np.float32([5.0])) == 0).all()                # N < 2
    assert (qes.normalize_fitness(np.float32([1e-20, 1e-20, 1e-20])) == 0).all()


def test_argument_checks_precede_any_gpu_call():
    """Refusals that depend on the arguments alone are returned before the first HIP call, so they
    can be observed without a GPU (the device pointer below is never dereferenced): a tensor above
    the element limit, a bad width, a population above the limit, more records than the entry point
    that allocates nothing holds."""
    import paper_2602_03120_amd.binding as b
    lib = b._load()
    seeds = np.zeros(2048, dtype=np.uint64)
    fit = np.zeros(2048, dtype=np.float32)

    def call(name, out_f, in_f, bits=4, N=4, hist_len=0):
        d = b._QesTensor(4096, None, out_f, in_f, bits, 0, -8 if bits == 4 else -127, 7 if bits == 4 else 127, 1)
        hs = np.zeros((max(hist_len, 1), N), dtype=np.uint64)
        hf = np.zeros((max(hist_len, 1), N), dtype=np.float32)
        return getattr(lib, name)(ctypes.byref(d), seeds.ctypes.data, fit.ctypes.data, hs.ctypes.data, hf.ctypes.data,
                                  hist_len, N, 1.0, 0.5, 0.9, None, None)

    assert call("qes_update", 65536, 131072) == -2            # 2^33 elements
    assert call("qes_update", 65537, 131070) == -2            # 2^33 - 4096 < elements < 2^33
    assert call("qes_update", 64, 64, bits=5) == -1
    assert call("qes_update", 64, 63) == -1                   # odd in_features
    assert call("qes_update", 64, 64, N=1025) == -1
    assert call("qes_update", 64, 64, hist_len=257) == -1
    assert call("qes_update_noalloc", 64, 64, N=1024, hist_len=16) == -5      # 17 * 1024 records > 16384
    assert call("qes_update_noalloc", 64, 64, N=1025) == -1
    assert "scratch" in b.status_string(-5) or "exceeds" in b.status_string(-5)


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2602_03120_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".hpp", ".h")):
                src = open(os.path.join(dirpath, fn)).read()
                assert "import oracle" not in src and "from oracle" not in src and "qes_oracle" not in src, fn


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_missing_library_fails_loudly(tmp_path, monkeypatch):
    """No CPU fallback: a binding pointed at a missing library raises on first use."""
    import importlib
    import paper_2602_03120_amd.binding as b
    fresh = importlib.reload(b)
    try:
        monkeypatch.setattr(fresh, "_LIB_PATH", str(tmp_path / "libqes.so"))
        monkeypatch.setattr(fresh, "_lib", None)
        try:
            fresh.abi_version()
        except ImportError as e:
            assert "no fallback" in str(e)
        else:
            raise AssertionError("a missing library must raise")
    finally:
        importlib.reload(b)

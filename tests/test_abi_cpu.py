"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares, and rejects bad
arguments before touching a device.  No compute call is made here."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2407_13218_amd as L
    if not os.path.exists(L.lib_path()):
        from paper_2407_13218_amd import build as B
        B.build()
    return L.load_library()


def test_every_declared_symbol_is_exported(lib):
    import paper_2407_13218_amd as L
    header = open(os.path.join(ROOT, "include", "linr.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(linr_[a-z0-9_]+)\s*\(", header))
    assert declared == set(L.binding.EXPORTS), declared ^ set(L.binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_filter_record_is_40_bytes():
    import synth_inputs as S
    header = open(os.path.join(ROOT, "include", "linr.h")).read()
    assert "LINR_MAX_ANY 4" in header
    assert S.FILTER_DTYPE.itemsize == 40
    assert [S.FILTER_DTYPE.fields[n][1] for n in ("all_bits", "none_bits", "any_bits", "n_any", "ts_min", "ts_max")] == [0, 4, 8, 24, 28, 32]


def test_strerror_and_host_side_validation(lib):
    import paper_2407_13218_amd as L
    assert L.strerror(0) == "ok" and "k out of range" in L.strerror(-4)
    h = C.c_void_p()
    assert lib.linr_index_create(None, 10, 64, L.I8, 0) == -1                     # NULL out
    assert lib.linr_index_create(C.byref(h), 10, 64, 7, 0) == -3                   # bad dtype
    assert lib.linr_index_create(C.byref(h), 10, 0, L.I8, 0) == -2                 # d == 0
    assert lib.linr_index_create(C.byref(h), 10, 24, L.I8, 0) == -2                # row not a multiple of 16 bytes
    assert lib.linr_index_create(C.byref(h), 10, 1024, L.I8, 0) == -2              # row longer than 512 bytes
    assert lib.linr_index_create(C.byref(h), 0, 64, L.I8, 0) == -5
    assert lib.linr_index_create(C.byref(h), 2 ** 32 - 1, 64, L.I8, 0) == -5       # id space
    assert lib.linr_index_destroy(None) == -1
    assert lib.linr_search_filtered(None, None, None, 1, 1, None, 10, None, None, None, None, None, 0, None, 0) == -1
    assert lib.linr_set_tuning(None) == 0
    with pytest.raises(L.LinrError):
        L.set_tuning(sample_ratio=3)
    L.set_tuning()


def test_missing_library_fails_loudly(tmp_path, monkeypatch):
    import paper_2407_13218_amd.binding as Bd
    monkeypatch.setattr(Bd, "_lib", None)
    monkeypatch.setattr(Bd, "_LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(ImportError):
        Bd.load_library()


def test_bench_refuses_more_than_one_gpu():
    """every box has one GPU: bench.py --gpus N > 1 says so and exits without touching a device"""
    import subprocess
    import sys
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=60)
    assert res.returncode != 0 and "one GPU" in res.stderr and res.stdout.strip() == ""


def test_product_package_does_not_import_the_oracle():
    """the oracle is test infrastructure: nothing under the package, and bench.py only in its baseline legs, names it"""
    pkg = os.path.join(ROOT, "paper_2407_13218_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".cpp", ".hip", ".h")):
                text = open(os.path.join(dirpath, f), errors="replace").read()
                assert "import oracle" not in text and "from oracle" not in text and "linr_oracle" not in text, f
    assert "import oracle" not in open(os.path.join(ROOT, "synth_inputs.py")).read()

"""CPU-side checks of the C-ABI library: it loads, and it exports every symbol
that include/moshpit.h declares.  No compute call is made here."""
import ctypes
import os
import re

import pytest

from paper_2103_03239_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "moshpit.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moshpit_[a-z0-9_]+)\s*\(", text)))


def test_header_and_binding_agree():
    assert declared_functions() == sorted(binding.EXPORTS)


def test_library_exports_every_declared_symbol():
    if not os.path.exists(binding.LIB_PATH):
        pytest.fail("libmoshpit.so is not built: run `python __graft_entry__.py`")
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} is declared in moshpit.h but not exported"


def test_create_rejects_bad_shapes_without_a_gpu():
    """Argument checks run before any HIP call, so they work on a CPU machine."""
    lib = binding.load_library()
    h = ctypes.c_void_p()
    bad = [
        (15, 8, 4, 2, 0),     # N != M^d
        (16, 8, 4, 2, 7),     # unknown dtype
        (16, 0, 4, 2, 0),     # P < 1
        (1, 8, 1, 2, 0),      # M < 2
        (65 ** 2, 8, 65, 2, 0),  # M > 64
        (16, 8, 4, 0, 0),     # d < 1
    ]
    for N, P, M, d, dt in bad:
        assert lib.moshpit_create(N, P, M, d, dt, ctypes.byref(h)) == -1
        assert not h.value
        assert lib.moshpit_last_error(None) != b""
    with pytest.raises(binding.MoshpitError):
        binding.Moshpit(15, 8, 4, 2, 0)


def test_bench_refuses_more_than_one_gpu():
    """The benchmark measures one GPU's share; asking for more ends with a message, not a run."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    out = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert out.returncode == 2
    assert "ONE GPU" in out.stderr + out.stdout

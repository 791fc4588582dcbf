"""CPU-only checks of the C ABI: the library loads, exports every declared symbol, and its
host-side argument validation returns the documented error codes (no kernel is launched)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2501_09253_amd as ps
from paper_2501_09253_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "pserve.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pserve_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = ps.lib()
    syms = _declared_symbols()
    assert "pserve_plan" in syms and "pserve_block_forward" in syms and len(syms) >= 14
    for s in syms:
        assert hasattr(L, s), s


def test_plan_argument_validation():
    L = ps.lib()
    out = C.c_void_p()
    res = np.array([[16, 16]], dtype=np.int32)
    rp = res.ctypes.data_as(C.POINTER(C.c_int32))
    assert L.pserve_plan(rp, 0, 8, 8, None, C.byref(out)) == -1
    assert b"n > 0" in L.pserve_last_error()
    assert L.pserve_plan(None, 1, 8, 8, None, C.byref(out)) == -1
    assert L.pserve_plan(rp, 1, 8, 0, None, C.byref(out)) == -1          # half-specified patch
    assert L.pserve_plan(rp, 1, 5, 5, None, C.byref(out)) == -1          # not a multiple of the patch
    assert b"multiple" in L.pserve_last_error()
    bad = np.array([[16, -4]], dtype=np.int32)
    assert L.pserve_plan(bad.ctypes.data_as(C.POINTER(C.c_int32)), 1, 4, 4, None, C.byref(out)) == -1
    assert L.pserve_plan(rp, 1, 8, 8, None, None) == -1
    assert out.value is None


def test_block_argument_validation():
    L = ps.lib()
    out = C.c_void_p()
    desc = binding._BlockDesc()
    bp = binding._BlockParams()
    assert L.pserve_block_create(None, C.byref(bp), None, C.byref(out)) == -1
    desc.n_stages, desc.C, desc.G, desc.heads, desc.dtype, desc.eps = 1, 60, 8, 2, 0, 1e-5
    desc.stages[0] = 1
    assert L.pserve_block_create(C.byref(desc), C.byref(bp), None, C.byref(out)) == -1      # C % G
    desc.C = 64
    assert L.pserve_block_create(C.byref(desc), C.byref(bp), None, C.byref(out)) == -1      # NULL parameter
    assert b"NULL" in L.pserve_last_error()
    desc.stages[0] = 9
    assert L.pserve_block_create(C.byref(desc), C.byref(bp), None, C.byref(out)) == -1      # unknown stage
    desc.stages[0], desc.dtype = 1, 7
    assert L.pserve_block_create(C.byref(desc), C.byref(bp), None, C.byref(out)) == -1      # unknown dtype
    assert L.pserve_set_kernel_mode(5) == -1 and L.pserve_set_kernel_mode(0) == 0
    assert L.pserve_block_forward(None, None, None, None, None, None, None, None) == -1
    assert L.pserve_cache_create(None, None, 0, C.byref(out)) == -1
    info = binding._PlanInfo()
    assert L.pserve_plan_info(None, C.byref(info)) == -1


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "library_path", lambda: "/nonexistent/libpserve.so")
    with pytest.raises(ImportError):
        binding.lib()


def test_resample_argument_validation():
    L = ps.lib()
    out = C.c_void_p()
    assert L.pserve_resample_create(3, 8, 8, 1, None, None, None, C.byref(out)) == -1       # unknown kind
    assert L.pserve_resample_create(1, 8, 8, 1, None, None, None, C.byref(out)) == -1       # NULL parameters
    assert L.pserve_resample_forward(None, None, None, None, None, 0, None, None) == -1


def test_bench_refuses_more_than_one_gpu():
    """bench.py is a one-GPU program: any other count ends with a message and a non-zero status before touching a GPU."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=60)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""

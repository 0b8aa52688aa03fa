"""The C-ABI library loads without a GPU, exports every symbol the header declares, and rejects bad
arguments before touching the device (no compute call is made here)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "picassomesh.h")


@pytest.fixture(scope="module")
def pm():
    from paper_2112_01801_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    binding.lib()
    return binding


def header_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(pm_[a-z0-9_]+)\s*\(", src)))


def test_every_declared_symbol_is_exported(pm):
    names = header_functions()
    assert set(pm.EXPORTS) == set(names), (set(pm.EXPORTS) ^ set(names))
    for n in names:
        assert getattr(pm.lib(), n) is not None


def test_status_strings(pm):
    assert pm.lib().pm_status_string(0) == b"PM_OK"
    assert pm.lib().pm_status_string(-3) == b"PM_ERR_WORKSPACE"


def test_workspace_bytes_is_host_only_and_monotone(pm):
    a = pm.pm_workspace_bytes(pm.PM_OP_F2V, 1000, 2000, 0, 3, 64, 64, pm.PM_BF16)
    b = pm.pm_workspace_bytes(pm.PM_OP_F2V, 1000, 4000, 0, 3, 64, 64, pm.PM_BF16)
    assert 0 < a < b
    assert pm.pm_workspace_bytes(pm.PM_OP_F2V, 1000, 2000, 0, 6, 64, 64, pm.PM_BF16) == 0      # L > PM_MAX_L
    assert pm.pm_workspace_bytes(pm.PM_OP_F2V, -1, 2000, 0, 3, 64, 64, pm.PM_BF16) == 0
    for op in range(7):
        assert pm.pm_workspace_bytes(op, 100, 200, 900, 2, 8, 8, pm.PM_F32) > 0


def test_argument_errors_before_any_gpu_work(pm):
    lib = pm.lib()
    m = pm._PmMesh()
    m.n_mesh, m.n_vert, m.n_facet = 1, 10, 10
    a = pm._PmAdj()
    # NULL facet array
    s = lib.pm_f2v(C.byref(m), C.byref(a), 3, 0, 8, 8, 0, None, None, None, None, 0, None)
    assert s == -1 and b"NULL" in lib.pm_last_error()
    # degree out of range is reported as unsupported
    s = lib.pm_f2v(C.byref(m), C.byref(a), 9, 0, 8, 8, 0, None, None, None, None, 0, None)
    assert s == -2
    s = lib.pm_sh_basis_dirs(-5, None, 2, 0, None, None)
    assert s == -1
    s = lib.pm_f2f(10, 5, None, None, 2, 0, 3, 8, 0, None, None, None, None, 0, None)
    assert s == -1

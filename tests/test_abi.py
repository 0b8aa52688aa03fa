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


def test_workspace_sizes_of_the_later_operators(pm):
    lib = pm.lib()
    for op in range(7, 11):                               # separable operators
        assert pm.pm_workspace_bytes(op, 100, 200, 0, 3, 16, 24, pm.PM_BF16) > 0
    assert pm.pm_workspace_bytes(11, 100, 200, 0, 3, 16, 24, pm.PM_BF16) == 0
    assert 0 < lib.pm_cluster_ws_bytes(1000, 300) < lib.pm_cluster_ws_bytes(4000, 300)
    assert lib.pm_cluster_ws_bytes(-1, 3) == 0
    assert 0 < lib.pm_texture_ws_bytes(1000, 1) < lib.pm_texture_ws_bytes(9000, 4)
    fwd = lib.pm_pcloud_ws_bytes(0, 1000, 1000, 30000, 3, 64, 64, pm.PM_BF16)
    bwd = lib.pm_pcloud_ws_bytes(1, 1000, 1000, 30000, 3, 64, 64, pm.PM_BF16)
    assert 0 < fwd < bwd
    assert lib.pm_pcloud_ws_bytes(0, 1000, 1000, 30000, 7, 64, 64, pm.PM_BF16) == 0
    vf = lib.pm_v2v_sep_ws_bytes(0, 1000, 2000, 3, 64, 64, 64, pm.PM_BF16)
    vb = lib.pm_v2v_sep_ws_bytes(1, 1000, 2000, 3, 64, 64, 64, pm.PM_BF16)
    assert 0 < vf < lib.pm_v2v_sep_ws_bytes(0, 1000, 8000, 3, 64, 64, 64, pm.PM_BF16) and 0 < vb
    assert lib.pm_v2v_sep_ws_bytes(0, 1000, 2000, 3, 64, 0, 64, pm.PM_BF16) == 0
    assert lib.pm_v2v_sep_ws_bytes(0, -1, 2000, 3, 64, 64, 64, pm.PM_BF16) == 0


def test_argument_errors_of_the_later_operators(pm):
    lib = pm.lib()
    m = pm._PmMesh()
    m.n_mesh, m.n_vert, m.n_facet = 1, 10, 10
    a = pm._PmAdj()
    # separable: NULL mesh arrays, then parameter gradients that do not come together
    assert lib.pm_f2v_sep(C.byref(m), C.byref(a), 3, 0, 8, 8, 0, None, None, None, None, None, None, 0, None) == -1
    assert lib.pm_v2f_sep(C.byref(m), 9, 0, 8, 8, 0, None, None, None, None, None, 0, None) == -2
    # vertex2vertex block: NULL mesh arrays; degree out of range
    nul = [None] * 3
    assert lib.pm_v2v_sep(C.byref(m), C.byref(a), 3, 0, 8, 8, 8, 0, *nul, None, None, None, None, None, None, None, None, 0,
                          None) == -1
    assert lib.pm_v2v_sep_bwd(C.byref(m), C.byref(a), 9, 0, 8, 8, 8, 0, *nul, None, None, None, None, *([None] * 10), 0,
                              None) == -2
    # pooling: NULL map, unknown mode, bad channel count
    assert lib.pm_pool(None, 0, 8, 0, None, None, None, None) == -1
    cm = pm._PmClusterMap()
    cm.n_in, cm.n_out = 0, 0
    assert lib.pm_pool(C.byref(cm), 7, 8, 0, None, None, None, None) == -1 or lib.pm_pool(C.byref(cm), 7, 8, 0, None, None, None, None) == -2
    assert lib.pm_unpool(C.byref(cm), 0, 0, None, None, None) == -1
    assert lib.pm_build_cluster_map(-1, 3, None, None, None, None, None, None, 0, None) == -1
    # neighbour lists: NULL struct, non-positive radius
    assert lib.pm_pcloud_conv(None, 3, 0, 8, 8, 0, None, None, None, None, None, None, None, 0, None) == -1
    assert lib.pm_reverse_ws_bytes(100, 3000) > 0 and lib.pm_reverse_ws_bytes(-1, 5) == 0
    nb = pm._PmNbr()
    nb.n_query, nb.n_source, nb.nnz, nb.rho = 0, 0, 0, 0.0
    assert lib.pm_validate_neighbors(C.byref(nb), None, 0, None) == -1
    # input preparation: bad Eq. 8 parameters, NULL outputs
    assert lib.pm_texture_layout(C.byref(m), -1, 0, None, None, None, 0, None) == -1
    assert lib.pm_texture_bary(-3, None, None, 0, None, None) == -1
    big = pm._PmMesh()
    big.n_mesh, big.n_vert, big.n_facet = 1, 10, 2_000_000_000
    big.vert, big.facet = 256, 256                       # never dereferenced: the size check comes first
    assert lib.pm_texture_layout(C.byref(big), 3, 1, None, None, None, 0, None) == -1 and b"int32" in lib.pm_last_error()
    assert lib.pm_facet_geometry(C.byref(m), 0, 5, None, None) == -1 or lib.pm_facet_geometry(C.byref(m), 0, 5, None, None) == -2

"""A row's result must not depend on where the row sits in the launch: the row-wise operators run on a facet range of
a mesh and on the whole mesh give the same rows bit for bit (same inputs, same arithmetic, whichever workgroup, tile
or pipeline stage a row falls into).  Regression test: the gathered gradient rows of the weight-gradient kernel were
once rounded differently in the code before and inside its tile loop."""
import numpy as np
import pytest

from paper_2112_01801_amd import meshgen as mg
from parity_util import make_coeffs, make_features, pm_dtype, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pm():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2112_01801_amd import binding
    binding.lib()
    return binding


def _setup(pm, grid, cin, cout, L, dtype):
    rng = np.random.default_rng(41)
    b = mg.pack_batch([mg.heightfield(grid, grid, rng, random_diag=True)])
    mesh = pm.mesh_to_device(b)
    adj = pm.pm_build_vf_adjacency(mesh)
    return b, mesh, adj, rng, to_dev(make_coeffs(rng, (L + 1) ** 2, cin, cout, dtype), dtype)


def _ranges(F, n):
    cuts = [0] + [(F * i // n) // 8 * 8 + 8 * (i % 3) for i in range(1, n)] + [F]     # ragged on purpose, 16-byte aligned rows
    return list(zip(cuts[:-1], cuts[1:]))


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_f2v_backward_rows_on_facet_ranges(pm, dtype):
    import torch
    L, cin, cout = 3, 64, 64
    b, mesh, adj, rng, W = _setup(pm, 192, cin, cout, L, dtype)
    F, V = b.n_facet, b.n_vert
    h = to_dev(make_features(rng, F, cin, dtype), dtype)
    dg = to_dev(make_features(rng, V, cout, dtype), dtype)
    dt = pm_dtype(dtype)
    dh_all, dW_all = pm.pm_f2v_bwd(mesh, adj, L, h, W, dg, dt)
    dW_sum = torch.zeros_like(dW_all)
    for lo, hi in _ranges(F, 3):
        part = pm.Mesh(vert=mesh.vert, facet=mesh.facet[lo:hi], vert_off=None, facet_off=None, n_vert=V, n_mesh=1)
        dh, dW = pm.pm_f2v_bwd(part, adj, L, h[lo:hi], W, dg, dt)        # vertex degrees: those of the whole mesh
        assert torch.equal(dh, dh_all[lo:hi]), (dtype, lo, hi)
        dW_sum += dW
    # the weight gradient is a sum over rows: the same up to the order of the fp32 additions
    scale = float(dW_all.abs().max())
    assert float((dW_sum - dW_all).abs().max()) <= 1e-5 * scale


@pytest.mark.parametrize("cin,cout", [(64, 64), (32, 96), (20, 24)])
def test_v2f_forward_rows_on_facet_ranges(pm, cin, cout):
    import torch
    L, dtype = 3, "bf16"
    b, mesh, adj, rng, W = _setup(pm, 160, cin, cout, L, dtype)
    F, V = b.n_facet, b.n_vert
    h = to_dev(make_features(rng, V, cin, dtype), dtype)
    dt = pm_dtype(dtype)
    g_all = pm.pm_v2f(mesh, L, h, W, dt)
    for lo, hi in _ranges(F, 3):
        part = pm.Mesh(vert=mesh.vert, facet=mesh.facet[lo:hi], vert_off=None, facet_off=None, n_vert=V, n_mesh=1)
        assert torch.equal(pm.pm_v2f(part, L, h, W, dt), g_all[lo:hi]), (cin, cout, lo, hi)

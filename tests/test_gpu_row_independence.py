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


@pytest.mark.parametrize("cin,cout,dtype", [(64, 64, "bf16"), (3, 32, "bf16"), (16, 24, "f32")])
def test_f2f_rows_on_facet_ranges(pm, cin, cout, dtype):
    """facet2facet (Eq. 7): the facets of a range with their own points give the same facet rows, and the same
    gradient rows of their points, as inside the whole batch."""
    import torch
    L = 3
    rng = np.random.default_rng(43)
    b = mg.pack_batch([mg.heightfield(96, 96, rng, random_diag=True)])
    tex_off, bary = mg.texture_layout(b, 3, 1)
    F, P = b.n_facet, int(tex_off[-1])
    W = to_dev(make_coeffs(rng, (L + 1) ** 2, cin, cout, dtype), dtype)
    h = to_dev(make_features(rng, P, cin, dtype), dtype)
    dg = to_dev(make_features(rng, F, cout, dtype), dtype)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    off_d, bary_d = t(tex_off.astype(np.int32)), t(bary)
    dt = pm_dtype(dtype)
    g_all = pm.pm_f2f(off_d, bary_d, L, h, W, dt)
    dh_all, _ = pm.pm_f2f_bwd(off_d, bary_d, L, h, W, dg, dt)
    # cuts where the first point of the range starts a 16-byte aligned row in every array
    cuts = [0]
    for target in (F // 3, 2 * F // 3):
        f = target
        while (int(tex_off[f]) * cin) % 8 or int(tex_off[f]) % 4 or (f * cout) % 8:
            f += 1
        cuts.append(f)
    cuts.append(F)
    for lo, hi in zip(cuts[:-1], cuts[1:]):
        p0, p1 = int(tex_off[lo]), int(tex_off[hi])
        off_p = t((tex_off[lo:hi + 1] - tex_off[lo]).astype(np.int32))
        g = pm.pm_f2f(off_p, bary_d[p0:p1], L, h[p0:p1], W, dt)
        assert torch.equal(g, g_all[lo:hi]), (cin, cout, dtype, lo, hi)
        dh, _ = pm.pm_f2f_bwd(off_p, bary_d[p0:p1], L, h[p0:p1], W, dg[lo:hi], dt)
        assert torch.equal(dh, dh_all[p0:p1]), (cin, cout, dtype, lo, hi)


def test_pcloud_rows_on_query_ranges(pm):
    """Point-cloud convolution: a range of the query points with its own lists gives the whole call's rows."""
    import torch
    L, cin, cout, dtype = 3, 64, 32, "bf16"
    rng = np.random.default_rng(44)
    xs = rng.uniform(0.0, 1.0, size=(3000, 3)).astype(np.float32)
    rho = 0.12
    ptr, idx = mg.range_neighbors(xs, xs, rho)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    xs_d = t(xs)
    K = (L + 1) ** 2
    alpha = t((rng.standard_normal((K, cin)) * 0.3).astype(np.float32))
    c0 = t((rng.standard_normal(cin) * 0.3).astype(np.float32))
    Pw = to_dev(make_coeffs(rng, 1, cin, cout, dtype)[0], dtype)
    h = to_dev(make_features(rng, xs.shape[0], cin, dtype), dtype)
    dt = pm_dtype(dtype)
    g_all = pm.pm_pcloud_conv(pm.Neighbors(xs_d, xs_d, t(ptr.astype(np.int32)), t(idx.astype(np.int32)), rho), L, h, alpha, c0, Pw, dt)
    M = xs.shape[0]
    for lo, hi in ((0, 1000), (1000, 2104), (2104, M)):
        ptr_p = (ptr[lo:hi + 1] - ptr[lo]).astype(np.int32)
        idx_p = idx[ptr[lo]:ptr[hi]].astype(np.int32)
        nb = pm.Neighbors(xs_d[lo:hi], xs_d, t(ptr_p), t(idx_p), rho)
        assert torch.equal(pm.pm_pcloud_conv(nb, L, h, alpha, c0, Pw, dt), g_all[lo:hi]), (lo, hi)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_separable_rows_on_facet_ranges(pm, dtype):
    """Separable forms: vertex2facet forward rows and the facet gradients of facet2vertex on facet ranges."""
    import torch
    L, cin, cout = 3, 64, 64
    rng = np.random.default_rng(45)
    b = mg.pack_batch([mg.heightfield(160, 160, rng, random_diag=True)])
    mesh = pm.mesh_to_device(b)
    adj = pm.pm_build_vf_adjacency(mesh)
    F, V = b.n_facet, b.n_vert
    K = (L + 1) ** 2
    alpha = torch.from_numpy((rng.standard_normal((K, cin)) * 0.3).astype(np.float32)).cuda()
    Pw = to_dev(make_coeffs(rng, 1, cin, cout, dtype)[0], dtype)
    hV = to_dev(make_features(rng, V, cin, dtype), dtype)
    hF = to_dev(make_features(rng, F, cin, dtype), dtype)
    dgV = to_dev(make_features(rng, V, cout, dtype), dtype)
    dt = pm_dtype(dtype)
    g_all = pm.pm_v2f_sep(mesh, L, hV, alpha, Pw, dt)
    dh_all = pm.pm_f2v_sep_bwd(mesh, adj, L, hF, alpha, Pw, dgV, dt, want_dw=False)[0]
    for lo, hi in _ranges(F, 3):
        part = pm.Mesh(vert=mesh.vert, facet=mesh.facet[lo:hi], vert_off=None, facet_off=None, n_vert=V, n_mesh=1)
        assert torch.equal(pm.pm_v2f_sep(part, L, hV, alpha, Pw, dt), g_all[lo:hi]), (dtype, lo, hi)
        dh = pm.pm_f2v_sep_bwd(part, adj, L, hF[lo:hi], alpha, Pw, dgV, dt, want_dw=False)[0]
        assert torch.equal(dh, dh_all[lo:hi]), (dtype, lo, hi)

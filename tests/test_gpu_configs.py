"""Parity on the other benchmark configurations (1, 2, 4, 5), through the C ABI.

Small configurations are compared with the oracle element by element.  Where the oracle cannot finish
a whole tensor in seconds, feature outputs are compared on sampled rows it computes one by one; the
weight gradient (a sum over every row) is compared element by element on sampled rows dW[k, ci, :] that
the oracle sums over the whole batch, through the adjoint identity <W', dW> = <conv(h; W'), dg> with a
fresh W' (the forward it uses is sample-checked in the same test; the gap is measured against the 2-norm
of the summed terms, and a planted mistake in dW must fail it), and, every element of every output, on the
smallest mesh of the batch run as its own batch.

Config 4 (eight height-fields with random diagonals, 5 % of the facets deleted, vertices of valence 0) runs
at its full size: several GB of host-side random features per operator.
"""
import numpy as np
import pytest

import oracle
from paper_2112_01801_amd import meshgen as mg
from parity_util import (TOL, adjoint_ok as _adjoint_ok, make_coeffs, make_features, pm_dtype, rel_err, sample_rows,
                         sample_wrows as _wrows, to_dev, to_host)

pytestmark = pytest.mark.gpu
NS = 4096          # sampled output rows per tensor (config 4: NS4)
NS4 = 65536


@pytest.fixture(scope="module")
def pm():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2112_01801_amd import binding
    binding.lib()
    return binding


def _sub_batch(b, m):
    """Mesh m of a packed batch as its own batch."""
    v0, v1 = int(b.vert_off[m]), int(b.vert_off[m + 1])
    f0, f1 = int(b.facet_off[m]), int(b.facet_off[m + 1])
    return mg.pack_batch([(b.vert[v0:v1], b.facet[f0:f1] - v0)]), (v0, v1, f0, f1)


def check_f2v(pm, b, L, cin, cout, dtype, seed, full, ns=NS):
    rng = np.random.default_rng(seed)
    K = (L + 1) ** 2
    W, Wp = make_coeffs(rng, K, cin, cout, dtype), make_coeffs(rng, K, cin, cout, dtype)
    h, dg = make_features(rng, b.n_facet, cin, dtype), make_features(rng, b.n_vert, cout, dtype)
    mesh = pm.mesh_to_device(b)
    adj = pm.pm_build_vf_adjacency(mesh)
    h_d, W_d, dg_d, dt = to_dev(h, dtype), to_dev(W, dtype), to_dev(dg, dtype), pm_dtype(dtype)
    h, dg = h.astype(np.float64), dg.astype(np.float64)      # once, instead of a copy per oracle call
    g = pm.pm_f2v(mesh, adj, L, h_d, W_d, dt)
    dh, dW = pm.pm_f2v_bwd(mesh, adj, L, h_d, W_d, dg_d, dt)
    if full:
        assert rel_err(to_host(g), oracle.f2v(b.vert, b.facet, L, h, W)) < TOL[dtype]
        rdh, rdW = oracle.f2v_bwd(b.vert, b.facet, L, h, W, dg)
        assert rel_err(to_host(dh), rdh) < TOL[dtype] and rel_err(to_host(dW), rdW) < TOL[dtype]
        return
    rv, rf = sample_rows(rng, b.n_vert, ns), sample_rows(rng, b.n_facet, ns)
    assert rel_err(to_host(g[rv]), oracle.f2v(b.vert, b.facet, L, h, W, rows=rv)) < TOL[dtype]
    rdh, _ = oracle.f2v_bwd(b.vert, b.facet, L, h, W, dg, rows=rf, want_dW=False)
    assert rel_err(to_host(dh[rf]), rdh) < TOL[dtype]
    gp = pm.pm_f2v(mesh, adj, L, h_d, to_dev(Wp, dtype), dt)
    assert rel_err(to_host(gp[rv]), oracle.f2v(b.vert, b.facet, L, h, Wp, rows=rv)) < TOL[dtype]
    _adjoint_ok(lambda w: pm.pm_f2v(mesh, adj, L, h_d, w, dt), lambda: make_coeffs(rng, K, cin, cout, dtype), (Wp, gp), dW,
                dg_d, dtype)
    wr = _wrows(rng, K, cin)
    assert rel_err(to_host(dW).reshape(K * cin, cout)[wr], oracle.f2v_dW_rows(b.vert, b.facet, L, h, dg, wr)) < TOL[dtype]


def check_v2f(pm, b, L, cin, cout, dtype, seed, full, ns=NS):
    rng = np.random.default_rng(seed)
    K = (L + 1) ** 2
    W, Wp = make_coeffs(rng, K, cin, cout, dtype), make_coeffs(rng, K, cin, cout, dtype)
    h, dg = make_features(rng, b.n_vert, cin, dtype), make_features(rng, b.n_facet, cout, dtype)
    mesh = pm.mesh_to_device(b)
    adj = pm.pm_build_vf_adjacency(mesh)
    h_d, W_d, dg_d, dt = to_dev(h, dtype), to_dev(W, dtype), to_dev(dg, dtype), pm_dtype(dtype)
    h, dg = h.astype(np.float64), dg.astype(np.float64)      # once, instead of a copy per oracle call
    g = pm.pm_v2f(mesh, L, h_d, W_d, dt)
    dh, dW = pm.pm_v2f_bwd(mesh, adj, L, h_d, W_d, dg_d, dt)
    if full:
        assert rel_err(to_host(g), oracle.v2f(b.n_vert, b.facet, L, h, W)) < TOL[dtype]
        rdh, rdW = oracle.v2f_bwd(b.n_vert, b.facet, L, h, W, dg)
        assert rel_err(to_host(dh), rdh) < TOL[dtype] and rel_err(to_host(dW), rdW) < TOL[dtype]
        return
    rv, rf = sample_rows(rng, b.n_vert, ns), sample_rows(rng, b.n_facet, ns)
    assert rel_err(to_host(g[rf]), oracle.v2f(b.n_vert, b.facet, L, h, W, rows=rf)) < TOL[dtype]
    rdh, _ = oracle.v2f_bwd(b.n_vert, b.facet, L, h, W, dg, rows=rv, want_dW=False)
    assert rel_err(to_host(dh[rv]), rdh) < TOL[dtype]
    gp = pm.pm_v2f(mesh, L, h_d, to_dev(Wp, dtype), dt)
    assert rel_err(to_host(gp[rf]), oracle.v2f(b.n_vert, b.facet, L, h, Wp, rows=rf)) < TOL[dtype]
    _adjoint_ok(lambda w: pm.pm_v2f(mesh, L, h_d, w, dt), lambda: make_coeffs(rng, K, cin, cout, dtype), (Wp, gp), dW, dg_d,
                dtype)
    wr = _wrows(rng, K, cin)
    assert rel_err(to_host(dW).reshape(K * cin, cout)[wr], oracle.v2f_dW_rows(b.n_vert, b.facet, L, h, dg, wr)) < TOL[dtype]


def check_f2f(pm, b, L, cin, cout, dtype, seed, full, ns=NS):
    import torch
    rng = np.random.default_rng(seed)
    K = (L + 1) ** 2
    tex_off, bary = mg.texture_layout(b, 3, 1)
    P = int(tex_off[-1])
    W, Wp = make_coeffs(rng, K, cin, cout, dtype), make_coeffs(rng, K, cin, cout, dtype)
    h, dg = make_features(rng, P, cin, dtype), make_features(rng, b.n_facet, cout, dtype)
    t_off, t_bary = torch.from_numpy(tex_off).cuda(), torch.from_numpy(bary).cuda()
    h_d, W_d, dg_d, dt = to_dev(h, dtype), to_dev(W, dtype), to_dev(dg, dtype), pm_dtype(dtype)
    h, dg = h.astype(np.float64), dg.astype(np.float64)      # once, instead of a copy per oracle call
    g = pm.pm_f2f(t_off, t_bary, L, h_d, W_d, dt)
    dh, dW = pm.pm_f2f_bwd(t_off, t_bary, L, h_d, W_d, dg_d, dt)
    if full:
        assert rel_err(to_host(g), oracle.f2f(tex_off, bary, L, h, W)) < TOL[dtype]
        rdh, rdW = oracle.f2f_bwd(tex_off, bary, L, h, W, dg)
        assert rel_err(to_host(dh), rdh) < TOL[dtype] and rel_err(to_host(dW), rdW) < TOL[dtype]
        return
    rf, rp = sample_rows(rng, b.n_facet, ns), sample_rows(rng, P, ns)
    assert rel_err(to_host(g[rf]), oracle.f2f(tex_off, bary, L, h, W, rows=rf)) < TOL[dtype]
    rdh, _ = oracle.f2f_bwd(tex_off, bary, L, h, W, dg, rows=rp, want_dW=False)
    assert rel_err(to_host(dh[rp]), rdh) < TOL[dtype]
    gp = pm.pm_f2f(t_off, t_bary, L, h_d, to_dev(Wp, dtype), dt)
    assert rel_err(to_host(gp[rf]), oracle.f2f(tex_off, bary, L, h, Wp, rows=rf)) < TOL[dtype]
    _adjoint_ok(lambda w: pm.pm_f2f(t_off, t_bary, L, h_d, w, dt), lambda: make_coeffs(rng, K, cin, cout, dtype), (Wp, gp),
                dW, dg_d, dtype)
    wr = _wrows(rng, K, cin)
    assert rel_err(to_host(dW).reshape(K * cin, cout)[wr], oracle.f2f_dW_rows(tex_off, bary, L, h, dg, wr)) < TOL[dtype]


CHECK = {"f2v": check_f2v, "v2f": check_v2f, "f2f": check_f2f}


# ------------------------------------------------------------------------------------------ config 1
@pytest.mark.parametrize("op", ["f2v", "v2f", "f2f"])
def test_config1_every_element(pm, op):
    cfg = mg.config1()
    assert (cfg.batch.n_vert, cfg.batch.n_facet) == (642, 1280)
    CHECK[op](pm, cfg.batch, cfg.L, cfg.cin, cfg.cout, "f32", 101, full=True)


# ------------------------------------------------------------------------------------------ config 2
@pytest.fixture(scope="module")
def c2():
    return mg.config2(16)


@pytest.mark.parametrize("op", ["f2v", "v2f", "f2f"])
def test_config2_sampled_and_adjoint(pm, c2, op):
    b = c2.batch
    assert 81920 <= b.n_facet <= 327680 and b.n_mesh == 16
    CHECK[op](pm, b, c2.L, c2.cin, c2.cout, "f32", 202, full=False)


@pytest.mark.parametrize("op", ["f2v", "v2f", "f2f"])
def test_config2_smallest_mesh_every_element(pm, c2, op):
    b = c2.batch
    m = int(np.argmin(np.diff(b.facet_off)))
    sub, _ = _sub_batch(b, m)
    CHECK[op](pm, sub, c2.L, c2.cin, c2.cout, "f32", 203, full=True)


# ------------------------------------------------------------------------------------------ config 4
@pytest.fixture(scope="module")
def c4():
    return mg.config4()


def test_config4_adjacency_all_meshes(pm, c4):
    b = c4.batch
    assert b.n_mesh == 8 and 8 * 200_000 * 0.9 <= b.n_facet <= 8 * 1_500_000
    mesh = pm.mesh_to_device(b)
    pm.pm_validate_mesh(mesh)
    adj = pm.pm_build_vf_adjacency(mesh)
    rp, col = oracle.vf_adjacency(b.n_vert, b.facet)
    assert np.array_equal(adj.row_ptr.cpu().numpy(), rp)
    assert np.array_equal(adj.col.cpu().numpy(), col)
    deg = np.diff(rp)
    assert deg.min() == 0 and deg.max() <= 8          # deleted facets leave isolated vertices; grid caps valence


@pytest.mark.parametrize("op,cin,cout", [("v2f", 32, 128), ("f2v", 128, 128), ("f2f", 32, 128)])
def test_config4_sampled_and_adjoint(pm, c4, op, cin, cout):
    CHECK[op](pm, c4.batch, c4.L, cin, cout, "f32", 404, full=False, ns=NS4)


@pytest.mark.parametrize("op,cin,cout", [("v2f", 32, 128), ("f2v", 128, 128), ("f2f", 32, 128)])
def test_config4_smallest_mesh_every_element(pm, c4, op, cin, cout):
    """The smallest mesh of the batch as its own batch: every output and every element of dW against the oracle."""
    b = c4.batch
    m = int(np.argmin(np.diff(b.facet_off)))
    sub, _ = _sub_batch(b, m)
    assert sub.n_facet >= 150_000
    CHECK[op](pm, sub, c4.L, cin, cout, "f32", 405, full=True)


# ------------------------------------------------------------------------------------------ config 5
@pytest.fixture(scope="module")
def c5():
    return mg.config5_levels()


@pytest.mark.parametrize("level", [0, 1, 2, 3])
@pytest.mark.parametrize("op", ["f2v", "v2f", "f2f"])
def test_config5_levels_sampled_and_adjoint(pm, c5, op, level):
    cfg = c5[level]
    assert cfg.batch.n_facet == (2093058, 522242, 130050, 32258)[level]
    assert cfg.cin == (32, 64, 128, 256)[level]
    CHECK[op](pm, cfg.batch, cfg.L, cfg.cin, cfg.cout, "bf16", 505 + level, full=False)


@pytest.mark.parametrize("op", ["f2v", "v2f", "f2f"])
def test_config5_coarsest_level_every_element(pm, c5, op):
    """Level 3 (32,258 facets, 256 -> 256 channels, bf16): every output and every element of dW against the oracle."""
    cfg = c5[3]
    b = cfg.batch
    if op == "f2f":     # 210k texture points x 256 x 256 x 16 take the oracle a minute: the first quarter of the grid rows
        nx = 128
        b = mg.pack_batch([(b.vert[:32 * nx], b.facet[:2 * 31 * (nx - 1)])])
    CHECK[op](pm, b, cfg.L, cfg.cin, cfg.cout, "bf16", 515, full=True)

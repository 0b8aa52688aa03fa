"""Parity at the benchmark's full size and launch configuration (config 3: 2,093,058 facets, bf16).

The oracle cannot finish the whole mesh in seconds, so outputs are compared on sampled rows it computes
one by one; the weight gradient, a sum over all facets, is compared element by element on sampled rows
dW[k, ci, :] that the oracle sums over the whole mesh, through the adjoint identity
<W', dW> = <conv(h; W'), dg> (bilinearity; the forward it uses is itself sample-checked here) and
directly against the oracle on a strip of the mesh run through the same entry points.
"""
import numpy as np
import pytest

import oracle
from paper_2112_01801_amd import meshgen as mg
from parity_util import TOL, adjoint_ok, rel_err, sample_rows, sample_wrows, to_dev, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pm():
    import torch
    assert torch.cuda.is_available()
    from paper_2112_01801_amd import binding
    binding.lib()
    return binding


@pytest.fixture(scope="module")
def c3(pm):
    cfg = mg.config3(1024)
    b = cfg.batch
    rng = mg.rng_for(3, 1)
    h = mg.round_to_bf16(mg.normal_features(rng, b.n_facet, cfg.cin))
    W = mg.round_to_bf16(mg.glorot_coeffs(rng, cfg.K, cfg.cin, cfg.cout))
    dg = mg.round_to_bf16(mg.normal_features(rng, b.n_vert, cfg.cout))
    mesh = pm.mesh_to_device(b)
    adj = pm.pm_build_vf_adjacency(mesh)
    return dict(cfg=cfg, b=b, h=h, W=W, dg=dg, mesh=mesh, adj=adj)


def test_config3_sizes_and_adjacency(pm, c3):
    b = c3["b"]
    assert (b.n_vert, b.n_facet) == (1048576, 2093058)
    rp, col = oracle.vf_adjacency(b.n_vert, b.facet)
    assert np.array_equal(c3["adj"].row_ptr.cpu().numpy(), rp)
    assert np.array_equal(c3["adj"].col.cpu().numpy(), col)


def test_config3_f2v_forward_sampled(pm, c3):
    cfg, b = c3["cfg"], c3["b"]
    g = pm.pm_f2v(c3["mesh"], c3["adj"], cfg.L, to_dev(c3["h"], "bf16"), to_dev(c3["W"], "bf16"), pm.PM_BF16)
    rows = sample_rows(np.random.default_rng(5), b.n_vert, 4096)
    rows[:4] = [0, 1023, b.n_vert - 1024, b.n_vert - 1]          # grid corners (valence 1 or 2)
    ref = oracle.f2v(b.vert, b.facet, cfg.L, c3["h"], c3["W"], rows=rows)
    assert rel_err(to_host(g[rows]), ref) < TOL["bf16"]
    c3["g"] = g


def test_config3_f2v_backward_sampled_and_adjoint(pm, c3):
    import torch
    cfg, b = c3["cfg"], c3["b"]
    h_d, W_d, dg_d = to_dev(c3["h"], "bf16"), to_dev(c3["W"], "bf16"), to_dev(c3["dg"], "bf16")
    dh, dW = pm.pm_f2v_bwd(c3["mesh"], c3["adj"], cfg.L, h_d, W_d, dg_d, pm.PM_BF16)
    rows = sample_rows(np.random.default_rng(6), b.n_facet, 4096)
    rows[:2] = [0, b.n_facet - 1]
    rdh, _ = oracle.f2v_bwd(b.vert, b.facet, cfg.L, c3["h"], c3["W"], c3["dg"], rows=rows, want_dW=False)
    assert rel_err(to_host(dh[rows]), rdh) < TOL["bf16"]
    # adjoint identity with a fresh random W'
    Wp = mg.round_to_bf16(mg.glorot_coeffs(np.random.default_rng(7), cfg.K, cfg.cin, cfg.cout))
    gp = pm.pm_f2v(c3["mesh"], c3["adj"], cfg.L, h_d, to_dev(Wp, "bf16"), pm.PM_BF16)
    r7 = np.random.default_rng(70)
    adjoint_ok(lambda w: pm.pm_f2v(c3["mesh"], c3["adj"], cfg.L, h_d, w, pm.PM_BF16),
               lambda: mg.round_to_bf16(mg.glorot_coeffs(r7, cfg.K, cfg.cin, cfg.cout)), (Wp, gp), dW, dg_d, "bf16")
    # rows dW[k, ci, :] summed by the oracle over all 2,093,058 facets, element by element
    wr = sample_wrows(np.random.default_rng(8), cfg.K, cfg.cin)
    ref = oracle.f2v_dW_rows(b.vert, b.facet, cfg.L, c3["h"], c3["dg"], wr)
    assert rel_err(to_host(dW).reshape(cfg.K * cfg.cin, cfg.cout)[wr], ref) < TOL["bf16"]


def test_config3_strip_dW_against_oracle(pm, c3):
    """The first 96 grid rows as their own mesh: every output, dW included, against the full oracle."""
    cfg, b = c3["cfg"], c3["b"]
    rows, nx = 96, 1024
    Vs, Fs = rows * nx, 2 * (rows - 1) * (nx - 1)
    sub = mg.pack_batch([(b.vert[:Vs], b.facet[:Fs])])
    h, dg, W = c3["h"][:Fs], c3["dg"][:Vs], c3["W"]
    mesh = pm.mesh_to_device(sub)
    adj = pm.pm_build_vf_adjacency(mesh)
    dh, dW = pm.pm_f2v_bwd(mesh, adj, cfg.L, to_dev(h, "bf16"), to_dev(W, "bf16"), to_dev(dg, "bf16"), pm.PM_BF16)
    rdh, rdW = oracle.f2v_bwd(sub.vert, sub.facet, cfg.L, h, W, dg)
    assert rel_err(to_host(dW), rdW) < TOL["bf16"]
    assert rel_err(to_host(dh), rdh) < TOL["bf16"]

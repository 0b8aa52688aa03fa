"""Point-cloud convolution with the radial term: HIP path vs the fp64 oracle through the C ABI."""
import numpy as np
import pytest

import rounding_model as rm
from oracle import pcloud as opc
from paper_2112_01801_amd import meshgen as mg
from parity_util import TOL, make_features, pm_dtype, rel_err, rel_err_rows, sample_rows, to_dev, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pm():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2112_01801_amd import binding
    binding.lib()
    return binding


def _params(rng, L, cin, cout, dtype):
    K = (L + 1) ** 2
    alpha = (rng.uniform(-1, 1, (K, cin)) / np.sqrt(K)).astype(np.float32)
    c0 = rng.uniform(-1, 1, cin).astype(np.float32)
    P = (rng.uniform(-1, 1, (cin, cout)) * np.sqrt(3.0 / cin)).astype(np.float32)
    return alpha, c0, (mg.round_to_bf16(P) if dtype == "bf16" else P)


def _cloud(seed, M, N, rho, same=False, max_nbr=0):
    """Points on a bumpy sheet (the vertices of a surface), with duplicates of some sources so that r = 0 occurs."""
    rng = np.random.default_rng(seed)
    xs = np.stack([rng.uniform(0, 1, N), rng.uniform(0, 1, N), 0.1 * rng.standard_normal(N)], 1).astype(np.float32)
    if same:
        xq = xs
    else:
        xq = np.stack([rng.uniform(0, 1, M), rng.uniform(0, 1, M), 0.1 * rng.standard_normal(M)], 1).astype(np.float32)
        xq[:5] = xs[:5]
    ptr, idx = mg.range_neighbors(xq, xs, rho, max_nbr, rng)
    return xq, xs, ptr, idx


def _nbr(pm, xq, xs, ptr, idx, rho):
    import torch
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    xs_d = t(xs)
    xq_d = xs_d if xq is xs else t(xq)
    return pm.Neighbors(xq_d, xs_d, t(ptr), t(idx), rho)


CASES = [(3, 64, 64, "bf16"), (3, 64, 64, "f32"), (2, 20, 24, "f32"), (4, 32, 128, "bf16"), (5, 8, 40, "f32"),
         (0, 16, 16, "bf16"), (1, 3, 5, "f32"), (3, 136, 16, "bf16"),
         # bf16 with more than 32 basis rows (fp32 tiles), and channel runs that are not whole (element-wise access)
         (5, 16, 24, "bf16"), (3, 20, 12, "bf16"), (4, 10, 8, "bf16")]


@pytest.mark.parametrize("L,cin,cout,dtype", CASES)
def test_forward_backward_against_the_oracle(pm, L, cin, cout, dtype):
    import torch
    rho = 0.11
    xq, xs, ptr, idx = _cloud(300 + L, 700, 900, rho)
    deg = np.diff(ptr)
    assert deg.min() == 0 or deg.max() > 3 * max(deg.min(), 1)          # ragged lists
    rng = np.random.default_rng(310 + L)
    alpha, c0, P = _params(rng, L, cin, cout, dtype)
    h = make_features(rng, xs.shape[0], cin, dtype)
    dg = make_features(rng, xq.shape[0], cout, dtype)
    nb = _nbr(pm, xq, xs, ptr, idx, rho)
    pm.pm_validate_neighbors(nb)
    a_d, c_d, P_d, dt = torch.from_numpy(alpha).cuda(), torch.from_numpy(c0).cuda(), to_dev(P, dtype), pm_dtype(dtype)
    g = pm.pm_pcloud_conv(nb, L, to_dev(h, dtype), a_d, c_d, P_d, dt)
    assert rel_err(to_host(g), opc.pcloud_conv(xq, xs, ptr, idx, rho, L, h, alpha, c0, P)) < TOL[dtype]
    dh, da, dc, dP = pm.pm_pcloud_conv_bwd(nb, L, to_dev(h, dtype), a_d, c_d, P_d, to_dev(dg, dtype), dt)
    rdh, rda, rdc, rdP = opc.pcloud_conv_bwd(xq, xs, ptr, idx, rho, L, h, alpha, c0, P, dg)
    assert rel_err(to_host(dh), rdh) < TOL[dtype]
    assert rel_err(to_host(da), rda) < TOL[dtype]
    assert rel_err(to_host(dc)[None, :], rdc[None, :]) < TOL[dtype]
    assert rel_err(to_host(dP), rdP) < TOL[dtype]
    dh1, n1, n2, n3 = pm.pm_pcloud_conv_bwd(nb, L, to_dev(h, dtype), a_d, c_d, P_d, to_dev(dg, dtype), dt, want_dw=False)
    assert n1 is None and n2 is None and n3 is None and torch.equal(dh1, dh)
    n0, da1, dc1, dP1 = pm.pm_pcloud_conv_bwd(nb, L, to_dev(h, dtype), a_d, c_d, P_d, to_dev(dg, dtype), dt, want_dh=False)
    assert n0 is None and torch.equal(da1, da) and torch.equal(dc1, dc) and torch.equal(dP1, dP)
    # reverse lists built once and the depth-wise output handed out by the forward call: the same bits
    nb2 = pm.pm_build_reverse_neighbors(nb)
    g2, y = pm.pm_pcloud_conv(nb2, L, to_dev(h, dtype), a_d, c_d, P_d, dt, save_y=True)
    assert torch.equal(g2, g) and y.shape == (xq.shape[0], cin)
    dh2, da2, dc2, dP2 = pm.pm_pcloud_conv_bwd(nb2, L, to_dev(h, dtype), a_d, c_d, P_d, to_dev(dg, dtype), dt, y_saved=y)
    assert torch.equal(dh2, dh) and torch.equal(da2, da) and torch.equal(dc2, dc) and torch.equal(dP2, dP)


def test_vertices_of_a_coarse_mesh_level_sampled(pm):
    """A 256x256 level of the benchmark hierarchy (65,536 points, queries = sources, ~30 neighbours each, 1 to ~70)."""
    import torch
    L, cin, cout, dtype = 3, 64, 64, "bf16"
    v, _ = mg.heightfield(256, 256, np.random.default_rng(320))
    xs = v.astype(np.float32)
    span = float(xs[:, 0].max() - xs[:, 0].min())
    rho = 5.0 * span / 255
    ptr, idx = mg.range_neighbors(xs, xs, rho)
    assert 20 < np.diff(ptr).mean() < 40
    rng = np.random.default_rng(321)
    alpha, c0, P = _params(rng, L, cin, cout, dtype)
    h = make_features(rng, xs.shape[0], cin, dtype)
    dg = make_features(rng, xs.shape[0], cout, dtype)
    nb = _nbr(pm, xs, xs, ptr, idx, rho)
    a_d, c_d, P_d, dt = torch.from_numpy(alpha).cuda(), torch.from_numpy(c0).cuda(), to_dev(P, dtype), pm_dtype(dtype)
    g = pm.pm_pcloud_conv(nb, L, to_dev(h, dtype), a_d, c_d, P_d, dt)
    dh, da, dc, dP = pm.pm_pcloud_conv_bwd(nb, L, to_dev(h, dtype), a_d, c_d, P_d, to_dev(dg, dtype), dt)
    # the oracle on the whole set takes a few seconds (1.9 M pairs)
    ref = opc.pcloud_conv(xs, xs, ptr, idx, rho, L, h, alpha, c0, P)
    # border points have one or two neighbours, interior points average thirty: the depth-wise rows y (the bf16
    # operand of the point-wise matrix) differ in scale by sqrt(30), and half a bf16 unit of the large rows, measured
    # against the global rms, exceeds 2e-2 in ANY bf16 data path: rounding_model (the oracle with y and the output
    # rounded to bf16; tests/test_rounding_bounds.py pins it at 4.5e-2 on this very input) gives the bound.  The
    # result is held to that bound, to two bf16 units from the model itself, to the stated 2e-2 on the rows the scale argument
    # does not touch (own rms within twice the global one), and to 2e-2 of its own rms on every row.
    got = to_host(g)
    model = rm.pcloud_forward_bf16(xs, xs, ptr, idx, rho, L, h, alpha, c0, P)
    e, em, d = rel_err(got, ref), rel_err(model, ref), rel_err(got, model)
    print("pcloud forward: err %.2e  model %.2e  from model %.2e" % (e, em, d))
    assert e < rm.derived_bound(TOL[dtype], em) and d < 2.0 ** -6     # two bf16 units from the model
    row_rms, rms = np.sqrt(np.mean(ref ** 2, axis=1)), np.sqrt(np.mean(ref ** 2))
    plain = row_rms <= 2.0 * rms
    assert plain.mean() > 0.9
    den = np.maximum(np.abs(ref[plain]), rms)
    assert float(np.max(np.abs(got[plain] - ref[plain]) / den)) < TOL[dtype]
    assert rel_err_rows(got, ref) < TOL[dtype]
    rdh, rda, rdc, rdP = opc.pcloud_conv_bwd(xs, xs, ptr, idx, rho, L, h, alpha, c0, P, dg)
    assert rel_err(to_host(dh), rdh) < TOL[dtype]              # one store: the stated metric
    assert rel_err(to_host(da), rda) < TOL[dtype] and rel_err(to_host(dP), rdP) < TOL[dtype]
    assert rel_err(to_host(dc)[None, :], rdc[None, :]) < TOL[dtype]


def test_empty_lists_and_bad_lists(pm):
    import torch
    L, cin, cout = 2, 16, 8
    rng = np.random.default_rng(330)
    alpha, c0, P = _params(rng, L, cin, cout, "f32")
    a_d, c_d, P_d = torch.from_numpy(alpha).cuda(), torch.from_numpy(c0).cuda(), to_dev(P, "f32")
    xs = rng.uniform(0, 1, (10, 3)).astype(np.float32)
    xq = rng.uniform(0, 1, (6, 3)).astype(np.float32)
    h = make_features(rng, 10, cin, "f32")
    # no pairs at all
    nb = _nbr(pm, xq, xs, np.zeros(7, np.int32), np.zeros(0, np.int32), 0.5)
    g = pm.pm_pcloud_conv(nb, L, to_dev(h, "f32"), a_d, c_d, P_d, 0)
    assert g.shape == (6, cout) and not g.abs().any()
    dh, da, dc, dP = pm.pm_pcloud_conv_bwd(nb, L, to_dev(h, "f32"), a_d, c_d, P_d, torch.ones((6, cout), device="cuda"), 0)
    assert not dh.abs().any() and not da.abs().any() and not dc.abs().any() and not dP.abs().any()
    # lists that do not span idx / ids outside the source set are reported
    bad = _nbr(pm, xq, xs, np.array([0, 2, 1, 3, 3, 3, 3], np.int32), np.array([1, 2, 3], np.int32), 0.5)
    with pytest.raises(pm.PmError):
        pm.pm_validate_neighbors(bad)
    bad = _nbr(pm, xq, xs, np.array([0, 1, 1, 3, 3, 3, 3], np.int32), np.array([1, 10, 3], np.int32), 0.5)
    with pytest.raises(pm.PmError):
        pm.pm_validate_neighbors(bad)


def test_later_operators_replay_from_a_hip_graph(pm):
    """Separable, vertex2vertex, pooling and point-cloud entry points enqueue kernels only: captured into one HIP graph (their
    outputs and workspaces come from the graph's memory pool), replays with eager work in between reproduce
    the eager results bit for bit -- including the sums over the reverse lists built inside the call."""
    import torch
    from test_gpu_parity import small_batch
    L, cin, cout, dtype, dt = 3, 64, 64, "bf16", 1
    rng = np.random.default_rng(340)
    b = small_batch(34)
    mesh = pm.mesh_to_device(b)
    adj = pm.pm_build_vf_adjacency(mesh)
    alpha, c0, P = _params(rng, L, cin, cout, dtype)
    a_d, c_d, P_d = torch.from_numpy(alpha).cuda(), torch.from_numpy(c0).cuda(), to_dev(P, dtype)
    hF = to_dev(make_features(rng, b.n_facet, cin, dtype), dtype)
    dgV = to_dev(make_features(rng, b.n_vert, cout, dtype), dtype)
    xq, xs, ptr, idx = _cloud(341, 500, 600, 0.12)
    nb = _nbr(pm, xq, xs, ptr, idx, 0.12)
    hN = to_dev(make_features(rng, 600, cin, dtype), dtype)
    dgM = to_dev(make_features(rng, 500, cout, dtype), dtype)
    vc, io = mg.random_cluster_maps(rng, b.n_vert, b.n_vert // 4, drop_frac=0.05, heavy=40)
    vc_d, io_d = torch.from_numpy(vc).cuda(), torch.from_numpy(io).cuda()
    n_used = int((io[vc] >= 0).sum())               # members that reach an output vertex: the used part of col

    ep = pm.Epilogue(torch.rand(cout, device="cuda") + 0.5, torch.randn(cout, device="cuda") * 0.3, True)

    def work():
        out = list(pm.pm_f2v_sep_bwd(mesh, adj, L, hF, a_d, P_d, dgV, dt))
        o, g, z = pm.pm_v2v_sep(mesh, adj, L, dgV, a_d, P_d, ep, a_d, P_d, ep, dt, save=True)
        out += [o, g, z] + list(pm.pm_v2v_sep_bwd(mesh, adj, L, dgV, a_d, P_d, ep, a_d, P_d, ep, g, z, o, dgV, dt))
        out += list(pm.pm_pcloud_conv_bwd(nb, L, hN, a_d, c_d, P_d, dgM, dt))
        cm = pm.pm_build_cluster_map(vc_d, io_d, b.n_vert // 4)
        m, arg = pm.pm_pool(cm, pm.PM_POOL_MAX, dgV, dt)
        out += [cm.col[:n_used], m, arg, pm.pm_unpool_bwd(cm, dgV, dt)]
        return out

    ref = [t.clone() for t in work()]
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        work()
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            res = work()
    for rep in range(3):
        for t in res:
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (got, want) in enumerate(zip(res, ref)):
            assert torch.equal(got, want), "replay %d, output %d differs from the eager result" % (rep, i)

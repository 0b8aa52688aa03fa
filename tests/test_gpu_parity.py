"""HIP path vs the fp64 oracle, element by element, through the C ABI (small and medium sizes).

Index work (adjacency) must be bit-exact; fp32 outputs within 1e-4 and bf16 outputs within 2e-2 of
the oracle in the metric of parity_util.rel_err.  Sizes span several 512-row tiles plus a ragged tail.
"""
import numpy as np
import pytest

import oracle
from paper_2112_01801_amd import meshgen as mg
from parity_util import TOL, make_coeffs, make_features, pm_dtype, rel_err, to_dev, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pm():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2112_01801_amd import binding
    binding.lib()
    return binding


def small_batch(seed=0):
    """Three meshes, ~2.7k facets: spans 5 full 512-row tiles and a ragged tail; one isolated vertex."""
    rng = np.random.default_rng(seed)
    meshes = []
    for lvl in (3, 2, 3):
        v, f = mg.icosphere_f64(lvl)
        v = v * (1 + rng.normal(0, 0.03, (v.shape[0], 1))) * rng.uniform(0.5, 1.5, (1, 3))
        meshes.append((v.astype(np.float32), f))
    v, f = meshes[1]
    meshes[1] = (np.concatenate([v, [[9, 9, 9]]], 0).astype(np.float32), f)
    return mg.pack_batch(meshes)


# ---------------------------------------------------------------------------------- basis
@pytest.mark.parametrize("L", [0, 1, 2, 3, 4, 5])
@pytest.mark.parametrize("norm", [0, 1])
def test_sh_basis_dirs(pm, L, norm):
    import torch
    rng = np.random.default_rng(100 + L)
    d = rng.standard_normal((1000, 3)).astype(np.float32) * rng.uniform(0.1, 10, (1000, 1)).astype(np.float32)
    d[:6] = [[0, 0, 1], [0, 0, -1], [1, 0, 0], [0, 1, 0], [-1, 0, 0], [0, -2, 0]]
    got = to_host(pm.pm_sh_basis_dirs(torch.from_numpy(d).cuda(), L, norm))
    ref = oracle.sh_basis(d, L, norm)
    assert rel_err(got, ref) < 2e-5


def test_sh_basis_mesh_and_degenerate_facet(pm):
    b = small_batch(1)
    f = b.facet.copy()
    f[7] = [f[7, 0], f[7, 0], f[7, 1]]            # zero-area facet -> (0,0,1)
    b = mg.MeshBatch(b.vert, f, b.vert_off, b.facet_off)
    mesh = pm.mesh_to_device(b)
    got = to_host(pm.pm_sh_basis(mesh, 3))
    ref = oracle.sh_basis(oracle.facet_normals(b.vert, b.facet), 3)
    assert rel_err(got, ref) < 2e-5
    np.testing.assert_allclose(got[7], oracle.sh_basis(np.array([[0, 0, 1.0]]), 3)[0], atol=1e-6)


@pytest.mark.parametrize("L", [1, 3, 5])
def test_sh_basis_bwd(pm, L):
    import torch
    rng = np.random.default_rng(200 + L)
    d = rng.standard_normal((300, 3)).astype(np.float32)
    db = rng.standard_normal((300, (L + 1) ** 2)).astype(np.float32)
    got = to_host(pm.pm_sh_basis_bwd(torch.from_numpy(d).cuda(), L, torch.from_numpy(db).cuda()))
    ref = oracle.sh_basis_bwd(d, L, db)
    assert rel_err(got, ref) < 1e-4


# ---------------------------------------------------------------------------------- adjacency
def fan_mesh(n):
    """n facets around one hub vertex (valence n >> 64) plus an isolated vertex."""
    ang = np.linspace(0, 2 * np.pi, n, endpoint=False)
    v = np.concatenate([[[0, 0, 0.5]], np.stack([np.cos(ang), np.sin(ang), 0 * ang], 1), [[5, 5, 5]]], 0)
    f = np.stack([np.zeros(n, dtype=np.int64), 1 + np.arange(n), 1 + (np.arange(n) + 1) % n], 1)
    return v.astype(np.float32), f.astype(np.int32)


@pytest.mark.parametrize("case", ["batch", "fan", "deleted", "empty"])
def test_adjacency_bit_exact(pm, case):
    if case == "batch":
        b = small_batch(2)
    elif case == "fan":
        b = mg.pack_batch([fan_mesh(5000), mg.icosphere(2)])
    elif case == "deleted":
        rng = np.random.default_rng(3)
        v, f = mg.heightfield(70, 45, rng, random_diag=True)
        b = mg.pack_batch([(v, mg.delete_facets(f, 0.2, rng))])
    else:
        b = mg.pack_batch([(np.zeros((5, 3), np.float32), np.zeros((0, 3), np.int32))])
    mesh = pm.mesh_to_device(b)
    pm.pm_validate_mesh(mesh)
    adj = pm.pm_build_vf_adjacency(mesh)
    rp, col = oracle.vf_adjacency(b.n_vert, b.facet)
    assert np.array_equal(adj.row_ptr.cpu().numpy(), rp)
    assert np.array_equal(adj.col.cpu().numpy(), col)


def test_validate_mesh_rejects_bad_ids(pm):
    b = small_batch(4)
    f = b.facet.copy()
    f[100, 1] = b.vert_off[1] + 3          # facet of mesh 0 pointing into mesh 1
    mesh = pm.mesh_to_device(mg.MeshBatch(b.vert, f, b.vert_off, b.facet_off))
    with pytest.raises(pm.PmError) as e:
        pm.pm_validate_mesh(mesh)
    assert e.value.status == -5


# ---------------------------------------------------------------------------------- convolutions
CASES = [  # (L, cin, cout, dtype)
    (3, 16, 16, "f32"),
    (3, 64, 64, "f32"),
    (3, 64, 64, "bf16"),
    (2, 3, 5, "f32"),
    (4, 32, 128, "f32"),
    (1, 20, 24, "bf16"),
    (0, 8, 8, "f32"),
    (5, 8, 40, "bf16"),
    (3, 128, 96, "bf16"),
    (1, 64, 64, "bf16"),
    (4, 64, 128, "bf16"),
    (5, 64, 64, "bf16"),
    (3, 32, 32, "bf16"),     # staged vertex2facet tiles: 32-channel rows, operand row zero-padded to two chunks
    (2, 32, 96, "bf16"),
    (3, 64, 32, "bf16"),
    (4, 128, 128, "f32"),    # weight-gradient tiling with several k groups and (c, n) slabs; streamed weights
    (3, 256, 256, "bf16"),
    (3, 32, 64, "bf16"),     # 32-channel operand on one side of the fused weight-gradient kernel
    (3, 128, 32, "bf16"),
]


def _setup(pm, L, cin, cout, dtype, seed):
    b = small_batch(seed)
    rng = np.random.default_rng(seed + 1000)
    K = (L + 1) ** 2
    W = make_coeffs(rng, K, cin, cout, dtype)
    mesh = pm.mesh_to_device(b)
    adj = pm.pm_build_vf_adjacency(mesh)
    return b, rng, K, W, mesh, adj


@pytest.mark.parametrize("L,cin,cout,dtype", CASES)
def test_f2v_forward_backward(pm, L, cin, cout, dtype):
    b, rng, K, W, mesh, adj = _setup(pm, L, cin, cout, dtype, 10)
    h = make_features(rng, b.n_facet, cin, dtype)
    dg = make_features(rng, b.n_vert, cout, dtype)
    g = pm.pm_f2v(mesh, adj, L, to_dev(h, dtype), to_dev(W, dtype), pm_dtype(dtype))
    assert rel_err(to_host(g), oracle.f2v(b.vert, b.facet, L, h, W)) < TOL[dtype]
    dh, dW = pm.pm_f2v_bwd(mesh, adj, L, to_dev(h, dtype), to_dev(W, dtype), to_dev(dg, dtype), pm_dtype(dtype))
    rdh, rdW = oracle.f2v_bwd(b.vert, b.facet, L, h, W, dg)
    assert rel_err(to_host(dh), rdh) < TOL[dtype]
    assert rel_err(to_host(dW), rdW) < TOL[dtype]


@pytest.mark.parametrize("L,cin,cout,dtype", CASES)
def test_v2f_forward_backward(pm, L, cin, cout, dtype):
    b, rng, K, W, mesh, adj = _setup(pm, L, cin, cout, dtype, 20)
    h = make_features(rng, b.n_vert, cin, dtype)
    dg = make_features(rng, b.n_facet, cout, dtype)
    g = pm.pm_v2f(mesh, L, to_dev(h, dtype), to_dev(W, dtype), pm_dtype(dtype))
    assert rel_err(to_host(g), oracle.v2f(b.n_vert, b.facet, L, h, W)) < TOL[dtype]
    dh, dW = pm.pm_v2f_bwd(mesh, adj, L, to_dev(h, dtype), to_dev(W, dtype), to_dev(dg, dtype), pm_dtype(dtype))
    rdh, rdW = oracle.v2f_bwd(b.n_vert, b.facet, L, h, W, dg)
    assert rel_err(to_host(dh), rdh) < TOL[dtype]
    assert rel_err(to_host(dW), rdW) < TOL[dtype]


@pytest.mark.parametrize("L,cin,cout,dtype", CASES)
def test_f2f_forward_backward(pm, L, cin, cout, dtype):
    import torch
    b = small_batch(30)
    rng = np.random.default_rng(1030)
    K = (L + 1) ** 2
    W = make_coeffs(rng, K, cin, cout, dtype)
    tex_off, bary = mg.texture_layout(b, 3, 1)
    tex_off = tex_off.copy()
    P = int(tex_off[-1])
    h = make_features(rng, P, cin, dtype)
    dg = make_features(rng, b.n_facet, cout, dtype)
    t_off, t_bary = torch.from_numpy(tex_off).cuda(), torch.from_numpy(bary).cuda()
    g = pm.pm_f2f(t_off, t_bary, L, to_dev(h, dtype), to_dev(W, dtype), pm_dtype(dtype))
    assert rel_err(to_host(g), oracle.f2f(tex_off, bary, L, h, W)) < TOL[dtype]
    dh, dW = pm.pm_f2f_bwd(t_off, t_bary, L, to_dev(h, dtype), to_dev(W, dtype), to_dev(dg, dtype), pm_dtype(dtype))
    rdh, rdW = oracle.f2f_bwd(tex_off, bary, L, h, W, dg)
    assert rel_err(to_host(dh), rdh) < TOL[dtype]
    assert rel_err(to_host(dW), rdW) < TOL[dtype]


@pytest.mark.parametrize("L,cin,cout", [(3, 64, 64), (2, 64, 128)])
def test_f2v_backward_single_gradients(pm, L, cin, cout):
    """dh alone and dW alone take other kernel paths than the joint call (which shares the gathered rows)."""
    dtype = "bf16"
    b, rng, K, W, mesh, adj = _setup(pm, L, cin, cout, dtype, 15)
    h = make_features(rng, b.n_facet, cin, dtype)
    dg = make_features(rng, b.n_vert, cout, dtype)
    args = (mesh, adj, L, to_dev(h, dtype), to_dev(W, dtype), to_dev(dg, dtype), pm_dtype(dtype))
    rdh, rdW = oracle.f2v_bwd(b.vert, b.facet, L, h, W, dg)
    dh, none = pm.pm_f2v_bwd(*args, want_dW=False)
    assert none is None and rel_err(to_host(dh), rdh) < TOL[dtype]
    none, dW = pm.pm_f2v_bwd(*args, want_dh=False)
    assert none is None and rel_err(to_host(dW), rdW) < TOL[dtype]
    dh2, dW2 = pm.pm_f2v_bwd(*args)
    assert rel_err(to_host(dh2), rdh) < TOL[dtype] and rel_err(to_host(dW2), rdW) < TOL[dtype]
    assert np.array_equal(to_host(dW2), to_host(dW))           # the weight gradient does not depend on the pairing


@pytest.mark.parametrize("dtype,cin,cout", [("bf16", 64, 64), ("f32", 24, 40), ("bf16", 128, 64)])
def test_v2f_backward_single_gradients(pm, dtype, cin, cout):
    """Each gradient alone and both together (dW gathers the corner rows either way; dh goes through the per-vertex slot sums)."""
    L = 3
    b, rng, K, W, mesh, adj = _setup(pm, L, cin, cout, dtype, 25)
    h = make_features(rng, b.n_vert, cin, dtype)
    dg = make_features(rng, b.n_facet, cout, dtype)
    args = (mesh, adj, L, to_dev(h, dtype), to_dev(W, dtype), to_dev(dg, dtype), pm_dtype(dtype))
    rdh, rdW = oracle.v2f_bwd(b.n_vert, b.facet, L, h, W, dg)
    dh, none = pm.pm_v2f_bwd(*args, want_dW=False)
    assert none is None and rel_err(to_host(dh), rdh) < TOL[dtype]
    none, dW = pm.pm_v2f_bwd(*args, want_dh=False)
    assert none is None and rel_err(to_host(dW), rdW) < TOL[dtype]
    dh2, dW2 = pm.pm_v2f_bwd(*args)
    assert rel_err(to_host(dh2), rdh) < TOL[dtype] and rel_err(to_host(dW2), rdW) < TOL[dtype]


@pytest.mark.parametrize("dtype,L,cin,cout", [("f32", 3, 3, 32), ("bf16", 3, 3, 32), ("bf16", 3, 4, 64), ("f32", 1, 1, 8),
                                              ("bf16", 2, 3, 96), ("f32", 3, 5, 32)])
def test_f2f_empty_facets_and_paper_shape(pm, dtype, L, cin, cout):
    """Few input channels (Cin = 3 colours is the paper's own shape; up to four take the per-facet staging, five the
    per-point path), some facets without texture points, forward and backward."""
    import torch
    rng = np.random.default_rng(40)
    res = rng.choice([0, 1, 3, 6, 10, 15], size=1700)
    tex_off = np.concatenate([[0], np.cumsum(res)]).astype(np.int32)
    bary = np.concatenate([mg.bary_lattice({0: 0, 1: 0, 3: 1, 6: 2, 10: 3, 15: 4}[r]) for r in res if r > 0], 0)
    K = (L + 1) ** 2
    W = make_coeffs(rng, K, cin, cout, dtype)
    h = make_features(rng, bary.shape[0], cin, dtype)
    dg = make_features(rng, res.shape[0], cout, dtype)
    t_off, t_bary = torch.from_numpy(tex_off).cuda(), torch.from_numpy(bary).cuda()
    g = pm.pm_f2f(t_off, t_bary, L, to_dev(h, dtype), to_dev(W, dtype), pm_dtype(dtype))
    ref = oracle.f2f(tex_off, bary, L, h, W)
    assert rel_err(to_host(g), ref) < TOL[dtype]
    assert np.all(to_host(g)[res == 0] == 0)
    dh, dW = pm.pm_f2f_bwd(t_off, t_bary, L, to_dev(h, dtype), to_dev(W, dtype), to_dev(dg, dtype), pm_dtype(dtype))
    rdh, rdW = oracle.f2f_bwd(tex_off, bary, L, h, W, dg)
    assert rel_err(to_host(dh), rdh) < TOL[dtype] and rel_err(to_host(dW), rdW) < TOL[dtype]
    dh1, none = pm.pm_f2f_bwd(t_off, t_bary, L, to_dev(h, dtype), to_dev(W, dtype), to_dev(dg, dtype), pm_dtype(dtype),
                              want_dW=False)
    assert none is None and torch.equal(dh1, dh)


def test_fan_vertex_and_orthonormal_variant(pm):
    """Valence 5000 at one vertex, an isolated vertex, and the sqrt(2)-scaled basis family."""
    b = mg.pack_batch([fan_mesh(5000)])
    rng = np.random.default_rng(50)
    L, cin, cout = 2, 16, 16
    W = make_coeffs(rng, 9, cin, cout, "f32")
    h = make_features(rng, b.n_facet, cin, "f32")
    mesh = pm.mesh_to_device(b)
    adj = pm.pm_build_vf_adjacency(mesh)
    g = to_host(pm.pm_f2v(mesh, adj, L, to_dev(h, "f32"), to_dev(W, "f32"), 0, norm=1))
    ref = oracle.f2v(b.vert, b.facet, L, h, W, norm=1)
    assert rel_err(g, ref) < 1e-4
    assert np.all(g[-1] == 0)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_v2f_backward_on_fan_and_isolated_vertices(pm, dtype):
    """The per-vertex corner-slot sums with one segment of 5000 entries and vertices without any facet."""
    b = mg.pack_batch([fan_mesh(5000), mg.icosphere(2)])
    rng = np.random.default_rng(55)
    L, cin, cout = 3, 64, 64
    W = make_coeffs(rng, 16, cin, cout, dtype)
    h = make_features(rng, b.n_vert, cin, dtype)
    dg = make_features(rng, b.n_facet, cout, dtype)
    mesh = pm.mesh_to_device(b)
    adj = pm.pm_build_vf_adjacency(mesh)
    dh, dW = pm.pm_v2f_bwd(mesh, adj, L, to_dev(h, dtype), to_dev(W, dtype), to_dev(dg, dtype), pm_dtype(dtype))
    rdh, rdW = oracle.v2f_bwd(b.n_vert, b.facet, L, h, W, dg)
    # the hub row sums 5000 facet rows and is ~50x larger than every other row: bf16 operand rounding scales
    # with it, so it is measured against its own rms, the other rows against theirs
    got = to_host(dh)
    assert rel_err(got[:1], rdh[:1]) < TOL[dtype]
    assert rel_err(got[1:], rdh[1:]) < TOL[dtype]
    assert rel_err(to_host(dW), rdW) < TOL[dtype]
    iso = np.setdiff1d(np.arange(b.n_vert), np.unique(b.facet))
    assert iso.size > 0 and np.all(to_host(dh)[iso] == 0)


def test_f2f_bf16_with_empty_facets(pm):
    import torch
    rng = np.random.default_rng(41)
    res = rng.choice([0, 3, 6, 10], size=900)
    tex_off = np.concatenate([[0], np.cumsum(res)]).astype(np.int32)
    bary = np.concatenate([mg.bary_lattice({3: 1, 6: 2, 10: 3}[r]) for r in res if r > 0], 0)
    L, cin, cout = 3, 64, 64
    W = make_coeffs(rng, 16, cin, cout, "bf16")
    h = make_features(rng, bary.shape[0], cin, "bf16")
    dg = make_features(rng, 900, cout, "bf16")
    t_off, t_bary = torch.from_numpy(tex_off).cuda(), torch.from_numpy(bary).cuda()
    g = pm.pm_f2f(t_off, t_bary, L, to_dev(h, "bf16"), to_dev(W, "bf16"), 1)
    assert rel_err(to_host(g), oracle.f2f(tex_off, bary, L, h, W)) < TOL["bf16"]
    assert np.all(to_host(g)[res == 0] == 0)
    dh, dW = pm.pm_f2f_bwd(t_off, t_bary, L, to_dev(h, "bf16"), to_dev(W, "bf16"), to_dev(dg, "bf16"), 1)
    rdh, rdW = oracle.f2f_bwd(tex_off, bary, L, h, W, dg)
    assert rel_err(to_host(dh), rdh) < TOL["bf16"] and rel_err(to_host(dW), rdW) < TOL["bf16"]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_empty_inputs(pm, dtype):
    """No facets (and no texture points): every sum is empty, so feature outputs and weight gradients are zero."""
    import torch
    b = mg.pack_batch([(np.random.default_rng(3).random((5, 3)).astype(np.float32), np.zeros((0, 3), np.int32))])
    mesh = pm.mesh_to_device(b)
    adj = pm.pm_build_vf_adjacency(mesh)
    L, cin, cout, dt = 3, 64, 64, pm_dtype(dtype)
    tdt = torch.bfloat16 if dt else torch.float32
    W = torch.ones((16, cin, cout), device="cuda", dtype=tdt)
    hF, hV = torch.zeros((0, cin), device="cuda", dtype=tdt), torch.ones((5, cin), device="cuda", dtype=tdt)
    dgV, dgF = torch.ones((5, cout), device="cuda", dtype=tdt), torch.zeros((0, cout), device="cuda", dtype=tdt)
    g = pm.pm_f2v(mesh, adj, L, hF, W, dt)
    assert g.shape == (5, cout) and not g.float().abs().any()
    dh, dW = pm.pm_f2v_bwd(mesh, adj, L, hF, W, dgV, dt)
    assert dh.shape == (0, cin) and not dW.abs().any()
    assert pm.pm_v2f(mesh, L, hV, W, dt).shape == (0, cout)
    dh, dW = pm.pm_v2f_bwd(mesh, adj, L, hV, W, dgF, dt)
    assert dh.shape == (5, cin) and not dh.float().abs().any() and not dW.abs().any()
    t_off = torch.zeros(4, dtype=torch.int32, device="cuda")          # three facets without texture points
    bary = torch.zeros((0, 3), device="cuda")
    g = pm.pm_f2f(t_off, bary, L, hF, W, dt)
    assert g.shape == (3, cout) and not g.float().abs().any()
    dh, dW = pm.pm_f2f_bwd(t_off, bary, L, hF, W, torch.ones((3, cout), device="cuda", dtype=tdt), dt)
    assert dh.shape == (0, cin) and not dW.abs().any()


def test_results_are_bitwise_reproducible(pm):
    import torch
    L, cin, cout, dtype = 3, 64, 64, "bf16"
    b, rng, K, W, mesh, adj = _setup(pm, L, cin, cout, dtype, 60)
    h = to_dev(make_features(rng, b.n_facet, cin, dtype), dtype)
    dg = to_dev(make_features(rng, b.n_vert, cout, dtype), dtype)
    Wd = to_dev(W, dtype)
    outs = []
    for _ in range(2):
        g = pm.pm_f2v(mesh, adj, L, h, Wd, 1)
        dh, dW = pm.pm_f2v_bwd(mesh, adj, L, h, Wd, dg, 1)
        torch.cuda.synchronize()
        outs.append((g.clone(), dh.clone(), dW.clone()))
    for a, c in zip(outs[0], outs[1]):
        assert torch.equal(a, c)


def test_argument_errors(pm):
    import torch
    b = small_batch(70)
    mesh = pm.mesh_to_device(b)
    adj = pm.pm_build_vf_adjacency(mesh)
    h = torch.zeros((b.n_facet, 8), device="cuda")
    W = torch.zeros((16, 8, 8), device="cuda")
    with pytest.raises(pm.PmError) as e:
        pm.pm_f2v(mesh, adj, 6, h, torch.zeros((49, 8, 8), device="cuda"), 0)
    assert e.value.status == -2
    with pytest.raises(pm.PmError) as e:
        pm.pm_f2v(mesh, adj, 3, h, W, 0, ws=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.status == -3
    with pytest.raises(pm.PmError) as e:
        pm.pm_f2v(mesh, adj, 3, h, torch.zeros(16 * 8 * 8 + 1, device="cuda")[1:].view(16, 8, 8), 0)
    assert e.value.status == -1


def test_peak_probes_report_sane_rates(pm):
    """The measurement aid: rates within the physical range of the device, clock readings present."""
    import torch
    ws = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
    ones, clk1 = pm.pm_peak_probe(pm.PM_PEAK_MFMA_BF16_ONES, ws)
    rnd, clk2 = pm.pm_peak_probe(pm.PM_PEAK_MFMA_BF16_RANDOM, ws)
    f32, _ = pm.pm_peak_probe(pm.PM_PEAK_MFMA_F32, ws)
    copy, _ = pm.pm_peak_probe(pm.PM_PEAK_HBM_COPY, ws)
    assert 500 < rnd <= ones * 1.05 < 2700 and 30 < f32 < 170 and 500 < copy < 8500
    assert 500 < clk2 <= clk1 * 1.05 < 3000
    with pytest.raises(pm.PmError) as e:
        pm.pm_peak_probe(pm.PM_PEAK_HBM_COPY, torch.empty(1024, dtype=torch.uint8, device="cuda"))
    assert e.value.status == -3


def test_step_replays_from_a_hip_graph(pm):
    """The entry points enqueue kernels only (no allocation, no synchronisation, caller's workspace), so a
    forward+backward step can be captured into a HIP graph.  Replays, with eager work and synchronisations
    in between, must reproduce the eager results bit for bit."""
    import torch
    L, cin, cout, dtype = 3, 64, 64, "bf16"
    b, rng, K, W, mesh, adj = _setup(pm, L, cin, cout, dtype, 80)
    h = to_dev(make_features(rng, b.n_facet, cin, dtype), dtype)
    dg = to_dev(make_features(rng, b.n_vert, cout, dtype), dtype)
    Wd = to_dev(W, dtype)
    V, F = b.n_vert, b.n_facet
    ws_f = pm.alloc_workspace(pm.pm_workspace_bytes(pm.PM_OP_F2V, V, F, 0, L, cin, cout, 1))
    ws_b = pm.alloc_workspace(pm.pm_workspace_bytes(pm.PM_OP_F2V_BWD, V, F, 0, L, cin, cout, 1))
    g = torch.empty((V, cout), dtype=torch.bfloat16, device="cuda")
    dh = torch.empty((F, cin), dtype=torch.bfloat16, device="cuda")
    dW = torch.empty((K, cin, cout), dtype=torch.float32, device="cuda")

    def step(stream=None):
        pm.pm_f2v(mesh, adj, L, h, Wd, 1, out=g, ws=ws_f, stream=stream)
        pm.pm_f2v_bwd(mesh, adj, L, h, Wd, dg, 1, dh=dh, dW=dW, ws=ws_b, stream=stream)

    step()
    torch.cuda.synchronize()
    ref = (g.clone(), dh.clone(), dW.clone())
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step(side)                                  # warm-up on the capture stream (function attributes are set here)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step(side)
    for rep in range(3):
        for t in (g, dh, dW):
            t.zero_()                               # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip((g, dh, dW), ref):
            assert torch.equal(got, want), "replay %d differs from the eager result" % rep

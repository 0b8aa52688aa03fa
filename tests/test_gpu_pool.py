"""Mesh pooling / unpooling over vertex clusters: HIP path vs the oracle through the C ABI.

Index work (cluster map, argmax) and maxima are compared bit for bit; averages and sums within the
floating-point bar of the convolutions."""
import numpy as np
import pytest

from oracle import pool as op
from paper_2112_01801_amd import meshgen as mg
from parity_util import TOL, make_features, pm_dtype, rel_err, to_dev, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pm():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2112_01801_amd import binding
    binding.lib()
    return binding


def _dev_i32(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def _check_all(pm, vc, io, n_out, C, dtype, seed, ties=False):
    import torch
    rng = np.random.default_rng(seed)
    n_in = vc.shape[0]
    cm = pm.pm_build_cluster_map(_dev_i32(vc), _dev_i32(io), n_out)
    rp, col = op.cluster_members(vc, io, n_out)
    assert np.array_equal(cm.target.cpu().numpy(), op.cluster_target(vc, io))
    assert np.array_equal(cm.row_ptr.cpu().numpy(), rp)
    assert np.array_equal(cm.col.cpu().numpy()[:rp[-1]], col)
    h = make_features(rng, n_in, C, dtype)
    if ties:
        h = np.round(h * 2).astype(np.float32) / 2          # few distinct values (exact in bf16): many ties
    dg_o = make_features(rng, n_out, C, dtype)
    dg_i = make_features(rng, n_in, C, dtype)
    dt = pm_dtype(dtype)
    # max pooling: values and indices are exact
    m, arg = pm.pm_pool(cm, pm.PM_POOL_MAX, to_dev(h, dtype), dt)
    rm, rarg = op.pool(vc, io, n_out, h, op.POOL_MAX)
    assert np.array_equal(to_host(m), rm)
    assert np.array_equal(arg.cpu().numpy(), rarg)
    g = pm.pm_pool_bwd(cm, pm.PM_POOL_MAX, to_dev(dg_o, dtype), dt, argmax=arg)
    assert np.array_equal(to_host(g), op.pool_bwd(vc, io, n_out, dg_o, op.POOL_MAX, rarg))
    m2, none = pm.pm_pool(cm, pm.PM_POOL_MAX, to_dev(h, dtype), dt, want_argmax=False)
    assert none is None and torch.equal(m2, m)
    # average pooling
    a, _ = pm.pm_pool(cm, pm.PM_POOL_AVG, to_dev(h, dtype), dt)
    assert rel_err(to_host(a), op.pool(vc, io, n_out, h, op.POOL_AVG)[0]) < TOL[dtype]
    ga = pm.pm_pool_bwd(cm, pm.PM_POOL_AVG, to_dev(dg_o, dtype), dt)
    assert rel_err(to_host(ga), op.pool_bwd(vc, io, n_out, dg_o, op.POOL_AVG)) < TOL[dtype]
    # unpooling: a copy, exact
    u = pm.pm_unpool(cm, to_dev(dg_o, dtype), dt)
    assert np.array_equal(to_host(u), op.unpool(vc, io, dg_o))
    gu = pm.pm_unpool_bwd(cm, to_dev(dg_i, dtype), dt)
    ref = op.unpool_bwd(vc, io, n_out, dg_i)
    if dtype == "bf16":
        # a long cluster sums thousands of bf16 values: compare each row against its own scale
        err = np.abs(to_host(gu) - ref).max(axis=1) / np.maximum(np.sqrt((ref ** 2).mean(axis=1)), 1e-30)
        assert err.max() < TOL[dtype]
    else:
        assert rel_err(to_host(gu), ref) < TOL[dtype]
    return cm


@pytest.mark.parametrize("C,dtype", [(64, "bf16"), (64, "f32"), (20, "f32"), (7, "bf16"), (520, "bf16"), (1, "f32")])
def test_random_clusters_with_drops_and_a_heavy_cluster(pm, C, dtype):
    rng = np.random.default_rng(40 + C)
    vc, io = mg.random_cluster_maps(rng, 5000, 1300, drop_frac=0.1, heavy=700)
    _check_all(pm, vc, io, 1300, C, dtype, 41 + C)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_ties_go_to_the_lowest_input_index(pm, dtype):
    rng = np.random.default_rng(50)
    vc, io = mg.random_cluster_maps(rng, 3000, 400, drop_frac=0.05, heavy=100)
    _check_all(pm, vc, io, 400, 32, dtype, 51, ties=True)


def test_grid_hierarchy_of_the_benchmark_mesh(pm):
    """The 2x2 clustering that links the levels of config 5 (1024^2 -> 512^2), at full size, sampled."""
    import torch
    nx = ny = 1024
    vc, io = mg.grid_cluster_maps(nx, ny)
    n_in, n_out, C, dtype = nx * ny, (nx // 2) * (ny // 2), 64, "bf16"
    pm.pm_validate_clusters(_dev_i32(vc), _dev_i32(io), n_out)
    cm = pm.pm_build_cluster_map(_dev_i32(vc), _dev_i32(io), n_out)
    rp, col = op.cluster_members(vc, io, n_out)
    assert np.array_equal(cm.row_ptr.cpu().numpy(), rp) and np.array_equal(cm.col.cpu().numpy(), col)
    rng = np.random.default_rng(60)
    h = make_features(rng, n_in, C, dtype)
    dt = pm_dtype(dtype)
    m, arg = pm.pm_pool(cm, pm.PM_POOL_MAX, to_dev(h, dtype), dt)
    rm, rarg = op.pool(vc, io, n_out, h, op.POOL_MAX)
    assert np.array_equal(to_host(m), rm) and np.array_equal(arg.cpu().numpy(), rarg)
    a, _ = pm.pm_pool(cm, pm.PM_POOL_AVG, to_dev(h, dtype), dt)
    assert rel_err(to_host(a), op.pool(vc, io, n_out, h, op.POOL_AVG)[0]) < TOL[dtype]
    u = pm.pm_unpool(cm, m, dt)
    assert np.array_equal(to_host(u), op.unpool(vc, io, rm))
    # pooling what unpooling made returns the coarse features
    back, _ = pm.pm_pool(cm, pm.PM_POOL_MAX, u, dt)
    assert torch.equal(back, m)


def test_global_pooling_per_mesh_and_empty_inputs(pm):
    import torch
    # one cluster per mesh of a packed batch: vcluster = own index, iomap = mesh id
    sizes = [700, 1, 2300]
    mesh_id = np.repeat(np.arange(3), sizes).astype(np.int32)
    n_in = mesh_id.shape[0]
    vc = np.arange(n_in, dtype=np.int32)
    rng = np.random.default_rng(70)
    h = make_features(rng, n_in, 48, "f32")
    cm = pm.pm_build_cluster_map(_dev_i32(vc), _dev_i32(mesh_id), 3)
    m, arg = pm.pm_pool(cm, pm.PM_POOL_MAX, to_dev(h, "f32"), 0)
    a, _ = pm.pm_pool(cm, pm.PM_POOL_AVG, to_dev(h, "f32"), 0)
    off = np.concatenate([[0], np.cumsum(sizes)])
    for i in range(3):
        seg = h[off[i]:off[i + 1]].astype(np.float64)
        assert np.array_equal(to_host(m)[i], seg.max(axis=0))
        assert np.array_equal(arg.cpu().numpy()[i], off[i] + seg.argmax(axis=0))
        assert np.allclose(to_host(a)[i], seg.mean(axis=0), rtol=1e-5, atol=1e-6)
    # an output vertex without members, and no input vertices at all
    vc2, io2 = np.array([0, 0, 2], np.int32), np.array([1, -1, -1], np.int32)
    cm2 = pm.pm_build_cluster_map(_dev_i32(vc2), _dev_i32(io2), 3)
    h2 = torch.tensor([[1.0, -2.0], [3.0, -5.0], [9.0, 9.0]], device="cuda")
    m2, arg2 = pm.pm_pool(cm2, pm.PM_POOL_MAX, h2, 0)
    assert m2.tolist() == [[0, 0], [3, -2], [0, 0]] and arg2.tolist() == [[-1, -1], [1, 0], [-1, -1]]
    assert pm.pm_unpool(cm2, m2, 0).tolist() == [[3, -2], [3, -2], [0, 0]]
    e = torch.zeros(0, dtype=torch.int32, device="cuda")
    cm0 = pm.pm_build_cluster_map(e, e, 4)
    assert cm0.row_ptr.tolist() == [0] * 5
    m0, arg0 = pm.pm_pool(cm0, pm.PM_POOL_MAX, torch.zeros((0, 8), device="cuda"), 0)
    assert m0.shape == (4, 8) and not m0.abs().any() and (arg0 == -1).all()
    assert pm.pm_unpool_bwd(cm0, torch.zeros((0, 8), device="cuda"), 0).abs().sum() == 0


def test_out_of_range_ids_are_reported_and_never_followed(pm):
    vc = np.array([0, 5, 1, -1, 2], np.int32)        # 5 and -1 are outside [0, 5)
    io = np.array([0, 7, -2, -1, -1], np.int32)      # 7 and -2 are outside [-1, 2)
    with pytest.raises(pm.PmError) as e:
        pm.pm_validate_clusters(_dev_i32(vc), _dev_i32(io), 2)
    assert e.value.status == -5
    cm = pm.pm_build_cluster_map(_dev_i32(vc), _dev_i32(io), 2)
    assert cm.target.tolist() == [0, -1, -1, -1, -1]
    assert cm.row_ptr.tolist() == [0, 1, 1]

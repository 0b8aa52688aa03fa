"""Facet geometric features (Eq. 9) and the texture resolution rule with its interpolation points (Eq. 8):
HIP path vs the oracle through the C ABI.  Features to the floating-point bar.  Eq. 8 floors a real ratio q: the
oracle evaluates it in fp64, the kernel in fp32, so gamma is compared bit for bit wherever q is farther from an
integer than the fp32 evaluation can move it; on the other facets (if any) either neighbouring integer is valid.
Offsets and lattice points follow from gamma by integer work and are compared bit for bit given gamma."""
import numpy as np
import pytest

from oracle import geom as og
from paper_2112_01801_amd import meshgen as mg
from parity_util import TOL, rel_err, to_host
from test_gpu_parity import small_batch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pm():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2112_01801_amd import binding
    binding.lib()
    return binding


def _batches():
    rng = np.random.default_rng(80)
    yield "small", small_batch(21)
    yield "grids", mg.pack_batch([mg.heightfield(40, 33, rng, random_diag=True), mg.icosphere(2), mg.heightfield(5, 5, rng)])
    # degenerate facets: collinear corners, a repeated vertex
    v = np.array([[0, 0, 0], [1, 0, 0], [2, 0, 0], [0, 1, 0], [0, 0, 0]], np.float32)
    yield "degenerate", mg.pack_batch([(v, np.array([[0, 1, 2], [0, 4, 1], [0, 1, 3]], np.int32))])


@pytest.mark.parametrize("name,b", list(_batches()))
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("with_heights", [False, True])
def test_facet_geometry(pm, name, b, dtype, with_heights):
    mesh = pm.mesh_to_device(b)
    got = to_host(pm.pm_facet_geometry(mesh, 1 if dtype == "bf16" else 0, with_heights))
    ref = og.facet_geometry(b.vert, b.facet, with_heights)
    assert got.shape == ref.shape
    # every column against its own scale (lengths, cosines, normal components and heights differ in size)
    tol = 2e-5 if dtype == "f32" else 8e-3          # bf16: one rounding of the stored value, 2^-8 relative
    for c in range(ref.shape[1]):
        assert rel_err(got[:, c:c + 1], ref[:, c:c + 1]) < tol, c


def _check_layout(b, alpha, beta, gamma, tex_off, bary, lattice_facets=None):
    """gamma against the oracle where Eq. 8's floor is decided beyond fp32 rounding, valid elsewhere; offsets and
    lattice points bit for bit.  Returns the fraction of facets whose floor is within rounding of an integer."""
    q = og.texture_ratio(b.vert, b.facet, b.facet_off, alpha)
    rg = og.texture_resolution(b.vert, b.facet, b.facet_off, alpha, beta)
    A = og.facet_area(b.vert, b.facet)
    # fp32 evaluation of q: a handful of roundings of relative size 2^-24 on A, amplified by Amax / (Amax - Amin)
    tol = np.zeros(b.n_facet)
    for m in range(b.n_mesh):
        s_ = slice(int(b.facet_off[m]), int(b.facet_off[m + 1]))
        if s_.stop > s_.start and A[s_].max() > A[s_].min():
            tol[s_] = 16 * max(alpha, 1) * 2.0 ** -24 * A[s_].max() / (A[s_].max() - A[s_].min())
    near = (np.abs(q - np.round(q)) <= tol) & (q > 0) & (q < alpha)        # the extremes are exact in any precision
    assert np.array_equal(gamma[~near], rg[~near])
    assert np.all((gamma[near] == np.round(q[near]) + beta) | (gamma[near] == np.round(q[near]) - 1 + beta))
    same = gamma == rg
    roff = og.texture_offsets(rg)
    if same.all():
        assert np.array_equal(tex_off, roff)
    assert tex_off[0] == 0 and np.array_equal(np.diff(tex_off), (gamma.astype(np.int64) + 1) * (gamma + 2) // 2)
    fs = np.nonzero(same)[0] if lattice_facets is None else lattice_facets[same[lattice_facets]]
    if lattice_facets is None and same.all():
        assert np.array_equal(bary, og.texture_bary(rg))
    else:
        for f in fs:
            assert np.array_equal(bary[tex_off[f]:tex_off[f + 1]], og.texture_bary(rg[f:f + 1]))
    return float(near.mean())


@pytest.mark.parametrize("name,b", list(_batches()))
@pytest.mark.parametrize("alpha,beta", [(3, 1), (0, 0), (5, 0), (2, 3)])
def test_texture_layout(pm, name, b, alpha, beta):
    mesh = pm.mesh_to_device(b)
    gamma, tex_off, bary = pm.pm_texture_layout(mesh, alpha, beta)
    _check_layout(b, alpha, beta, gamma.cpu().numpy(), tex_off.cpu().numpy().astype(np.int64), bary.cpu().numpy())


def test_texture_layout_of_the_benchmark_mesh_feeds_facet2facet(pm):
    """Config 3 at full size: gamma over all 2,093,058 facets, offsets, sampled lattices; the device-made layout equals
    the generator's (which the facet2facet parity tests use) except where an area ratio sits on a rounding boundary."""
    cfg = mg.config3()
    b = cfg.batch
    mesh = pm.mesh_to_device(b)
    gamma, tex_off, bary = pm.pm_texture_layout(mesh, 3, 1)
    got = bary.cpu().numpy()
    fs = np.unique(np.random.default_rng(81).integers(0, b.n_facet, 512))
    near = _check_layout(b, 3, 1, gamma.cpu().numpy(), tex_off.cpu().numpy().astype(np.int64), got, lattice_facets=fs)
    assert near < 1e-3
    assert np.allclose(got.sum(axis=1), 1, atol=1e-6)
    gen_off, _ = mg.texture_layout(b, 3, 1)
    assert (np.diff(gen_off) != np.diff(tex_off.cpu().numpy())).mean() < 1e-3


def test_empty_mesh(pm):
    e = mg.pack_batch([(np.zeros((4, 3), np.float32), np.zeros((0, 3), np.int32))])
    mesh = pm.mesh_to_device(e)
    assert pm.pm_facet_geometry(mesh, 0).shape == (0, 9)
    gamma, tex_off, bary = pm.pm_texture_layout(mesh, 3, 1)
    assert gamma.numel() == 0 and tex_off.tolist() == [0] and bary.shape == (0, 3)

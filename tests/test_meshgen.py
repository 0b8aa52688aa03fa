"""Input generators: counts, closedness, determinism (no method arithmetic is tested here)."""
import numpy as np
import pytest

from paper_2112_01801_amd import meshgen as mg


def edge_counts(f):
    e = np.concatenate([f[:, [0, 1]], f[:, [1, 2]], f[:, [2, 0]]], 0).astype(np.int64)
    e.sort(axis=1)
    _, c = np.unique(e[:, 0] * (f.max() + 1) + e[:, 1], return_counts=True)
    return c


@pytest.mark.parametrize("level", [0, 1, 2, 3])
def test_icosphere_counts_and_manifold(level):
    v, f = mg.icosphere(level)
    assert v.shape[0] == 10 * 4 ** level + 2 and f.shape[0] == 20 * 4 ** level
    assert f.shape[0] == 2 * v.shape[0] - 4
    assert np.all(edge_counts(f) == 2)
    np.testing.assert_allclose(np.linalg.norm(v, axis=1), 1.0, atol=1e-6)
    deg = np.bincount(f.ravel())
    assert sorted(set(deg.tolist())) in ([5], [5, 6])
    # outward orientation
    n = np.cross(v[f[:, 1]] - v[f[:, 0]], v[f[:, 2]] - v[f[:, 0]])
    assert np.all(np.einsum("ij,ij->i", n, v[f].mean(1)) > 0)


def test_grid_and_hierarchy_counts():
    rng = mg.rng_for(3)
    v, f = mg.heightfield(64, 64, rng)
    assert v.shape[0] == 64 * 64 and f.shape[0] == 2 * 63 * 63
    n = np.cross(v[f[:, 1]] - v[f[:, 0]], v[f[:, 2]] - v[f[:, 0]])
    assert np.all(n[:, 2] > 0)
    v2, f2, cx, cy = mg.cluster_grid_2x2(v, 64, 64)
    assert (cx, cy) == (32, 32) and v2.shape[0] == 32 * 32 and f2.shape[0] == 2 * 31 * 31
    assert np.all(edge_counts(f2) <= 2)
    n2 = np.cross(v2[f2[:, 1]] - v2[f2[:, 0]], v2[f2[:, 2]] - v2[f2[:, 0]])
    assert np.all(n2[:, 2] > 0)


def test_config_sizes_and_determinism():
    c1 = mg.config1()
    assert (c1.batch.n_vert, c1.batch.n_facet, c1.K) == (642, 1280, 16)
    assert np.array_equal(c1.batch.vert, mg.config1().batch.vert)
    c2 = mg.config2(4)
    assert c2.batch.n_mesh == 4 and c2.batch.facet.max() == c2.batch.n_vert - 1
    assert np.array_equal(np.diff(c2.batch.facet_off), [20 * 4 ** l for l in c2.info["levels"]])
    c3 = mg.config3(64)
    assert c3.batch.n_facet == 2 * 63 * 63
    c4 = mg.config4(2, 2000, 8000)
    deg = np.bincount(c4.batch.facet.ravel(), minlength=c4.batch.n_vert)
    assert deg.max() <= 8
    lv = mg.config5_levels(64, 3)
    assert [c.batch.n_facet for c in lv] == [2 * 63 * 63, 2 * 31 * 31, 2 * 15 * 15]


def test_texture_layout_and_bf16_rounding():
    for g in range(5):
        lat = mg.bary_lattice(g)
        assert lat.shape[0] == (g + 1) * (g + 2) // 2
        np.testing.assert_allclose(lat.sum(1), 1.0, atol=1e-6)
    b = mg.config2(2).batch
    tex_off, bary = mg.texture_layout(b, 3, 1)
    r = np.diff(tex_off)
    assert set(r.tolist()) <= {3, 6, 10, 15} and bary.shape[0] == tex_off[-1]
    x = np.array([1.0, 1.00390625, 1.01171875, -3.1415926, 1e-20], dtype=np.float32)
    y = mg.round_to_bf16(x)
    assert y[0] == 1.0 and y[1] == 1.0 and y[2] == np.float32(1.015625)   # ties to even
    assert np.array_equal(mg.bf16_from_bits(mg.bf16_bits(y)), y)
    import torch
    assert np.array_equal(torch.from_numpy(x).to(torch.bfloat16).float().numpy(), y)

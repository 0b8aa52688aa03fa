"""Pins of the geometric-feature (Eq. 9) and texture-resolution (Eq. 8) oracle."""
import numpy as np
import pytest

from oracle import geom as og
from paper_2112_01801_amd import meshgen as mg


def test_right_and_equilateral_triangles_closed_forms():
    # 3-4-5 triangle in the xy plane, right angle at x1; equilateral triangle of side 2 tilted out of plane
    v = np.array([[0, 0, 0], [3, 0, 0], [0, 4, 0], [1, 1, 1], [3, 1, 1], [2, 1, 1 + np.sqrt(3.0)]], np.float64)
    f = np.array([[0, 1, 2], [3, 4, 5]])
    g = og.facet_geometry(v, f, with_heights=True)
    assert np.allclose(g[0], [3, 5, 4, 0.0, 0.6, 0.8, 0, 0, 1, 0, 0, 0], atol=1e-14)
    assert np.allclose(g[1, :6], [2, 2, 2, 0.5, 0.5, 0.5], atol=1e-14)
    assert np.allclose(g[1, 6:9], [0, -1, 0], atol=1e-14)            # (x2-x1) x (x3-x1) = (2,0,0) x (1,0,sqrt3)
    assert np.allclose(g[1, 9:], [1, 1, 1 + np.sqrt(3.0)])
    # corner order matters: rotating the corners rotates l and theta together, the normal stays
    g2 = og.facet_geometry(v, f[:, [1, 2, 0]])
    assert np.allclose(g2[0, :6], [5, 4, 3, 0.6, 0.8, 0.0], atol=1e-14) and np.allclose(g2[0, 6:9], [0, 0, 1])
    # swapping two corners flips the normal
    assert np.allclose(og.facet_geometry(v, f[:, [0, 2, 1]])[0, 6:9], [0, 0, -1])


def test_law_of_cosines_angle_sum_and_invariances():
    rng = np.random.default_rng(0)
    v = rng.standard_normal((50, 3))
    f = np.stack([rng.permutation(50)[:3] for _ in range(200)])
    g = og.facet_geometry(v, f)
    l1, l2, l3, t1, t2, t3 = g[:, :6].T
    # law of cosines at each corner: the opposite side of corner 1 is l2, of corner 2 is l3, of corner 3 is l1
    assert np.allclose(l2 ** 2, l1 ** 2 + l3 ** 2 - 2 * l1 * l3 * t1)
    assert np.allclose(l3 ** 2, l1 ** 2 + l2 ** 2 - 2 * l1 * l2 * t2)
    assert np.allclose(l1 ** 2, l2 ** 2 + l3 ** 2 - 2 * l2 * l3 * t3)
    assert np.allclose(np.arccos(t1) + np.arccos(t2) + np.arccos(t3), np.pi)
    n = g[:, 6:9]
    assert np.allclose(np.linalg.norm(n, axis=1), 1)
    for a, b in ((1, 0), (2, 0), (2, 1)):
        assert np.allclose(np.einsum("ij,ij->i", n, v[f[:, a]] - v[f[:, b]]), 0, atol=1e-12)
    # rotation + translation + scale: lengths scale, cosines stay, normals rotate
    q, _ = np.linalg.qr(rng.standard_normal((3, 3)))
    q *= np.sign(np.linalg.det(q))
    g2 = og.facet_geometry(2.5 * v @ q.T + np.array([1.0, -2.0, 3.0]), f)
    assert np.allclose(g2[:, :3], 2.5 * g[:, :3]) and np.allclose(g2[:, 3:6], g[:, 3:6]) and np.allclose(g2[:, 6:9], n @ q.T)


def test_degenerate_facets():
    v = np.array([[0, 0, 0], [1, 0, 0], [2, 0, 0], [0, 0, 0]], np.float64)
    g = og.facet_geometry(v, np.array([[0, 1, 2], [0, 3, 1]]))
    assert np.allclose(g[0], [1, 1, 2, 1, -1, 1, 0, 0, 1])          # collinear: cosines +-1, fallback normal
    assert np.allclose(g[1], [0, 1, 1, 0, 0, 1, 0, 0, 1])           # repeated point: zero-length products give 0


def test_texture_resolution_extremes_counts_and_lattice():
    rng = np.random.default_rng(1)
    b = mg.pack_batch([mg.heightfield(9, 7, rng), mg.icosphere(1), mg.heightfield(4, 4, rng)])
    alpha, beta = 3, 1
    gamma = og.texture_resolution(b.vert, b.facet, b.facet_off, alpha, beta)
    A = og.facet_area(b.vert, b.facet)
    for m in range(b.n_mesh):
        s = slice(int(b.facet_off[m]), int(b.facet_off[m + 1]))
        a, g = A[s], gamma[s]
        assert g[np.argmin(a)] == beta and g[np.argmax(a)] == alpha + beta      # per-mesh extremes
        assert g.min() >= beta and g.max() <= alpha + beta
        order = np.argsort(a, kind="stable")
        assert np.all(np.diff(g[order]) >= 0)                                    # monotone in the area
    # the area against Heron's formula on the edge lengths of the separately pinned Eq. 9 oracle
    l1, l2, l3 = og.facet_geometry(b.vert, b.facet)[:, :3].T
    sp = 0.5 * (l1 + l2 + l3)
    assert np.allclose(A, np.sqrt(np.maximum(sp * (sp - l1) * (sp - l2) * (sp - l3), 0)), rtol=1e-9)
    off = og.texture_offsets(gamma)
    bary = og.texture_bary(gamma)
    assert off[-1] == bary.shape[0] and np.array_equal(np.diff(off), (gamma + 1) * (gamma + 2) // 2)
    assert np.allclose(bary.sum(axis=1), 1, atol=1e-6) and bary.min() >= 0
    for fi in (0, 5, int(np.argmax(gamma))):
        pts = bary[off[fi]:off[fi + 1]]
        assert np.unique(np.round(pts * gamma[fi]).astype(int), axis=0).shape[0] == pts.shape[0]   # all distinct
        for corner in np.eye(3):
            assert (np.abs(pts - corner).sum(axis=1) < 1e-6).any()                                # corners included
    # the input generator of the facet2facet tests draws its layouts by the same rule (a check of the generator)
    tex_off, bary_gen = mg.texture_layout(b, alpha, beta)
    assert np.array_equal(tex_off, off) and np.array_equal(bary_gen, bary)


def test_texture_resolution_worked_by_hand():
    """Right triangles with legs (1, a) in the plane: areas a/2 = 0.5, 0.75, 1.0, 1.25, 1.7, 2.0.  With alpha = 3:
    q = 3 (A - 0.5) / 1.5 = 0, 0.5, 1, 1.5, 2.4, 3 and gamma - beta = 0, 0, 1, 1, 2, 3 (q = 1 exactly: floor keeps it)."""
    legs = [1.0, 1.5, 2.0, 2.5, 3.4, 4.0]
    v, f = [], []
    for i, a in enumerate(legs):
        o = 10.0 * i
        v += [[o, 0, 0], [o + 1, 0, 0], [o, a, 0]]
        f.append([3 * i, 3 * i + 1, 3 * i + 2])
    v, f = np.array(v, np.float32), np.array(f)
    assert np.allclose(og.facet_area(v, f), [0.5, 0.75, 1.0, 1.25, 1.7, 2.0], rtol=1e-6)
    assert np.allclose(og.texture_ratio(v, f, [0, 6], 3), [0, 0.5, 1, 1.5, 2.4, 3], atol=1e-6)
    assert list(og.texture_resolution(v, f, [0, 6], 3, 1)) == [1, 1, 2, 2, 3, 4]
    assert list(og.texture_resolution(v, f, [0, 6], 3, 0)) == [0, 0, 1, 1, 2, 3]
    # two meshes: each takes its own extremes (facets 0-2: areas 0.5..1.0 -> q = 0, 1.5, 3; facets 3-5: 1.25..2.0 -> 0, 1.8, 3)
    assert list(og.texture_resolution(v, f, [0, 3, 6], 3, 1)) == [1, 2, 4, 1, 2, 4]
    assert list(np.diff(og.texture_offsets(og.texture_resolution(v, f, [0, 6], 3, 1)))) == [3, 3, 6, 6, 10, 15]


def test_single_area_mesh_and_the_point_count_formula():
    v = np.array([[0, 0, 0], [1, 0, 0], [0, 1, 0], [1, 1, 0]], np.float32)
    f = np.array([[0, 1, 2], [1, 3, 2]])
    g = og.texture_resolution(v, f, [0, 2], 5, 2)
    assert list(g) == [2, 2]                                      # equal areas: gamma = beta
    assert list(np.diff(og.texture_offsets(np.arange(5)))) == [1, 3, 6, 10, 15]
    assert np.allclose(og.texture_bary([0]), 1 / 3) and og.texture_bary([2]).shape == (6, 3)
    assert np.array_equal(og.texture_bary([1]), np.array([[1, 0, 0], [0, 1, 0], [0, 0, 1]], np.float32))

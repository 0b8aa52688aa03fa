"""CPU oracle of the facet geometric features (Section "Geometric Features", Eq. 9) and of the texture
resolution rule (Eq. 8) -- TEST INFRASTRUCTURE, not the product.  Plain numpy; shares nothing with the HIP path.

Eq. 9: edge lengths l1 = |x2-x1|, l2 = |x3-x2|, l3 = |x1-x3| (the pairing the denominators of Eq. 9 fix), the
three normalised inner products of the edges meeting at each corner (the paper calls them inner angles; they
are their cosines and are kept as cosines), the unit normal (x2-x1) x (x3-x1), optionally the three heights
z1, z2, z3.  Feature order per facet: [l1 l2 l3, theta1 theta2 theta3, nx ny nz, (z1 z2 z3)], fp64.
Readings: a corner whose two edges have a zero length product gets theta = 0; a facet whose cross product has
squared length < 1e-30 gets the normal (0, 0, 1).

Eq. 8: gamma = floor(alpha (A - Amin) / (Amax - Amin)) + beta with the extreme areas taken per mesh of the
batch, K = (gamma+1)(gamma+2)/2 points per facet.  A floating-point value decides an integer here, so the
decision is taken in the kernel's precision: fp32, one IEEE operation at a time, in this order:
  e1 = x2-x1, e2 = x3-x1, c = e1 x e2 (each component a*b - c*d as two products and a difference),
  A = 0.5 * sqrt((cx*cx + cy*cy) + cz*cz),  q = (float(alpha) * (A - Amin)) / (Amax - Amin),  gamma = floor(q) + beta;
Amax == Amin (or a mesh with one facet) gives gamma = beta.  The interpolation points of a facet are the
lattice (i, j, gamma-i-j)/gamma, i descending then j descending, and the centroid for gamma = 0.

Parity status: pinned by tests/test_oracle_geom.py.
"""
from __future__ import annotations

import numpy as np


def facet_geometry(vert, facet, with_heights: bool = False) -> np.ndarray:
    v = np.asarray(vert, dtype=np.float64)
    f = np.asarray(facet, dtype=np.int64)
    x1, x2, x3 = v[f[:, 0]], v[f[:, 1]], v[f[:, 2]]
    l1 = np.linalg.norm(x2 - x1, axis=1)
    l2 = np.linalg.norm(x3 - x2, axis=1)
    l3 = np.linalg.norm(x1 - x3, axis=1)

    def cosine(a, b, la, lb):
        den = la * lb
        dot = np.einsum("ij,ij->i", a, b)
        return np.where(den > 0, dot / np.where(den > 0, den, 1.0), 0.0)
    t1 = cosine(x2 - x1, x3 - x1, l1, l3)
    t2 = cosine(x1 - x2, x3 - x2, l1, l2)
    t3 = cosine(x1 - x3, x2 - x3, l3, l2)
    c = np.cross(x2 - x1, x3 - x1)
    n2 = np.einsum("ij,ij->i", c, c)
    ok = n2 >= 1e-30
    n = np.where(ok[:, None], c / np.sqrt(np.where(ok, n2, 1.0))[:, None], np.array([0.0, 0.0, 1.0])[None, :])
    cols = [l1, l2, l3, t1, t2, t3, n[:, 0], n[:, 1], n[:, 2]]
    if with_heights:
        cols += [x1[:, 2], x2[:, 2], x3[:, 2]]
    return np.stack(cols, axis=1)


def facet_area_f32(vert, facet) -> np.ndarray:
    """Facet areas in fp32, one rounding per operation, in the order the header states."""
    v = np.asarray(vert, dtype=np.float32)
    f = np.asarray(facet, dtype=np.int64)
    e1 = v[f[:, 1]] - v[f[:, 0]]
    e2 = v[f[:, 2]] - v[f[:, 0]]
    cx = e1[:, 1] * e2[:, 2] - e1[:, 2] * e2[:, 1]
    cy = e1[:, 2] * e2[:, 0] - e1[:, 0] * e2[:, 2]
    cz = e1[:, 0] * e2[:, 1] - e1[:, 1] * e2[:, 0]
    s = (cx * cx + cy * cy) + cz * cz
    return (np.float32(0.5) * np.sqrt(s)).astype(np.float32)


def texture_resolution(vert, facet, facet_off, alpha: int, beta: int) -> np.ndarray:
    """gamma [F] int32 of Eq. 8, extreme areas per mesh (facet_off [n_mesh+1])."""
    A = facet_area_f32(vert, facet)
    gamma = np.full(A.shape[0], beta, dtype=np.int32)
    off = np.asarray(facet_off, dtype=np.int64)
    for m in range(off.shape[0] - 1):
        a = A[off[m]:off[m + 1]]
        if a.size == 0:
            continue
        lo, hi = a.min(), a.max()
        if hi > lo:
            q = (np.float32(alpha) * (a - lo)) / (hi - lo)
            gamma[off[m]:off[m + 1]] = np.floor(q).astype(np.int32) + beta
    return gamma


def texture_offsets(gamma) -> np.ndarray:
    g = np.asarray(gamma, dtype=np.int64)
    off = np.zeros(g.shape[0] + 1, dtype=np.int64)
    np.cumsum((g + 1) * (g + 2) // 2, out=off[1:])
    return off


def texture_bary(gamma) -> np.ndarray:
    """Interpolation points of every facet, [P, 3] float32."""
    out = []
    for g in np.asarray(gamma, dtype=np.int64):
        if g == 0:
            out.append([1.0 / 3.0] * 3)
            continue
        for i in range(g, -1, -1):
            for j in range(g - i, -1, -1):
                out.append([i / g, j / g, (g - i - j) / g])
    return np.asarray(out, dtype=np.float64).reshape(-1, 3).astype(np.float32)

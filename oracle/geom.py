"""CPU oracle of the facet geometric features (Section "Geometric Features", Eq. 9) and of the texture
resolution rule (Eq. 8) -- TEST INFRASTRUCTURE, not the product.  Plain numpy; shares nothing with the HIP path.

Eq. 9: edge lengths l1 = |x2-x1|, l2 = |x3-x2|, l3 = |x1-x3| (the pairing the denominators of Eq. 9 fix), the
three normalised inner products of the edges meeting at each corner (the paper calls them inner angles; they
are their cosines and are kept as cosines), the unit normal (x2-x1) x (x3-x1), optionally the three heights
z1, z2, z3.  Feature order per facet: [l1 l2 l3, theta1 theta2 theta3, nx ny nz, (z1 z2 z3)], fp64.
Readings: a corner whose two edges have a zero length product gets theta = 0; a facet whose cross product has
squared length < 1e-30 gets the normal (0, 0, 1).

Eq. 8: gamma = floor(alpha (A - Amin) / (Amax - Amin)) + beta with the extreme areas taken per mesh of the
batch, K = (gamma+1)(gamma+2)/2 points per facet.  Evaluated as written, in fp64, from the fp32 vertex positions:
A = |(x2-x1) x (x3-x1)| / 2, q = alpha ((A - Amin) / (Amax - Amin)), gamma = floor(q) + beta; Amax == Amin (or a mesh
with one facet) gives gamma = beta.  A floor of a real number has no tolerance: a data path that evaluates q in
lower precision may land on the other side of an integer when q is within its rounding error of one, and both
values are then valid -- texture_ratio returns q so that a comparison can tell those facets apart (the extreme
facets, q = 0 and q = alpha, are exact in any precision).  The interpolation points of a facet are the lattice
(i, j, gamma-i-j)/gamma, i descending then j descending, and the centroid for gamma = 0.

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


def facet_area(vert, facet) -> np.ndarray:
    """Facet areas |(x2-x1) x (x3-x1)| / 2 in fp64."""
    v = np.asarray(vert, dtype=np.float64)
    f = np.asarray(facet, dtype=np.int64)
    return 0.5 * np.linalg.norm(np.cross(v[f[:, 1]] - v[f[:, 0]], v[f[:, 2]] - v[f[:, 0]]), axis=1)


def texture_ratio(vert, facet, facet_off, alpha: int) -> np.ndarray:
    """q [F] = alpha (A - Amin) / (Amax - Amin) of Eq. 8 in fp64, extreme areas per mesh; 0 where Amax == Amin."""
    A = facet_area(vert, facet)
    q = np.zeros(A.shape[0], dtype=np.float64)
    off = np.asarray(facet_off, dtype=np.int64)
    for m in range(off.shape[0] - 1):
        a = A[off[m]:off[m + 1]]
        if a.size == 0:
            continue
        lo, hi = a.min(), a.max()
        if hi > lo:
            q[off[m]:off[m + 1]] = alpha * ((a - lo) / (hi - lo))
    return q


def texture_resolution(vert, facet, facet_off, alpha: int, beta: int) -> np.ndarray:
    """gamma [F] int32 of Eq. 8."""
    return np.floor(texture_ratio(vert, facet, facet_off, alpha)).astype(np.int32) + np.int32(beta)


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

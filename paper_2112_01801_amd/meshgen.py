"""Seeded synthetic mesh and feature generators.

This module only *creates inputs* (geometry, index arrays, random features, random
filter coefficients, host-side rounding of inputs to bf16).  It holds none of the
arithmetic of the mesh convolutions: no spherical harmonics, no adjacency, no
contraction.  Both the CPU oracle's tests and the HIP path's tests draw their inputs
from here so that the two sides see bit-identical arrays.  Neither the HIP library nor
its Python binding imports it.

Two input recipes follow rules the paper states, because the synthetic inputs are meant
to have the structure of the paper's: the facet2facet texture layouts are drawn by the
area rule of Eq. 8 (`texture_layout`), and the coarse levels of the hierarchy by a 2x2
vertex clustering with mean positions (`cluster_grid_2x2`).  They shape inputs only: the
device-side Eq. 8 (`pm_texture_layout`) is checked against the oracle in `oracle/geom.py`,
never against this module, and the library takes any layout a caller supplies.

Meshes are returned in the packed heterogeneous-batch layout of the paper's
"Heterogeneous Batching" subsection: vertex arrays concatenated, facet index arrays
concatenated with the running vertex count added, 0-indexed.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

BASE_SEED = 20211201


def rng_for(config_id: int, stream: int = 0) -> np.random.Generator:
    """Deterministic generator for a config; `stream` separates independent draws."""
    return np.random.Generator(np.random.PCG64([BASE_SEED + config_id, stream]))


# --------------------------------------------------------------------------------------
# elementary closed shapes
# --------------------------------------------------------------------------------------
def tetrahedron() -> Tuple[np.ndarray, np.ndarray]:
    """Regular tetrahedron centred at the origin, outward-facing (right-hand rule)."""
    v = np.array([[1, 1, 1], [1, -1, -1], [-1, 1, -1], [-1, -1, 1]], dtype=np.float64)
    v /= np.sqrt(3.0)
    f = np.array([[0, 1, 2], [0, 3, 1], [0, 2, 3], [1, 3, 2]], dtype=np.int32)
    f = _orient_outward(v, f)
    return v.astype(np.float32), f


def icosahedron() -> Tuple[np.ndarray, np.ndarray]:
    """Regular icosahedron on the unit sphere, outward-facing."""
    p = (1.0 + np.sqrt(5.0)) / 2.0
    v = np.array(
        [[-1, p, 0], [1, p, 0], [-1, -p, 0], [1, -p, 0],
         [0, -1, p], [0, 1, p], [0, -1, -p], [0, 1, -p],
         [p, 0, -1], [p, 0, 1], [-p, 0, -1], [-p, 0, 1]], dtype=np.float64)
    v /= np.linalg.norm(v, axis=1, keepdims=True)
    f = np.array(
        [[0, 11, 5], [0, 5, 1], [0, 1, 7], [0, 7, 10], [0, 10, 11],
         [1, 5, 9], [5, 11, 4], [11, 10, 2], [10, 7, 6], [7, 1, 8],
         [3, 9, 4], [3, 4, 2], [3, 2, 6], [3, 6, 8], [3, 8, 9],
         [4, 9, 5], [2, 4, 11], [6, 2, 10], [8, 6, 7], [9, 8, 1]], dtype=np.int32)
    f = _orient_outward(v, f)
    return v.astype(np.float32), f


def _orient_outward(v: np.ndarray, f: np.ndarray) -> np.ndarray:
    """Flip facets of a star-shaped closed mesh (about the origin) so normals point out."""
    a, b, c = v[f[:, 0]], v[f[:, 1]], v[f[:, 2]]
    n = np.cross(b - a, c - a)
    inward = np.einsum("ij,ij->i", n, a + b + c) < 0
    f = f.copy()
    f[inward] = f[inward][:, [0, 2, 1]]
    return f


def icosphere_f64(level: int) -> Tuple[np.ndarray, np.ndarray]:
    """Icosphere by `level` rounds of midpoint subdivision (V = 10*4^level + 2)."""
    v32, f = icosahedron()
    v = v32.astype(np.float64)
    v /= np.linalg.norm(v, axis=1, keepdims=True)
    for _ in range(level):
        nv = v.shape[0]
        e = np.concatenate([f[:, [0, 1]], f[:, [1, 2]], f[:, [2, 0]]], axis=0).astype(np.int64)
        e.sort(axis=1)
        key = e[:, 0] * nv + e[:, 1]
        uniq, inv = np.unique(key, return_inverse=True)
        mid = 0.5 * (v[uniq // nv] + v[uniq % nv])
        mid /= np.linalg.norm(mid, axis=1, keepdims=True)
        v = np.concatenate([v, mid], axis=0)
        nf = f.shape[0]
        m01 = (nv + inv[0:nf]).astype(np.int32)
        m12 = (nv + inv[nf:2 * nf]).astype(np.int32)
        m20 = (nv + inv[2 * nf:3 * nf]).astype(np.int32)
        a, b, c = f[:, 0], f[:, 1], f[:, 2]
        f = np.concatenate([
            np.stack([a, m01, m20], 1), np.stack([b, m12, m01], 1),
            np.stack([c, m20, m12], 1), np.stack([m01, m12, m20], 1)], axis=0).astype(np.int32)
    return v, f


def icosphere(level: int) -> Tuple[np.ndarray, np.ndarray]:
    v, f = icosphere_f64(level)
    return v.astype(np.float32), f


# --------------------------------------------------------------------------------------
# open surfaces (scene stand-ins)
# --------------------------------------------------------------------------------------
def grid_facets(nx: int, ny: int, diag: Optional[np.ndarray] = None) -> np.ndarray:
    """Triangulate an nx-by-ny vertex grid (vertex id = i*ny + j).

    diag[i, j] == 0 splits cell (i, j) along (i,j)-(i+1,j+1); 1 along (i+1,j)-(i,j+1).
    Facets of a cell are consecutive (2*cell, 2*cell+1), counter-clockwise seen from +z
    when x grows with i and y grows with j.
    """
    i, j = np.meshgrid(np.arange(nx - 1), np.arange(ny - 1), indexing="ij")
    v00 = (i * ny + j).ravel()
    v10 = ((i + 1) * ny + j).ravel()
    v01 = (i * ny + j + 1).ravel()
    v11 = ((i + 1) * ny + j + 1).ravel()
    if diag is None:
        t0 = np.stack([v00, v10, v11], 1)
        t1 = np.stack([v00, v11, v01], 1)
    else:
        d = diag.ravel().astype(bool)
        t0 = np.where(d[:, None], np.stack([v00, v10, v01], 1), np.stack([v00, v10, v11], 1))
        t1 = np.where(d[:, None], np.stack([v10, v11, v01], 1), np.stack([v00, v11, v01], 1))
    f = np.empty((2 * t0.shape[0], 3), dtype=np.int32)
    f[0::2] = t0
    f[1::2] = t1
    return f


def heightfield(nx: int, ny: int, rng: np.random.Generator, *, random_diag: bool = False,
                extent: Tuple[float, float] = (1.0, 1.0)) -> Tuple[np.ndarray, np.ndarray]:
    """Height-field on [0,ex]x[0,ey]: z = sum of 8 random sinusoids + N(0, 0.01) noise."""
    amp = rng.uniform(0.01, 0.05, size=8)
    fx = rng.integers(1, 9, size=8)
    fy = rng.integers(1, 9, size=8)
    ph = rng.uniform(0.0, 2.0 * np.pi, size=8)
    x = np.linspace(0.0, extent[0], nx)
    y = np.linspace(0.0, extent[1], ny)
    X, Y = np.meshgrid(x, y, indexing="ij")
    Z = np.zeros_like(X)
    for q in range(8):
        Z += amp[q] * np.sin(2.0 * np.pi * (fx[q] * X / extent[0] + fy[q] * Y / extent[1]) + ph[q])
    Z += rng.normal(0.0, 0.01, size=Z.shape)
    diag = rng.integers(0, 2, size=(nx - 1, ny - 1)) if random_diag else None
    v = np.stack([X.ravel(), Y.ravel(), Z.ravel()], 1).astype(np.float32)
    return v, grid_facets(nx, ny, diag)


def delete_facets(f: np.ndarray, frac: float, rng: np.random.Generator) -> np.ndarray:
    """Drop a uniformly random fraction of facets; vertices are kept (some become isolated)."""
    keep = rng.random(f.shape[0]) >= frac
    return np.ascontiguousarray(f[keep])


def cluster_grid_2x2(v: np.ndarray, nx: int, ny: int) -> Tuple[np.ndarray, np.ndarray, int, int]:
    """Uniform vertex clustering of a fixed-diagonal grid mesh in 2x2 blocks.

    Cluster position = mean of its members; facets are remapped, degenerate and duplicate
    facets dropped.  For a fixed-diagonal grid this yields the fixed-diagonal grid of the
    cluster lattice, in the same facet order convention as `grid_facets`.
    """
    assert nx % 2 == 0 and ny % 2 == 0
    cx, cy = nx // 2, ny // 2
    vv = v.reshape(nx, ny, 3).astype(np.float64)
    vc = vv.reshape(cx, 2, cy, 2, 3).mean(axis=(1, 3))
    i = np.arange(nx)[:, None] // 2
    j = np.arange(ny)[None, :] // 2
    cmap = (i * cy + j).ravel().astype(np.int32)
    f = grid_facets(nx, ny)
    g = cmap[f]
    ok = (g[:, 0] != g[:, 1]) & (g[:, 1] != g[:, 2]) & (g[:, 0] != g[:, 2])
    g = g[ok]
    # drop duplicates irrespective of rotation of the corner order, keep first occurrence
    rot = np.argmin(g, axis=1)
    canon = np.stack([np.take_along_axis(g, ((rot + s) % 3)[:, None], 1)[:, 0] for s in range(3)], 1)
    _, first = np.unique(canon, axis=0, return_index=True)
    g = g[np.sort(first)]
    return vc.reshape(-1, 3).astype(np.float32), np.ascontiguousarray(g.astype(np.int32)), cx, cy


def grid_cluster_maps(nx: int, ny: int) -> Tuple[np.ndarray, np.ndarray]:
    """(VCluster, IOmap) of `cluster_grid_2x2`: the representative of a 2x2 block is its vertex with even
    grid coordinates, and it maps to the block's index in the coarse grid; every other IOmap entry is -1."""
    assert nx % 2 == 0 and ny % 2 == 0
    cy = ny // 2
    i = np.arange(nx)[:, None]
    j = np.arange(ny)[None, :]
    vcluster = ((i // 2 * 2) * ny + (j // 2 * 2)).ravel().astype(np.int32)
    iomap = np.full(nx * ny, -1, np.int32)
    rep = np.unique(vcluster)
    iomap[rep] = ((rep // ny) // 2 * cy + (rep % ny) // 2).astype(np.int32)
    return vcluster, iomap


def random_cluster_maps(rng: np.random.Generator, n_in: int, n_out: int, drop_frac: float = 0.0,
                        heavy: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """(VCluster, IOmap) of a random clustering shaped like an edge-contraction decimation: `n_out` distinct
    representatives in random output order, every other vertex joins a random one; `heavy` extra vertices all
    join the first representative (one long cluster); a fraction of the vertices joins a dead representative
    whose IOmap is -1 (they reach no output vertex)."""
    assert 0 < n_out <= n_in
    perm = rng.permutation(n_in)
    rep = perm[:n_out]
    dead = perm[n_out] if n_out < n_in else -1
    vcluster = np.empty(n_in, np.int32)
    vcluster[rep] = rep
    rest = perm[n_out:]
    vcluster[rest] = rep[rng.integers(0, n_out, rest.size)]
    vcluster[rest[:min(heavy, rest.size)]] = rep[0]
    if dead >= 0 and drop_frac > 0:
        d = rest[rng.random(rest.size) < drop_frac]
        vcluster[d] = dead
        vcluster[dead] = dead
    iomap = np.full(n_in, -1, np.int32)
    iomap[rep] = rng.permutation(n_out).astype(np.int32)
    return vcluster, iomap


def range_neighbors(xq: np.ndarray, xs: np.ndarray, rho: float, max_nbr: int = 0,
                    rng: Optional[np.random.Generator] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Neighbour lists of a range search (all sources within rho of each query), as CSR (ptr [M+1], idx) with
    ascending source ids; lists longer than `max_nbr` (> 0) keep a random subset.  Input preparation only:
    the search itself is not part of the library."""
    from scipy.spatial import cKDTree
    lists = cKDTree(np.asarray(xs, np.float64)).query_ball_point(np.asarray(xq, np.float64), rho)
    out = []
    for l in lists:
        l = np.sort(np.asarray(l, dtype=np.int64))
        if max_nbr > 0 and l.shape[0] > max_nbr:
            l = np.sort(rng.choice(l, max_nbr, replace=False))
        out.append(l)
    ptr = np.zeros(len(out) + 1, np.int64)
    np.cumsum([l.shape[0] for l in out], out=ptr[1:])
    assert ptr[-1] < 2 ** 31
    idx = np.concatenate(out) if out else np.zeros(0, np.int64)
    return ptr.astype(np.int32), idx.astype(np.int32)


# --------------------------------------------------------------------------------------
# batching
# --------------------------------------------------------------------------------------
@dataclass
class MeshBatch:
    vert: np.ndarray          # [V,3] float32
    facet: np.ndarray         # [F,3] int32, global ids
    vert_off: np.ndarray      # [n_mesh+1] int32
    facet_off: np.ndarray     # [n_mesh+1] int32

    @property
    def n_vert(self) -> int:
        return int(self.vert.shape[0])

    @property
    def n_facet(self) -> int:
        return int(self.facet.shape[0])

    @property
    def n_mesh(self) -> int:
        return int(self.vert_off.shape[0] - 1)

    def mesh(self, i: int) -> "MeshBatch":
        v0, v1 = int(self.vert_off[i]), int(self.vert_off[i + 1])
        f0, f1 = int(self.facet_off[i]), int(self.facet_off[i + 1])
        return pack_batch([(self.vert[v0:v1], self.facet[f0:f1] - v0)])


def pack_batch(meshes: Sequence[Tuple[np.ndarray, np.ndarray]]) -> MeshBatch:
    vs, fs, vo, fo = [], [], [0], [0]
    for v, f in meshes:
        fs.append(np.asarray(f, dtype=np.int32) + np.int32(vo[-1]))
        vs.append(np.asarray(v, dtype=np.float32))
        vo.append(vo[-1] + v.shape[0])
        fo.append(fo[-1] + f.shape[0])
    return MeshBatch(np.ascontiguousarray(np.concatenate(vs, 0)),
                     np.ascontiguousarray(np.concatenate(fs, 0)),
                     np.asarray(vo, dtype=np.int32), np.asarray(fo, dtype=np.int32))


# --------------------------------------------------------------------------------------
# textures for facet2facet inputs (the area rule of Eq. 8 shapes the synthetic input only)
# --------------------------------------------------------------------------------------
def bary_lattice(gamma: int) -> np.ndarray:
    """(gamma+1)(gamma+2)/2 barycentric lattice points (i,j,k)/gamma; centroid if gamma=0."""
    if gamma == 0:
        return np.full((1, 3), 1.0 / 3.0, dtype=np.float32)
    pts = [(i, j, gamma - i - j) for i in range(gamma, -1, -1) for j in range(gamma - i, -1, -1)]
    return (np.asarray(pts, dtype=np.float64) / gamma).astype(np.float32)


def texture_layout(batch: MeshBatch, alpha: int, beta: int) -> Tuple[np.ndarray, np.ndarray]:
    """Per-facet texture resolution from facet area (per mesh A_min/A_max), lattice points.

    Returns (tex_off [F+1] int32, bary [P,3] float32); points of a facet are contiguous.
    """
    v = batch.vert.astype(np.float64)
    f = batch.facet
    area = 0.5 * np.linalg.norm(np.cross(v[f[:, 1]] - v[f[:, 0]], v[f[:, 2]] - v[f[:, 0]]), axis=1)
    gamma = np.empty(f.shape[0], dtype=np.int64)
    for m in range(batch.n_mesh):
        f0, f1 = int(batch.facet_off[m]), int(batch.facet_off[m + 1])
        a = area[f0:f1]
        if a.size == 0:
            continue
        lo, hi = a.min(), a.max()
        if hi > lo:
            gamma[f0:f1] = np.floor(alpha * ((a - lo) / (hi - lo))).astype(np.int64) + beta
        else:
            gamma[f0:f1] = beta
    res = (gamma + 1) * (gamma + 2) // 2
    tex_off = np.zeros(f.shape[0] + 1, dtype=np.int64)
    np.cumsum(res, out=tex_off[1:])
    bary = np.empty((int(tex_off[-1]), 3), dtype=np.float32)
    for g in np.unique(gamma):
        lat = bary_lattice(int(g))
        idx = np.nonzero(gamma == g)[0]
        pos = tex_off[idx][:, None] + np.arange(lat.shape[0])[None, :]
        bary[pos.ravel()] = np.tile(lat, (idx.size, 1))
    assert tex_off[-1] < 2 ** 31
    return tex_off.astype(np.int32), bary


# --------------------------------------------------------------------------------------
# features, filter coefficients, bf16 input rounding
# --------------------------------------------------------------------------------------
def glorot_coeffs(rng: np.random.Generator, K: int, cin: int, cout: int) -> np.ndarray:
    a = np.sqrt(6.0 / (K * cin + cout))
    return rng.uniform(-a, a, size=(K, cin, cout)).astype(np.float32)


def normal_features(rng: np.random.Generator, n: int, c: int) -> np.ndarray:
    return rng.standard_normal(size=(n, c), dtype=np.float32)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 to the nearest bf16 (ties to even); returns float32 holding bf16 values."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + r) & np.uint32(0xFFFF0000)).view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of an array that already holds bf16-representable float32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    assert not np.any(u & np.uint32(0xFFFF)), "values are not bf16-representable"
    return (u >> 16).astype(np.uint16)


def bf16_from_bits(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


# --------------------------------------------------------------------------------------
# the five benchmark configurations
# --------------------------------------------------------------------------------------
@dataclass
class Config:
    name: str
    L: int
    dtype: str                      # "f32" | "bf16"
    batch: MeshBatch
    cin: int
    cout: int
    info: Dict[str, object] = field(default_factory=dict)

    @property
    def K(self) -> int:
        return (self.L + 1) ** 2


def config1() -> Config:
    rng = rng_for(1)
    v, f = icosphere_f64(3)
    v = v * (1.0 + rng.uniform(-0.05, 0.05, size=(v.shape[0], 1)))
    return Config("c1_icosphere3", 3, "f32", pack_batch([(v.astype(np.float32), f)]), 16, 16)


def config2(n_mesh: int = 16) -> Config:
    rng = rng_for(2)
    meshes = []
    levels = []
    for _ in range(n_mesh):
        lvl = int(rng.integers(4, 6))
        levels.append(lvl)
        v, f = icosphere_f64(lvl)
        v = v * (1.0 + rng.normal(0.0, 0.02, size=(v.shape[0], 1)))
        v = v * rng.uniform(0.5, 1.5, size=(1, 3))
        meshes.append((v.astype(np.float32), f))
    return Config("c2_shapes16", 3, "f32", pack_batch(meshes), 64, 64, {"levels": levels})


def config3(n: int = 1024) -> Config:
    rng = rng_for(3)
    v, f = heightfield(n, n, rng)
    return Config("c3_heightfield%d" % n, 3, "bf16", pack_batch([(v, f)]), 64, 64, {"nx": n, "ny": n})


def config4(n_mesh: int = 8, fmin: int = 200_000, fmax: int = 1_500_000) -> Config:
    rng = rng_for(4)
    meshes, dims = [], []
    for _ in range(n_mesh):
        target = rng.uniform(fmin, fmax)
        aspect = np.exp(rng.uniform(np.log(0.25), np.log(4.0)))
        cells = target / 2.0 / 0.95
        nx = max(3, int(round(np.sqrt(cells * aspect))) + 1)
        ny = max(3, int(round(np.sqrt(cells / aspect))) + 1)
        v, f = heightfield(nx, ny, rng, random_diag=True, extent=(1.0, float(ny - 1) / float(nx - 1)))
        f = delete_facets(f, 0.05, rng)
        meshes.append((v, f))
        dims.append((nx, ny))
    return Config("c4_scenes%d" % n_mesh, 4, "f32", pack_batch(meshes), 32, 128, {"dims": dims})


def config5_levels(n: int = 1024, n_levels: int = 4) -> List[Config]:
    rng = rng_for(3)           # same mesh as config 3
    v, f = heightfield(n, n, rng)
    chans = (32, 64, 128, 256)
    out = []
    nx = ny = n
    for lvl in range(n_levels):
        out.append(Config("c5_level%d" % lvl, 3, "bf16", pack_batch([(v, f)]), chans[lvl], chans[lvl],
                          {"nx": nx, "ny": ny}))
        if lvl + 1 < n_levels:
            v, f, nx, ny = cluster_grid_2x2(v, nx, ny)
    return out

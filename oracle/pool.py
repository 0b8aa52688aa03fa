"""fp64 CPU oracle of mesh pooling / unpooling over vertex clusters -- TEST INFRASTRUCTURE, not the product.

Section "Mesh decimation", paragraph "(Un)poolings": decimation records two vectors of the input mesh's
vertex count, VCluster (the cluster of each input vertex) and IOmap (the mapping between input and output
vertices).  Pooling takes the maximum or the average of the features of a cluster; unpooling copies the
feature of the vertex the cluster was contracted to onto every member.

Reading used here (the paper gives no encoding): VCluster[v] is the input-mesh index of the representative
vertex of v's cluster, IOmap[u] is the output-mesh index of input vertex u when it is a representative and
-1 otherwise; so the output vertex of v is target(v) = IOmap[VCluster[v]], and -1 means v belongs to no output
vertex.  Maximum ties go to the lowest input index; an output vertex without members gets 0.

Plain numpy definitions (ufunc.at scatter forms); nothing here is shared with the HIP path.
Parity status: pinned by tests/test_oracle_pool.py (the paper's worked example, brute force, closed forms,
adjoint identities, finite differences).
"""
from __future__ import annotations

import numpy as np

POOL_MAX, POOL_AVG = 0, 1


def cluster_target(vcluster, iomap) -> np.ndarray:
    """target[v] = IOmap[VCluster[v]] (int64), -1 where there is none."""
    vcluster = np.asarray(vcluster, dtype=np.int64)
    iomap = np.asarray(iomap, dtype=np.int64)
    return iomap[vcluster]


def cluster_members(vcluster, iomap, n_out: int):
    """CSR (row_ptr [n_out+1], col) of the members of every output vertex, ascending."""
    t = cluster_target(vcluster, iomap)
    v = np.nonzero(t >= 0)[0]
    order = np.lexsort((v, t[v]))
    col = v[order].astype(np.int32)
    cnt = np.bincount(t[v], minlength=n_out)
    row_ptr = np.zeros(n_out + 1, np.int32)
    row_ptr[1:] = np.cumsum(cnt)
    return row_ptr, col


def pool(vcluster, iomap, n_out: int, h_in, mode: int):
    """Returns (h_out [n_out, C] fp64, argmax [n_out, C] int32 or None)."""
    h = np.asarray(h_in, dtype=np.float64)
    t = cluster_target(vcluster, iomap)
    v = np.nonzero(t >= 0)[0]
    C = h.shape[1]
    if mode == POOL_AVG:
        s = np.zeros((n_out, C))
        np.add.at(s, t[v], h[v])
        cnt = np.bincount(t[v], minlength=n_out).astype(np.float64)
        return s / np.maximum(cnt, 1.0)[:, None], None
    m = np.full((n_out, C), -np.inf)
    np.maximum.at(m, t[v], h[v])
    big = np.iinfo(np.int64).max
    arg = np.full((n_out, C), big, np.int64)
    cand = np.where(h[v] == m[t[v]], v[:, None], big)
    np.minimum.at(arg, t[v], cand)
    empty = arg == big
    m[empty] = 0.0
    arg[empty] = -1
    return m, arg.astype(np.int32)


def pool_bwd(vcluster, iomap, n_out: int, dg_out, mode: int, argmax=None) -> np.ndarray:
    """Gradient with respect to the input-mesh features, [n_in, C]."""
    dg = np.asarray(dg_out, dtype=np.float64)
    t = cluster_target(vcluster, iomap)
    n_in, C = t.shape[0], dg.shape[1]
    out = np.zeros((n_in, C))
    v = np.nonzero(t >= 0)[0]
    if mode == POOL_AVG:
        cnt = np.bincount(t[v], minlength=n_out).astype(np.float64)
        out[v] = dg[t[v]] / cnt[t[v]][:, None]
        return out
    arg = np.asarray(argmax, dtype=np.int64)
    out[v] = np.where(arg[t[v]] == v[:, None], dg[t[v]], 0.0)
    return out


def unpool(vcluster, iomap, h_coarse) -> np.ndarray:
    """Every input-mesh vertex takes the feature of its output vertex (0 where it has none)."""
    h = np.asarray(h_coarse, dtype=np.float64)
    t = cluster_target(vcluster, iomap)
    out = np.zeros((t.shape[0], h.shape[1]))
    v = np.nonzero(t >= 0)[0]
    out[v] = h[t[v]]
    return out


def unpool_bwd(vcluster, iomap, n_out: int, dg_fine) -> np.ndarray:
    dg = np.asarray(dg_fine, dtype=np.float64)
    t = cluster_target(vcluster, iomap)
    out = np.zeros((n_out, dg.shape[1]))
    v = np.nonzero(t >= 0)[0]
    np.add.at(out, t[v], dg[v])
    return out

"""Pins of the pooling / unpooling oracle: the paper's worked example, brute force with Python loops,
closed forms against numpy reductions, adjoint identities, finite differences."""
import os

import numpy as np
import pytest

from oracle import pool as op
from paper_2112_01801_amd import meshgen as mg

HERE = os.path.dirname(__file__)


def _brute(vc, io, n_out, h, mode):
    n_in, C = h.shape
    out = np.zeros((n_out, C))
    arg = -np.ones((n_out, C), np.int64)
    members = [[] for _ in range(n_out)]
    for v in range(n_in):
        t = io[vc[v]]
        if t >= 0:
            members[t].append(v)
    for o in range(n_out):
        for c in range(C):
            vals = [h[v, c] for v in members[o]]
            if not vals:
                continue
            if mode == op.POOL_AVG:
                out[o, c] = sum(vals) / len(vals)
            else:
                best = 0
                for i in range(1, len(vals)):
                    if vals[i] > vals[best]:
                        best = i
                out[o, c] = vals[best]
                arg[o, c] = members[o][best]
    return out, arg, members


def test_worked_example_of_the_vertex_cluster_figure():
    lines = [l.split() for l in open(os.path.join(HERE, "golden", "pool_worked_example.txt")) if not l.startswith("#")]
    names = "abcdefg"
    members = [names.index(x) for x in lines[0][1:]]
    out_v = int(lines[1][1])
    n_in = 7
    vc = np.arange(n_in, dtype=np.int32)
    vc[members] = members[0]
    io = np.full(n_in, -1, np.int32)
    reps = [v for v in range(n_in) if vc[v] == v]
    others = [o for o in range(len(reps)) if o != out_v]
    io[members[0]] = out_v
    for v, o in zip([r for r in reps if r != members[0]], others):
        io[v] = o
    rng = np.random.default_rng(5)
    h = rng.standard_normal((n_in, 3))
    m, _ = op.pool(vc, io, len(reps), h, op.POOL_MAX)
    assert np.array_equal(m[out_v], np.max(h[members], axis=0))
    up = op.unpool(vc, io, m)
    for v in members:
        assert np.array_equal(up[v], m[out_v])


@pytest.mark.parametrize("mode", [op.POOL_MAX, op.POOL_AVG])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_pool_brute_force_with_ties_drops_and_a_heavy_cluster(mode, seed):
    rng = np.random.default_rng(seed)
    n_in, n_out, C = 60, 13, 4
    vc, io = mg.random_cluster_maps(rng, n_in, n_out, drop_frac=0.2, heavy=15)
    h = rng.integers(-3, 4, (n_in, C)).astype(np.float64)       # few distinct values: many ties
    ref, rarg, members = _brute(vc, io, n_out, h, mode)
    got, arg = op.pool(vc, io, n_out, h, mode)
    assert np.allclose(got, ref, rtol=0, atol=1e-15)
    if mode == op.POOL_MAX:
        assert np.array_equal(arg, rarg)
    rp, col = op.cluster_members(vc, io, n_out)
    for o in range(n_out):
        assert list(col[rp[o]:rp[o + 1]]) == members[o]
    assert rp[-1] == sum(len(m) for m in members) < n_in          # some vertices were dropped


def test_closed_forms_identity_and_global():
    rng = np.random.default_rng(3)
    n, C = 37, 5
    h = rng.standard_normal((n, C))
    ident = np.arange(n, dtype=np.int32)
    for mode in (op.POOL_MAX, op.POOL_AVG):
        out, _ = op.pool(ident, ident, n, h, mode)
        assert np.array_equal(out, h)
    assert np.array_equal(op.unpool(ident, ident, h), h)
    # all vertices in one cluster: numpy's own reductions
    vc = np.zeros(n, np.int32)
    io = np.full(n, -1, np.int32)
    io[0] = 0
    m, arg = op.pool(vc, io, 1, h, op.POOL_MAX)
    assert np.array_equal(m[0], h.max(axis=0)) and np.array_equal(arg[0], h.argmax(axis=0))
    a, _ = op.pool(vc, io, 1, h, op.POOL_AVG)
    assert np.allclose(a[0], h.mean(axis=0), rtol=1e-14)
    # permuted output order
    perm = rng.permutation(n).astype(np.int32)
    out, _ = op.pool(ident, perm, n, h, op.POOL_MAX)
    assert np.array_equal(out[perm], h)


def test_grid_cluster_maps_match_the_2x2_block_mean_of_the_mesh_generator():
    nx, ny = 8, 6
    rng = np.random.default_rng(4)
    v, f = mg.heightfield(nx, ny, rng)
    vcoarse, _, cx, cy = mg.cluster_grid_2x2(v, nx, ny)
    vc, io = mg.grid_cluster_maps(nx, ny)
    pos, _ = op.pool(vc, io, cx * cy, v, op.POOL_AVG)
    assert np.allclose(pos, vcoarse, atol=1e-6)


def test_adjoint_identities_and_pool_of_unpool():
    rng = np.random.default_rng(6)
    n_in, n_out, C = 80, 17, 3
    vc, io = mg.random_cluster_maps(rng, n_in, n_out, drop_frac=0.1, heavy=9)
    x, y = rng.standard_normal((n_in, C)), rng.standard_normal((n_out, C))
    # <avgpool(x), y> = <x, avgpool_bwd(y)>
    a, _ = op.pool(vc, io, n_out, x, op.POOL_AVG)
    assert np.isclose((a * y).sum(), (x * op.pool_bwd(vc, io, n_out, y, op.POOL_AVG)).sum(), rtol=1e-12)
    # <unpool(y), x> = <y, unpool_bwd(x)>
    assert np.isclose((op.unpool(vc, io, y) * x).sum(), (y * op.unpool_bwd(vc, io, n_out, x)).sum(), rtol=1e-12)
    # pooling what unpooling made gives the coarse features back (every output vertex has its representative)
    for mode in (op.POOL_MAX, op.POOL_AVG):
        back, _ = op.pool(vc, io, n_out, op.unpool(vc, io, y), mode)
        assert np.allclose(back, y, rtol=1e-14)


def test_max_pool_backward_by_finite_differences_and_tie_rule():
    rng = np.random.default_rng(7)
    n_in, n_out, C = 40, 9, 2
    vc, io = mg.random_cluster_maps(rng, n_in, n_out, drop_frac=0.1)
    h = rng.permutation(n_in * C).reshape(n_in, C).astype(np.float64)     # all distinct, gaps of 1
    dg = rng.standard_normal((n_out, C))
    m, arg = op.pool(vc, io, n_out, h, op.POOL_MAX)
    got = op.pool_bwd(vc, io, n_out, dg, op.POOL_MAX, arg)
    eps = 1e-3
    for v in range(n_in):
        for c in range(C):
            hp, hm = h.copy(), h.copy()
            hp[v, c] += eps
            hm[v, c] -= eps
            fd = ((op.pool(vc, io, n_out, hp, op.POOL_MAX)[0] - op.pool(vc, io, n_out, hm, op.POOL_MAX)[0]) * dg).sum() / (2 * eps)
            assert abs(fd - got[v, c]) < 1e-9
    # ties: the lowest input index takes the whole gradient
    h2 = np.zeros((n_in, C))
    m2, arg2 = op.pool(vc, io, n_out, h2, op.POOL_MAX)
    g2 = op.pool_bwd(vc, io, n_out, dg, op.POOL_MAX, arg2)
    rp, col = op.cluster_members(vc, io, n_out)
    for o in range(n_out):
        assert np.array_equal(g2[col[rp[o]]], dg[o]) and not g2[col[rp[o] + 1:rp[o + 1]]].any()

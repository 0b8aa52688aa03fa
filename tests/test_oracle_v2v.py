"""Pins of the oracle's separable vertex2vertex block (CPU only).

The block is vertex2facet followed by facet2vertex (both separable), with a per-channel affine map and ReLU
after each.  Pins: (1) equality with the composition of the separately pinned separable oracles (C code, own
loops), the affine maps and ReLU applied here in between; (2) brute-force Python loops on a tetrahedron for
filters that keep only the constant harmonic; (3) the degenerate cases (isolated vertex, every facet feature
cut off by ReLU); (4) every gradient against central differences of the forward function.
"""
import numpy as np
import pytest

import oracle
from oracle import v2v
from paper_2112_01801_amd import meshgen as mg


def _mesh(seed=0):
    rng = np.random.default_rng(seed)
    v, f = mg.icosphere_f64(1)
    v = v * (1 + rng.normal(0, 0.05, (v.shape[0], 1)))
    v = np.concatenate([v, [[3.0, 3.0, 3.0]]], 0)            # one isolated vertex
    return v.astype(np.float32), f.astype(np.int32)


def _params(rng, L, cin, cmid, cout):
    K = (L + 1) ** 2
    return (rng.standard_normal((K, cin)), rng.standard_normal((cin, cmid)) / np.sqrt(cin),
            rng.standard_normal((K, cmid)), rng.standard_normal((cmid, cout)) / np.sqrt(cmid))


def _eps(rng, cmid, cout, relu1, relu2):
    return ((rng.uniform(0.5, 1.5, cmid), rng.normal(0, 0.3, cmid), relu1),
            (rng.uniform(0.5, 1.5, cout), rng.normal(0, 0.3, cout), relu2))


@pytest.mark.parametrize("L,norm,relu1,relu2,affine", [(3, 0, False, False, False), (2, 1, True, True, True),
                                                       (1, 0, True, False, True), (0, 0, False, True, False)])
def test_equals_composition_of_the_separable_oracles(L, norm, relu1, relu2, affine):
    rng = np.random.default_rng(5 + L)
    v, f = _mesh(2)
    cin, cmid, cout = 6, 5, 7
    a1, P1, a2, P2 = _params(rng, L, cin, cmid, cout)
    ep1, ep2 = _eps(rng, cmid, cout, relu1, relu2)
    if not affine:
        ep1, ep2 = (None, None, relu1), (None, None, relu2)
    h = rng.standard_normal((v.shape[0], cin))
    u = oracle.v2f_sep(v.shape[0], f, L, h, a1, P1, norm)
    if affine:
        u = ep1[0] * u + ep1[1]
    g = np.maximum(u, 0) if relu1 else u
    q = oracle.f2v_sep(v, f, L, g, a2, P2, norm)
    if affine:
        q = ep2[0] * q + ep2[1]
    ref = np.maximum(q, 0) if relu2 else q
    o, g_o, z_o = v2v.v2v_sep(v, f, L, h, a1, P1, ep1, a2, P2, ep2, norm, parts=True)
    np.testing.assert_allclose(o, ref, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(g_o, g, rtol=1e-11, atol=1e-12)


def test_constant_harmonic_brute_force_on_a_tetrahedron():
    # only B_0 (a constant) kept in both filters: the block is plain averaging, written with Python loops
    rng = np.random.default_rng(11)
    v, f = mg.tetrahedron()
    L, cin, cmid, cout = 2, 3, 4, 2
    K = (L + 1) ** 2
    a1, P1, a2, P2 = _params(rng, L, cin, cmid, cout)
    a1[1:] = 0
    a2[1:] = 0
    b0 = oracle.sh_basis(np.array([[0.3, -0.2, 0.9]]), L)[0, 0]       # the constant harmonic
    h = rng.standard_normal((v.shape[0], cin))
    ref = np.zeros((v.shape[0], cout))
    for vi in range(v.shape[0]):
        acc, n = np.zeros(cmid), 0
        for fi in range(f.shape[0]):
            if vi in f[fi]:
                t = np.zeros(cin)
                for j in range(3):
                    t += b0 * a1[0] * h[f[fi, j]]
                acc += b0 * a2[0] * np.maximum(t @ P1, 0.0)
                n += 1
        ref[vi] = (acc / n) @ P2
    got = v2v.v2v_sep(v, f, L, h, a1, P1, (None, None, True), a2, P2, None)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-13)
    assert K == a1.shape[0]


def test_degenerate_cases():
    rng = np.random.default_rng(12)
    v, f = _mesh(3)
    L, cin, cmid, cout = 2, 4, 4, 3
    a1, P1, a2, P2 = _params(rng, L, cin, cmid, cout)
    h = rng.standard_normal((v.shape[0], cin))
    ep2 = (rng.uniform(0.5, 1.5, cout), rng.normal(0, 1, cout), True)
    # every facet feature cut off: the output is act2(b2) everywhere
    o = v2v.v2v_sep(v, f, L, h, a1, P1, (None, np.full(cmid, -1e6), True), a2, P2, ep2)
    np.testing.assert_allclose(o, np.broadcast_to(np.maximum(ep2[1], 0), o.shape), atol=0)
    # the isolated vertex has no facets: z = 0 there whatever the features
    o, g, z = v2v.v2v_sep(v, f, L, h, a1, P1, None, a2, P2, ep2, parts=True)
    assert np.all(z[-1] == 0)
    np.testing.assert_allclose(o[-1], np.maximum(ep2[1], 0), atol=0)
    # no facets at all
    o = v2v.v2v_sep(v, f[:0], L, h, a1, P1, None, a2, P2, ep2)
    np.testing.assert_allclose(o, np.broadcast_to(np.maximum(ep2[1], 0), o.shape), atol=0)


@pytest.mark.parametrize("L,norm,relu", [(2, 0, True), (3, 1, False), (1, 0, True)])
def test_gradients_against_central_differences(L, norm, relu):
    rng = np.random.default_rng(20 + L)
    v, f = _mesh(4)
    cin, cmid, cout = 4, 5, 3
    a1, P1, a2, P2 = _params(rng, L, cin, cmid, cout)
    ep1, ep2 = _eps(rng, cmid, cout, relu, relu)
    h = rng.standard_normal((v.shape[0], cin))
    R = rng.standard_normal((v.shape[0], cout))
    args = dict(h=h, alpha1=a1, P1=P1, alpha2=a2, P2=P2)

    def loss(**kw):
        a = dict(args); a.update(kw)
        return float((v2v.v2v_sep(v, f, L, a["h"], a["alpha1"], a["P1"], ep1, a["alpha2"], a["P2"], ep2, norm) * R).sum())

    grads = dict(zip(["h", "alpha1", "P1", "alpha2", "P2"], v2v.v2v_sep_bwd(v, f, L, h, a1, P1, ep1, a2, P2, ep2, R, norm)))
    eps = 1e-6
    for name, gvals in grads.items():
        assert gvals.shape == args[name].shape
        for _ in range(3):
            d = rng.standard_normal(args[name].shape)
            fd = (loss(**{name: args[name] + eps * d}) - loss(**{name: args[name] - eps * d})) / (2 * eps)
            an = float((gvals * d).sum())
            assert abs(fd - an) <= 1e-6 * max(1.0, abs(an)), (name, fd, an)

"""Pins of the point-cloud convolution oracle (radial extension of the SH filter)."""
import numpy as np
import pytest

import oracle
from oracle import pcloud as opc
from paper_2112_01801_amd import meshgen as mg


def _setup(seed, M=40, N=60, L=2, cin=5, cout=4, rho=0.9):
    rng = np.random.default_rng(seed)
    xs = rng.uniform(-1, 1, (N, 3))
    xq = rng.uniform(-1, 1, (M, 3))
    ptr, idx = mg.range_neighbors(xq, xs, rho)
    K = (L + 1) ** 2
    return dict(xq=xq, xs=xs, ptr=ptr, idx=idx, rho=rho, L=L, h=rng.standard_normal((N, cin)),
                alpha=rng.standard_normal((K, cin)), c0=rng.standard_normal(cin), P=rng.standard_normal((cin, cout)),
                dg=rng.standard_normal((M, cout)), rng=rng)


def _conv(d, **over):
    a = {**d, **over}
    return opc.pcloud_conv(a["xq"], a["xs"], a["ptr"], a["idx"], a["rho"], a["L"], a["h"], a["alpha"], a["c0"], a["P"])


def test_on_the_sphere_of_radius_rho_it_is_the_angular_filter_alone():
    """F(theta, phi, rho) = F(theta, phi): neighbours at distance rho reduce the operator to the segment mean of
    the dense SH convolution, which the separately pinned facet2facet oracle computes (W = alpha (x) P)."""
    rng = np.random.default_rng(0)
    b = mg.pack_batch([mg.icosphere(1)])
    tex_off, bary = mg.texture_layout(b, 3, 1)
    n_tex, F, L, cin, cout, rho = int(tex_off[-1]), b.n_facet, 3, 6, 5, 0.37
    K = (L + 1) ** 2
    alpha, P = rng.standard_normal((K, cin)), rng.standard_normal((cin, cout))
    h = rng.standard_normal((n_tex, cin))
    xq = rng.standard_normal((F, 3))
    owner = np.repeat(np.arange(F), np.diff(tex_off))
    d = bary.astype(np.float64) / np.linalg.norm(bary.astype(np.float64), axis=1, keepdims=True)
    xs = xq[owner] + rho * d
    got = opc.pcloud_conv(xq, xs, tex_off, np.arange(n_tex), rho, L, h, alpha, rng.standard_normal(cin), P)
    ref = oracle.f2f(tex_off, bary, L, h, alpha[:, :, None] * P[None, :, :])
    assert np.allclose(got, ref, rtol=1e-9, atol=1e-11)


def test_at_the_centre_only_c0_remains_and_halfway_it_is_the_even_mix():
    d = _setup(1)
    N, cin = d["h"].shape
    ptr, idx = np.arange(N + 1), np.arange(N)                   # every point its own single neighbour, r = 0
    got = opc.pcloud_conv(d["xs"], d["xs"], ptr, idx, d["rho"], d["L"], d["h"], d["alpha"], d["c0"], d["P"])
    assert np.allclose(got, (d["h"] * d["c0"][None, :]) @ d["P"], rtol=1e-13)
    # one neighbour at rho/2 along +z: B_k(0,0,1) is known in closed form for l <= 1 (Eq. 3-4: constant and cos(theta))
    xq, xs = np.zeros((1, 3)), np.array([[0, 0, 0.5 * d["rho"]]])
    h1 = d["h"][:1]
    B = oracle.sh_basis(np.array([[0.0, 0.0, 1.0]]), 1)[0]
    assert np.allclose(B[[1, 3]], 0)                            # the m != 0 functions vanish at the pole
    a1 = d["alpha"][:4]
    got = opc.pcloud_conv(xq, xs, [0, 1], [0], d["rho"], 1, h1, a1, d["c0"], d["P"])
    ref = ((0.5 * (B[0] * a1[0] + B[2] * a1[2]) + 0.5 * d["c0"]) * h1[0]) @ d["P"]
    assert np.allclose(got[0], ref, rtol=1e-13)


def test_brute_force_loops_and_the_mean_over_neighbours():
    d = _setup(2, M=12, N=15, L=2, cin=3, cout=2)
    got = _conv(d)
    ref = np.zeros_like(got)
    for i in range(12):
        e0, e1 = d["ptr"][i], d["ptr"][i + 1]
        acc = np.zeros(3)
        for e in range(e0, e1):
            q = d["idx"][e]
            delta = d["xs"][q] - d["xq"][i]
            r = np.sqrt((delta ** 2).sum())
            Z = r / d["rho"]
            B = oracle.sh_basis(delta[None, :], 2)[0]
            for c in range(3):
                F = sum(d["alpha"][k, c] * B[k] for k in range(9))
                acc[c] += (F * Z + d["c0"][c] * (1 - Z)) * d["h"][q, c]
        if e1 > e0:
            acc /= (e1 - e0)
        ref[i] = acc @ d["P"]
    assert np.allclose(got, ref, rtol=1e-12, atol=1e-13)
    assert (np.diff(d["ptr"]) > 1).any()


def test_backward_adjoint_identities_and_finite_differences():
    d = _setup(3)
    dh, dalpha, dc0, dP = opc.pcloud_conv_bwd(d["xq"], d["xs"], d["ptr"], d["idx"], d["rho"], d["L"], d["h"], d["alpha"],
                                              d["c0"], d["P"], d["dg"])
    rng = d["rng"]
    # linear in h, in (alpha, c0) jointly, and in P: <conv(x'), dg> = <x', dx>
    h2 = rng.standard_normal(d["h"].shape)
    assert np.isclose((_conv(d, h=h2) * d["dg"]).sum(), (h2 * dh).sum(), rtol=1e-11)
    a2, c2 = rng.standard_normal(d["alpha"].shape), rng.standard_normal(d["c0"].shape)
    assert np.isclose((_conv(d, alpha=a2, c0=c2) * d["dg"]).sum(), (a2 * dalpha).sum() + (c2 * dc0).sum(), rtol=1e-11)
    P2 = rng.standard_normal(d["P"].shape)
    assert np.isclose((_conv(d, P=P2) * d["dg"]).sum(), (P2 * dP).sum(), rtol=1e-11)
    # and one finite difference per parameter block
    eps = 1e-6
    for name, grad in (("h", dh), ("alpha", dalpha), ("c0", dc0), ("P", dP)):
        x = d[name]
        i = tuple(rng.integers(0, n) for n in x.shape)
        xp, xm = x.copy(), x.copy()
        xp[i] += eps
        xm[i] -= eps
        fd = ((_conv(d, **{name: xp}) - _conv(d, **{name: xm})) * d["dg"]).sum() / (2 * eps)
        assert np.isclose(fd, grad[i], rtol=1e-6, atol=1e-9), name


def test_query_without_neighbours_and_radius_clamp():
    d = _setup(4, M=5, N=8)
    ptr = np.array([0, 0, 2, 2, 3, 3])
    idx = np.array([1, 4, 7])
    got = opc.pcloud_conv(d["xq"], d["xs"], ptr, idx, d["rho"], d["L"], d["h"], d["alpha"], d["c0"], d["P"])
    assert not got[[0, 2, 4]].any() and got[[1, 3]].any()
    # a neighbour farther than rho counts as lying on the sphere (Z clamps at 1)
    xq, xs = np.zeros((1, 3)), np.array([[0.3, -0.2, 0.5]])
    far = opc.pcloud_conv(xq, 10 * xs, [0, 1], [0], 1.0, d["L"], d["h"][:1], d["alpha"], d["c0"], d["P"])
    on = opc.pcloud_conv(xq, xs / np.linalg.norm(xs), [0, 1], [0], 1.0, d["L"], d["h"][:1], d["alpha"], d["c0"], d["P"])
    assert np.allclose(far, on, rtol=1e-12)

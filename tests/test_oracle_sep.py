"""Pins of the oracle's depth-wise separable facet2vertex / vertex2facet (CPU only).

The separable form (per-channel SH coefficients alpha[k,ci], then a point-wise matrix P[ci,co]) is the
dense form with W[k,ci,co] = alpha[k,ci] P[ci,co].  The oracle evaluates it by its own staged loops, so
equality with the (independently pinned) dense functions on the expanded coefficients is a real check;
the chain rule gives dalpha and dP from the dense dW.  Finite differences, adjoint identities and two
closed forms pin the rest.
"""
import numpy as np
import pytest

import oracle
from paper_2112_01801_amd import meshgen as mg


def _mesh(seed=0):
    rng = np.random.default_rng(seed)
    v, f = mg.icosphere_f64(2)
    v = v * (1 + rng.normal(0, 0.05, (v.shape[0], 1)))
    v = np.concatenate([v, [[3.0, 3.0, 3.0]]], 0)            # one isolated vertex
    return v.astype(np.float32), f.astype(np.int32)


def _params(rng, L, cin, cout):
    K = (L + 1) ** 2
    return rng.standard_normal((K, cin)), rng.standard_normal((cin, cout))


@pytest.mark.parametrize("L,cin,cout,norm", [(3, 5, 7, 0), (2, 8, 3, 1), (0, 4, 4, 0)])
def test_separable_equals_dense_on_expanded_coefficients(L, cin, cout, norm):
    rng = np.random.default_rng(10 + L)
    v, f = _mesh(1)
    alpha, P = _params(rng, L, cin, cout)
    W = alpha[:, :, None] * P[None, :, :]
    hF, hV = rng.standard_normal((f.shape[0], cin)), rng.standard_normal((v.shape[0], cin))
    dgV, dgF = rng.standard_normal((v.shape[0], cout)), rng.standard_normal((f.shape[0], cout))
    # facet2vertex
    np.testing.assert_allclose(oracle.f2v_sep(v, f, L, hF, alpha, P, norm), oracle.f2v(v, f, L, hF, W, norm),
                               rtol=1e-11, atol=1e-12)
    dh, da, dP = oracle.f2v_sep_bwd(v, f, L, hF, alpha, P, dgV, norm)
    rdh, rdW = oracle.f2v_bwd(v, f, L, hF, W, dgV, norm)
    np.testing.assert_allclose(dh, rdh, rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(da, np.einsum("kio,io->ki", rdW, P), rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(dP, np.einsum("kio,ki->io", rdW, alpha), rtol=1e-10, atol=1e-10)
    # vertex2facet
    np.testing.assert_allclose(oracle.v2f_sep(v.shape[0], f, L, hV, alpha, P, norm),
                               oracle.v2f(v.shape[0], f, L, hV, W, norm), rtol=1e-11, atol=1e-12)
    dh, da, dP = oracle.v2f_sep_bwd(v.shape[0], f, L, hV, alpha, P, dgF, norm)
    rdh, rdW = oracle.v2f_bwd(v.shape[0], f, L, hV, W, dgF, norm)
    np.testing.assert_allclose(dh, rdh, rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(da, np.einsum("kio,io->ki", rdW, P), rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(dP, np.einsum("kio,ki->io", rdW, alpha), rtol=1e-10, atol=1e-10)


def test_separable_rows_subset_and_isolated_vertex():
    rng = np.random.default_rng(3)
    v, f = _mesh(2)
    L, cin, cout = 2, 6, 5
    alpha, P = _params(rng, L, cin, cout)
    h = rng.standard_normal((f.shape[0], cin))
    full = oracle.f2v_sep(v, f, L, h, alpha, P)
    rows = np.array([0, 7, v.shape[0] - 1, 3])
    np.testing.assert_array_equal(oracle.f2v_sep(v, f, L, h, alpha, P, rows=rows), full[rows])
    assert np.all(full[-1] == 0)                               # the isolated vertex
    dg = rng.standard_normal((v.shape[0], cout))
    dh, _, _ = oracle.f2v_sep_bwd(v, f, L, h, alpha, P, dg)
    fr = np.array([5, 0, f.shape[0] - 1])
    dhs, da, dP = oracle.f2v_sep_bwd(v, f, L, h, alpha, P, dg, rows=fr, want_dw=False)
    np.testing.assert_array_equal(dhs, dh[fr])
    assert da is None and dP is None


def test_separable_closed_forms():
    """Degree 0: the filter is the constant alpha[0,ci]/(2 sqrt(pi)), so F2V is a scaled adjacency average and
    V2F a scaled corner sum; with P = identity the channels do not mix."""
    rng = np.random.default_rng(4)
    v, f = _mesh(3)
    cin = 4
    alpha = rng.standard_normal((1, cin))
    P = np.eye(cin)
    hF, hV = rng.standard_normal((f.shape[0], cin)), rng.standard_normal((v.shape[0], cin))
    c = alpha[0] / (2 * np.sqrt(np.pi))
    g = oracle.f2v_sep(v, f, 0, hF, alpha, P)
    ref = np.zeros((v.shape[0], cin))
    deg = np.zeros(v.shape[0])
    for fi, tri in enumerate(f):
        for vid in tri:
            ref[vid] += hF[fi]
            deg[vid] += 1
    ref = ref / np.maximum(deg, 1)[:, None] * c
    np.testing.assert_allclose(g, ref, rtol=1e-12, atol=1e-13)
    g = oracle.v2f_sep(v.shape[0], f, 0, hV, alpha, P)
    np.testing.assert_allclose(g, (hV[f[:, 0]] + hV[f[:, 1]] + hV[f[:, 2]]) * c, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("op", ["f2v", "v2f"])
def test_separable_backward_finite_differences_and_adjoint(op):
    rng = np.random.default_rng(5)
    v, f = _mesh(4)
    L, cin, cout = 3, 3, 4
    alpha, P = _params(rng, L, cin, cout)
    nV, nF = v.shape[0], f.shape[0]
    if op == "f2v":
        h, dg = rng.standard_normal((nF, cin)), rng.standard_normal((nV, cout))
        fwd = lambda h_, a_, P_: oracle.f2v_sep(v, f, L, h_, a_, P_)
        dh, da, dP = oracle.f2v_sep_bwd(v, f, L, h, alpha, P, dg)
    else:
        h, dg = rng.standard_normal((nV, cin)), rng.standard_normal((nF, cout))
        fwd = lambda h_, a_, P_: oracle.v2f_sep(nV, f, L, h_, a_, P_)
        dh, da, dP = oracle.v2f_sep_bwd(nV, f, L, h, alpha, P, dg)
    loss = lambda h_, a_, P_: float((fwd(h_, a_, P_) * dg).sum())
    eps = 1e-6
    for arr, grad, which in ((alpha, da, 1), (P, dP, 2), (h, dh, 0)):
        for _ in range(6):
            idx = tuple(rng.integers(0, s) for s in arr.shape)
            d = np.zeros_like(arr)
            d[idx] = eps
            args_p = [h, alpha, P]
            args_m = [h, alpha, P]
            args_p[which] = arr + d
            args_m[which] = arr - d
            fd = (loss(*args_p) - loss(*args_m)) / (2 * eps)
            assert abs(fd - grad[idx]) <= 1e-6 * max(1.0, abs(fd)), (op, which, idx, fd, grad[idx])
    # bilinearity in (h, P): <g, dg> = <h, dh> = <P, dP>;  linear in alpha: = <alpha, dalpha>
    g = fwd(h, alpha, P)
    s = float((g * dg).sum())
    for a, b in ((h, dh), (P, dP), (alpha, da)):
        assert abs(float((a * b).sum()) - s) <= 1e-9 * max(1.0, abs(s))

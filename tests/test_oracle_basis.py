"""Pins for the oracle's SH basis (Eq. 3-4): none of these re-use the oracle's own recurrences."""
import math
import os

import numpy as np
import pytest
from scipy.special import sph_harm_y

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "sh_closed_forms.txt")


def unit_dirs(n, seed=0):
    rng = np.random.default_rng(seed)
    d = rng.standard_normal((n, 3))
    return d / np.linalg.norm(d, axis=1, keepdims=True)


def kidx(l, m):
    return l * (l + 1) + m


def test_closed_forms_from_golden_table():
    """Signs and scales of every l <= 3 function against hand-derived Cartesian closed forms."""
    d = unit_dirs(200, 1)
    x, y, z = d[:, 0], d[:, 1], d[:, 2]
    B = oracle.sh_basis(d, 3)
    seen = 0
    env = {"sqrt": math.sqrt, "pi": math.pi}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        l, m, coef, poly = line.split(None, 3)
        l, m = int(l), int(m)
        ref = eval(coef, env) * eval(poly, {"x": x, "y": y, "z": z}) * np.ones_like(x)
        np.testing.assert_allclose(B[:, kidx(l, m)], ref, rtol=0, atol=2e-14, err_msg="l=%d m=%d" % (l, m))
        seen += 1
    assert seen == 16


@pytest.mark.parametrize("L", [0, 1, 2, 3, 4, 5])
def test_gram_matrix_by_exact_quadrature(L):
    """Gauss-Legendre in cos(theta) x uniform phi integrates degree-2L products exactly.

    Eq. 4's functions as printed are orthogonal with squared norm 1 (m = 0) and 1/2 (m != 0);
    the sqrt(2)-rescaled variant is orthonormal (the abstract's wording).
    """
    nt, nphi = L + 2, 2 * L + 3
    t, wt = np.polynomial.legendre.leggauss(nt)
    phi = 2 * np.pi * np.arange(nphi) / nphi
    T, PH = np.meshgrid(t, phi, indexing="ij")
    s = np.sqrt(1 - T ** 2)
    d = np.stack([s * np.cos(PH), s * np.sin(PH), T], -1).reshape(-1, 3)
    w = (wt[:, None] * np.full((1, nphi), 2 * np.pi / nphi)).ravel()
    K = (L + 1) ** 2
    expect = np.ones(K)
    for l in range(L + 1):
        for m in range(-l, l + 1):
            if m != 0:
                expect[kidx(l, m)] = 0.5
    B = oracle.sh_basis(d, L, norm=0)
    G = (B * w[:, None]).T @ B
    np.testing.assert_allclose(G, np.diag(expect), rtol=0, atol=1e-13)
    Bo = oracle.sh_basis(d, L, norm=1)
    Go = (Bo * w[:, None]).T @ Bo
    np.testing.assert_allclose(Go, np.eye(K), rtol=0, atol=1e-13)


@pytest.mark.parametrize("L", [3, 5])
def test_against_library_complex_sh(L):
    """scipy's Y_l^m carries the Condon-Shortley phase (-1)^m; Eq. 3 does not."""
    d = unit_dirs(64, 2)
    theta = np.arccos(d[:, 2])
    phi = np.arctan2(d[:, 1], d[:, 0])
    B = oracle.sh_basis(d, L)
    for l in range(L + 1):
        for m in range(0, l + 1):
            Y = sph_harm_y(l, m, theta, phi) * (-1.0) ** m
            np.testing.assert_allclose(B[:, kidx(l, m)], Y.real, atol=1e-13, rtol=0)
            if m > 0:
                np.testing.assert_allclose(B[:, kidx(l, -m)], Y.imag, atol=1e-13, rtol=0)


@pytest.mark.parametrize("L", [1, 4, 5])
def test_addition_theorem(L):
    d = unit_dirs(100, 3)
    B = oracle.sh_basis(d, L)
    for l in range(L + 1):
        s = B[:, kidx(l, 0)] ** 2
        for m in range(1, l + 1):
            s = s + 2 * (B[:, kidx(l, m)] ** 2 + B[:, kidx(l, -m)] ** 2)
        np.testing.assert_allclose(s, (2 * l + 1) / (4 * np.pi), rtol=1e-13)


def _dfact(n):
    return 1.0 if n <= 0 else float(n) * _dfact(n - 2)


def test_pole_and_equator_values():
    """The three vertex2facet corner directions of Eq. 6: (pi/2,0), (pi/2,pi/2), (0,0)."""
    L = 5
    B = oracle.sh_basis(np.array([[1.0, 0, 0], [0, 1.0, 0], [0, 0, 1.0]]), L)
    for l in range(L + 1):
        for m in range(-l, l + 1):
            pole = math.sqrt((2 * l + 1) / (4 * math.pi)) if m == 0 else 0.0
            assert abs(B[2, kidx(l, m)] - pole) < 1e-14
            am = abs(m)
            if (l + am) % 2 == 1:
                p0 = 0.0
            else:  # P_l^m(0) without the Condon-Shortley phase
                p0 = (-1.0) ** ((l - am) // 2) * _dfact(l + am - 1) / _dfact(l - am)
            N = math.sqrt((2 * l + 1) / (4 * math.pi) * math.factorial(l - am) / math.factorial(l + am))
            ex = N * p0 * (1.0 if m >= 0 else 0.0)                      # phi = 0
            ey = N * p0 * (math.cos(am * math.pi / 2) if m >= 0 else math.sin(am * math.pi / 2))
            assert abs(B[0, kidx(l, m)] - ex) < 1e-13, (l, m)
            assert abs(B[1, kidx(l, m)] - ey) < 1e-13, (l, m)


def test_rotation_about_z_mixes_cos_sin_pairs():
    L, psi = 4, 0.37
    d = unit_dirs(50, 4)
    R = np.array([[math.cos(psi), -math.sin(psi), 0], [math.sin(psi), math.cos(psi), 0], [0, 0, 1]])
    B0 = oracle.sh_basis(d, L)
    B1 = oracle.sh_basis(d @ R.T, L)
    for l in range(L + 1):
        np.testing.assert_allclose(B1[:, kidx(l, 0)], B0[:, kidx(l, 0)], atol=1e-13)
        for m in range(1, l + 1):
            c, s = math.cos(m * psi), math.sin(m * psi)
            np.testing.assert_allclose(B1[:, kidx(l, m)], c * B0[:, kidx(l, m)] - s * B0[:, kidx(l, -m)], atol=1e-13)
            np.testing.assert_allclose(B1[:, kidx(l, -m)], s * B0[:, kidx(l, m)] + c * B0[:, kidx(l, -m)], atol=1e-13)


def test_direction_length_is_irrelevant_and_parity():
    d = unit_dirs(20, 5)
    B = oracle.sh_basis(d, 5)
    np.testing.assert_allclose(oracle.sh_basis(7.5 * d, 5), B, atol=1e-13)
    Bm = oracle.sh_basis(-d, 5)
    for l in range(6):
        for m in range(-l, l + 1):
            np.testing.assert_allclose(Bm[:, kidx(l, m)], (-1.0) ** l * B[:, kidx(l, m)], atol=1e-13)


def test_basis_gradient_against_closed_forms():
    """d/dd of B(d/|d|) for l <= 2, from the closed forms of the golden table."""
    rng = np.random.default_rng(6)
    d = rng.standard_normal((40, 3)) * rng.uniform(0.5, 2.0, (40, 1))
    r = np.linalg.norm(d, axis=1)
    u = d / r[:, None]
    K = 9
    for k, (coef, f, grad_u) in {
        kidx(1, 0): (math.sqrt(3 / (4 * math.pi)), None, lambda u: np.stack([0 * u[:, 0], 0 * u[:, 0], 1 + 0 * u[:, 0]], 1)),
        kidx(1, 1): (math.sqrt(3 / (8 * math.pi)), None, lambda u: np.stack([1 + 0 * u[:, 0], 0 * u[:, 0], 0 * u[:, 0]], 1)),
        kidx(2, 0): (math.sqrt(5 / (16 * math.pi)), None, lambda u: np.stack([0 * u[:, 0], 0 * u[:, 0], 6 * u[:, 2]], 1)),
        kidx(2, -2): (math.sqrt(15 / (32 * math.pi)), None, lambda u: np.stack([2 * u[:, 1], 2 * u[:, 0], 0 * u[:, 0]], 1)),
        kidx(2, 1): (math.sqrt(15 / (8 * math.pi)), None, lambda u: np.stack([u[:, 2], 0 * u[:, 0], u[:, 0]], 1)),
    }.items():
        db = np.zeros((d.shape[0], K))
        db[:, k] = 1.0
        got = oracle.sh_basis_bwd(d, 2, db)
        gu = coef * grad_u(u)                               # gradient w.r.t. the unit vector
        # chain rule through u = d/|d|:  (I - u u^T)/|d|
        ref = (gu - u * np.einsum("ij,ij->i", gu, u)[:, None]) / r[:, None]
        np.testing.assert_allclose(got, ref, atol=1e-9)

"""fp64 CPU oracle of the point-cloud convolution with the radial term -- TEST INFRASTRUCTURE, not the product.

Subsection "Extension to Point Cloud Convolution": the filter of Eq. 4 gets a radial control,
    F(theta, phi, r) = F(theta, phi) Z(r) + c0 (1 - Z(r)),   Z(r) = r / rho,  r in [0, rho],
and the convolution is depth-wise separable like facet2vertex / vertex2facet.  Written out with this build's
readings (the paper prints no sum for it):
    delta_e = xs[q_e] - xq[i]  for the neighbours q_e of query point i (lists supplied by the caller),
    r_e = |delta_e|, Z_e = min(r_e / rho, 1), direction delta_e / r_e (any direction when r_e = 0: Z_e = 0 there),
    s_e[c]  = Z_e sum_k alpha[k, c] B_k(direction_e) + c0[c] (1 - Z_e)                 (K + 1 numbers per channel)
    y_i[c]  = 1/|N(i)| sum_{e in N(i)} s_e[c] h[q_e][c]      (mean over the neighbours, as in Eq. 5; 0 if none)
    g_i     = y_i P                                           (point-wise Cin x Cout matrix)
The SH basis comes from this package's pinned sh_basis.  Plain numpy over the pair list; nothing is shared
with the HIP path.  Parity status: pinned by tests/test_oracle_pcloud.py.
"""
from __future__ import annotations

import numpy as np

from . import sh_basis


def _pairs(xq, xs, nbr_ptr, nbr_idx, rho):
    xq, xs = np.asarray(xq, np.float64), np.asarray(xs, np.float64)
    ptr, idx = np.asarray(nbr_ptr, np.int64), np.asarray(nbr_idx, np.int64)
    deg = np.diff(ptr)
    owner = np.repeat(np.arange(deg.shape[0]), deg)
    delta = xs[idx] - xq[owner]
    r = np.linalg.norm(delta, axis=1)
    Z = np.minimum(r / rho, 1.0)
    d = np.where((r > 0)[:, None], delta / np.where(r > 0, r, 1.0)[:, None], np.array([0.0, 0.0, 1.0])[None, :])
    return owner, idx, deg, Z, d


def pair_filter(xq, xs, nbr_ptr, nbr_idx, rho, L, alpha, c0, norm: int = 0):
    """s_e[c] for every pair, plus what the gradients need."""
    owner, idx, deg, Z, d = _pairs(xq, xs, nbr_ptr, nbr_idx, rho)
    B = sh_basis(d, L, norm) if d.shape[0] else np.zeros((0, (L + 1) ** 2))
    s = Z[:, None] * (B @ np.asarray(alpha, np.float64)) + (1.0 - Z)[:, None] * np.asarray(c0, np.float64)[None, :]
    return s, B, Z, owner, idx, deg


def pcloud_conv(xq, xs, nbr_ptr, nbr_idx, rho, L, h, alpha, c0, P, norm: int = 0) -> np.ndarray:
    h, P = np.asarray(h, np.float64), np.asarray(P, np.float64)
    s, _, _, owner, idx, deg = pair_filter(xq, xs, nbr_ptr, nbr_idx, rho, L, alpha, c0, norm)
    y = np.zeros((deg.shape[0], h.shape[1]))
    np.add.at(y, owner, s * h[idx])
    y /= np.maximum(deg, 1)[:, None]
    return y @ P


def pcloud_conv_bwd(xq, xs, nbr_ptr, nbr_idx, rho, L, h, alpha, c0, P, dg, norm: int = 0):
    """(dh [N, Cin], dalpha [K, Cin], dc0 [Cin], dP [Cin, Cout])."""
    h, P, dg = np.asarray(h, np.float64), np.asarray(P, np.float64), np.asarray(dg, np.float64)
    s, B, Z, owner, idx, deg = pair_filter(xq, xs, nbr_ptr, nbr_idx, rho, L, alpha, c0, norm)
    w = 1.0 / np.maximum(deg, 1)
    y = np.zeros((deg.shape[0], h.shape[1]))
    np.add.at(y, owner, s * h[idx])
    y *= w[:, None]
    dP = y.T @ dg
    dy = (dg @ P.T) * w[:, None]
    dh = np.zeros_like(h)
    np.add.at(dh, idx, s * dy[owner])
    p = h[idx] * dy[owner]
    dalpha = (Z[:, None] * B).T @ p
    dc0 = ((1.0 - Z)[:, None] * p).sum(axis=0)
    return dh, dalpha, dc0, dP

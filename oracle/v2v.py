"""fp64 CPU oracle of the separable vertex2vertex block -- TEST INFRASTRUCTURE, not the product.

Subsection "Angular Arguments in Different Convolutions" (last paragraph on vertex2facet) and the figure of the
four mesh convolutions: vertex2vertex is a vertex2facet convolution (Eq. 6) followed by a facet2vertex
convolution (Eq. 5), both depth-wise separable, with batch normalisation on the facet and on the vertex
features and ReLU as the activation.  Written out with this build's readings:
    s1_j[c]  = sum_k alpha1[k, c] B_k(e_j),  e_j the j-th barycentric unit vector        (three constant filters)
    u_f      = (sum_j s1_j * h[v_j(f)]) P1                                               (Eq. 6, then point-wise)
    g_f      = act1(a1 * u_f + b1)                   (normalisation with fixed statistics = per-channel affine)
    y_f[c]   = g_f[c] sum_k alpha2[k, c] B_k(n_f)                                        (Eq. 5, depth-wise)
    z_v      = 1/|N(v)| sum_{f in N(v)} y_f           (0 for a vertex without facets)
    o_v      = act2(a2 * (z_v P2) + b2)
act = ReLU or identity; a = 1, b = 0 when no affine is given.  The backward functions differentiate this with the
affine maps held fixed (frozen statistics); the activation's derivative is taken as [output > 0].
Uses this package's pinned sh_basis and facet_normals; everything else is plain numpy.  Nothing is shared with
the HIP path.  Parity status: pinned by tests/test_oracle_v2v.py (composition of the separately pinned
separable oracles, brute force on a tiny mesh for the constant filter, central differences for every gradient).
"""
from __future__ import annotations

import numpy as np

from . import facet_normals, sh_basis


def _ep(ep, C):
    """(scale [C], shift [C], relu) from None or a (scale | None, shift | None, relu) triple."""
    if ep is None:
        return np.ones(C), np.zeros(C), False
    a, b, relu = ep
    a = np.ones(C) if a is None else np.asarray(a, np.float64)
    b = np.zeros(C) if b is None else np.asarray(b, np.float64)
    return a, b, bool(relu)


def _act(x, relu):
    return np.maximum(x, 0.0) if relu else x


def _stages(vert, facet, L, h, alpha1, P1, ep1, alpha2, P2, ep2, norm):
    facet = np.asarray(facet, np.int64).reshape(-1, 3)
    h = np.asarray(h, np.float64)
    alpha1, P1 = np.asarray(alpha1, np.float64), np.asarray(P1, np.float64)
    alpha2, P2 = np.asarray(alpha2, np.float64), np.asarray(P2, np.float64)
    V, F = h.shape[0], facet.shape[0]
    K = (L + 1) ** 2
    s1 = sh_basis(np.eye(3), L, norm) @ alpha1                       # [3, cin]
    t = np.zeros((F, h.shape[1]))
    for j in range(3):
        t += s1[j][None, :] * h[facet[:, j]]
    a1, b1, r1 = _ep(ep1, P1.shape[1])
    g = _act(a1 * (t @ P1) + b1, r1)
    Bn = sh_basis(facet_normals(vert, facet), L, norm) if F else np.zeros((0, K))
    S2 = Bn @ alpha2                                                 # [F, cmid]
    deg = np.bincount(facet.reshape(-1), minlength=V).astype(np.float64)
    w = 1.0 / np.maximum(deg, 1.0)
    z = np.zeros((V, P1.shape[1]))
    for j in range(3):
        np.add.at(z, facet[:, j], S2 * g)
    z *= w[:, None]
    a2, b2, r2 = _ep(ep2, P2.shape[1])
    o = _act(a2 * (z @ P2) + b2, r2)
    return dict(facet=facet, h=h, s1=s1, t=t, g=g, Bn=Bn, S2=S2, w=w, z=z, o=o, a1=a1, a2=a2, r1=r1, r2=r2,
                alpha1=alpha1, P1=P1, alpha2=alpha2, P2=P2)


def v2v_sep(vert, facet, L, h, alpha1, P1, ep1, alpha2, P2, ep2, norm: int = 0, parts: bool = False):
    """o [V, Cout]; with parts=True also the facet features g [F, Cmid] and the vertex means z [V, Cmid]."""
    s = _stages(vert, facet, L, h, alpha1, P1, ep1, alpha2, P2, ep2, norm)
    return (s["o"], s["g"], s["z"]) if parts else s["o"]


def v2v_sep_bwd(vert, facet, L, h, alpha1, P1, ep1, alpha2, P2, ep2, d_out, norm: int = 0):
    """(dh [V, Cin], dalpha1 [K, Cin], dP1 [Cin, Cmid], dalpha2 [K, Cmid], dP2 [Cmid, Cout])."""
    s = _stages(vert, facet, L, h, alpha1, P1, ep1, alpha2, P2, ep2, norm)
    facet, hh = s["facet"], s["h"]
    d_out = np.asarray(d_out, np.float64)
    dq = d_out * s["a2"][None, :]                                    # gradient at z P2
    if s["r2"]:
        dq = dq * (s["o"] > 0)
    dP2 = s["z"].T @ dq
    dz = (dq @ s["P2"].T) * s["w"][:, None]                          # the mean's weight, per vertex
    dy = np.zeros_like(s["g"])
    for j in range(3):
        dy += dz[facet[:, j]]
    dalpha2 = s["Bn"].T @ (s["g"] * dy)
    dg = s["S2"] * dy
    du = dg * s["a1"][None, :]
    if s["r1"]:
        du = du * (s["g"] > 0)
    dP1 = s["t"].T @ du
    dt = du @ s["P1"].T
    Be = sh_basis(np.eye(3), L, norm)                                # [3, K]
    dh = np.zeros_like(hh)
    dalpha1 = np.zeros_like(s["alpha1"])
    for j in range(3):
        np.add.at(dh, facet[:, j], s["s1"][j][None, :] * dt)
        dalpha1 += np.outer(Be[j], (hh[facet[:, j]] * dt).sum(axis=0))
    return dh, dalpha1, dP1, dalpha2, dP2

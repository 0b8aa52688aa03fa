"""Pins for the oracle's convolutions (Eq. 5-7) and their backward passes.

Each test compares the oracle with something that is not the oracle: a closed form on a regular
solid, a brute-force O(V*F) scan, a sparse-matrix routine, finite differences, an adjoint
identity, or an invariance the paper states.
"""
import math

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from paper_2112_01801_amd import meshgen as mg


def kidx(l, m):
    return l * (l + 1) + m


def rand_inputs(seed, nrow_in, K, cin, cout):
    rng = np.random.default_rng(seed)
    h = rng.standard_normal((nrow_in, cin))
    W = rng.uniform(-1, 1, (K, cin, cout))
    return rng, h, W


def rotation(seed):
    rng = np.random.default_rng(seed)
    q, r = np.linalg.qr(rng.standard_normal((3, 3)))
    q = q * np.sign(np.diag(r))
    if np.linalg.det(q) < 0:
        q[:, 0] = -q[:, 0]
    return q


# ------------------------------------------------------------------ adjacency / normals
def test_adjacency_brute_force():
    v, f = mg.icosphere(1)
    V = v.shape[0]
    rp, col = oracle.vf_adjacency(V, f)
    assert rp[0] == 0 and rp[V] == 3 * f.shape[0]
    assert sorted(col.tolist()) == list(range(3 * f.shape[0]))
    for vv in range(V):
        brute = [3 * ff + j for ff in range(f.shape[0]) for j in range(3) if f[ff, j] == vv]
        assert col[rp[vv]:rp[vv + 1]].tolist() == brute


def test_normals_of_regular_solids():
    v, f = mg.tetrahedron()
    n = oracle.facet_normals(v, f)
    c = v[f].mean(axis=1)
    np.testing.assert_allclose(n, c / np.linalg.norm(c, axis=1, keepdims=True), atol=1e-6)
    np.testing.assert_allclose(np.abs(n), 1 / math.sqrt(3), atol=1e-6)
    v, f = mg.icosahedron()
    n = oracle.facet_normals(v, f)
    c = v[f].mean(axis=1)
    np.testing.assert_allclose(n, c / np.linalg.norm(c, axis=1, keepdims=True), atol=1e-6)


def test_degenerate_facet_normal_rule():
    v = np.array([[0, 0, 0], [1, 0, 0], [2, 0, 0], [0, 1, 0]], dtype=np.float32)
    f = np.array([[0, 1, 2], [0, 1, 3]], dtype=np.int32)
    n = oracle.facet_normals(v, f)
    np.testing.assert_array_equal(n, [[0, 0, 1], [0, 0, 1]])


# ------------------------------------------------------------------ facet2vertex
def test_f2v_tetrahedron_closed_form():
    """h == 1, L = 1: mean of the three adjacent outward normals of a regular tetrahedron is v_hat/3."""
    v, f = mg.tetrahedron()
    rng = np.random.default_rng(0)
    W = rng.uniform(-1, 1, (4, 1, 3))
    g = oracle.f2v(v, f, 1, np.ones((4, 1)), W)
    vh = v / np.linalg.norm(v, axis=1, keepdims=True)
    c0, c10, c11 = math.sqrt(1 / (4 * math.pi)), math.sqrt(3 / (4 * math.pi)), math.sqrt(3 / (8 * math.pi))
    ref = (c0 * W[0, 0][None, :]
           + (c10 * vh[:, 2:3] * W[kidx(1, 0), 0][None, :]
              + c11 * vh[:, 0:1] * W[kidx(1, 1), 0][None, :]
              + c11 * vh[:, 1:2] * W[kidx(1, -1), 0][None, :]) / 3.0)
    np.testing.assert_allclose(g, ref, atol=1e-7)   # vertices are float32


def test_f2v_icosahedron_closed_form():
    """Mean of the 5 adjacent unit normals at a vertex of a regular icosahedron = rho * v_hat."""
    v, f = mg.icosahedron()
    rho = math.sqrt((5 + 2 * math.sqrt(5)) / 15)
    rng = np.random.default_rng(1)
    W = rng.uniform(-1, 1, (4, 1, 2))
    g = oracle.f2v(v, f, 1, np.ones((20, 1)), W)
    vh = v / np.linalg.norm(v, axis=1, keepdims=True)
    c0, c10, c11 = math.sqrt(1 / (4 * math.pi)), math.sqrt(3 / (4 * math.pi)), math.sqrt(3 / (8 * math.pi))
    ref = (c0 * W[0, 0][None, :] + rho * (c10 * vh[:, 2:3] * W[2, 0][None, :] + c11 * vh[:, 0:1] * W[3, 0][None, :]
                                          + c11 * vh[:, 1:2] * W[1, 0][None, :]))
    np.testing.assert_allclose(g, ref, atol=1e-6)


def test_symmetry_sums_of_basis_over_regular_solids():
    """sum_f B_lm(n_f) vanishes for l = 1, 2 (tetrahedron) and l = 1..5 (icosahedron)."""
    v, f = mg.tetrahedron()
    B = oracle.sh_basis(oracle.facet_normals(v, f), 2)
    np.testing.assert_allclose(B[:, 1:].sum(0), 0, atol=1e-6)
    v, f = mg.icosahedron()
    B = oracle.sh_basis(oracle.facet_normals(v, f), 5)
    np.testing.assert_allclose(B[:, 1:].sum(0), 0, atol=2e-6)


def test_f2v_degree0_is_sparse_averaging():
    """L = 0: the filter is the constant W[0]/(2 sqrt(pi)); F2V = D^-1 A^T H W0 / (2 sqrt(pi))."""
    v, f = mg.icosphere(2)
    V, F = v.shape[0], f.shape[0]
    rng, h, W = rand_inputs(2, F, 1, 5, 7)
    g = oracle.f2v(v, f, 0, h, W)
    A = sp.coo_matrix((np.ones(3 * F), (f.ravel(), np.repeat(np.arange(F), 3))), shape=(V, F)).tocsr()
    deg = np.asarray(A.sum(1)).ravel()
    ref = (A @ h) / deg[:, None] @ W[0] / (2 * math.sqrt(math.pi))
    np.testing.assert_allclose(g, ref, atol=1e-12)
    # and it does not depend on the orientation of the mesh
    g2 = oracle.f2v((v @ rotation(3).T).astype(np.float32), f, 0, h, W)
    np.testing.assert_allclose(g2, g, atol=1e-12)


def f2v_brute(v, f, L, h, W):
    """Independent evaluation: per-facet basis from the library SH, O(V*F) corner scan."""
    from scipy.special import sph_harm_y
    vv = v.astype(np.float64)
    n = np.cross(vv[f[:, 1]] - vv[f[:, 0]], vv[f[:, 2]] - vv[f[:, 0]])
    n /= np.linalg.norm(n, axis=1, keepdims=True)
    theta, phi = np.arccos(np.clip(n[:, 2], -1, 1)), np.arctan2(n[:, 1], n[:, 0])
    K = (L + 1) ** 2
    B = np.zeros((f.shape[0], K))
    for l in range(L + 1):
        for m in range(l + 1):
            Y = sph_harm_y(l, m, theta, phi) * (-1.0) ** m
            B[:, kidx(l, m)] = Y.real
            if m:
                B[:, kidx(l, -m)] = Y.imag
    y = np.einsum("fk,fi,kio->fo", B, h, W)
    g = np.zeros((v.shape[0], W.shape[2]))
    for vi in range(v.shape[0]):
        cnt = 0
        for ff in range(f.shape[0]):
            for j in range(3):
                if f[ff, j] == vi:
                    g[vi] += y[ff]
                    cnt += 1
        if cnt:
            g[vi] /= cnt
    return g, y


def test_f2v_brute_force_and_conservation():
    v, f = mg.icosphere(1)
    rng = np.random.default_rng(4)
    v = (v * (1 + rng.uniform(-0.1, 0.1, (v.shape[0], 1)))).astype(np.float32)
    _, h, W = rand_inputs(5, f.shape[0], 16, 3, 4)
    g = oracle.f2v(v, f, 3, h, W)
    gb, y = f2v_brute(v, f, 3, h, W)
    np.testing.assert_allclose(g, gb, atol=1e-12)
    deg = np.bincount(f.ravel(), minlength=v.shape[0])
    np.testing.assert_allclose((deg[:, None] * g).sum(0), 3 * y.sum(0), atol=1e-10)


def test_f2v_rows_subset_and_isolated_vertex():
    v, f = mg.icosphere(1)
    v = np.concatenate([v, [[5, 5, 5]]], 0).astype(np.float32)   # isolated vertex at the end
    _, h, W = rand_inputs(6, f.shape[0], 4, 2, 3)
    g = oracle.f2v(v, f, 1, h, W)
    assert np.all(g[-1] == 0)
    rows = np.array([5, 0, 41, 42])
    np.testing.assert_array_equal(oracle.f2v(v, f, 1, h, W, rows=rows), g[rows])


def test_f2v_invariances():
    """Translation and uniform scale leave F2V unchanged; a rotation changes it for L >= 1 (Sec. 4.2)."""
    v, f = mg.icosphere(1)
    _, h, W = rand_inputs(7, f.shape[0], 9, 2, 2)
    g = oracle.f2v(v, f, 2, h, W)
    g_t = oracle.f2v((v.astype(np.float64) * 2.0 + np.array([1.0, -2.0, 0.5])).astype(np.float32), f, 2, h, W)
    np.testing.assert_allclose(g_t, g, atol=1e-5)
    g_r = oracle.f2v((v @ rotation(8).T).astype(np.float32), f, 2, h, W)
    assert np.abs(g_r - g).max() > 1e-2


def test_f2v_z_rotation_with_rotated_coefficients():
    """Rotating the mesh by psi about z equals rotating each (a_lm, b_lm) coefficient pair by -m psi."""
    v, f = mg.icosphere(1)
    L, psi = 3, 0.61
    _, h, W = rand_inputs(9, f.shape[0], 16, 2, 3)
    R = np.array([[math.cos(psi), -math.sin(psi), 0], [math.sin(psi), math.cos(psi), 0], [0, 0, 1]])
    v64 = v.astype(np.float64)
    g_rot = oracle.f2v((v64 @ R.T).astype(np.float32), f, L, h, W)
    W2 = W.copy()
    for l in range(L + 1):
        for m in range(1, l + 1):
            c, s = math.cos(m * psi), math.sin(m * psi)
            a, b = W[kidx(l, m)], W[kidx(l, -m)]
            # B'_{+m} = c B_{+m} - s B_{-m};  B'_{-m} = s B_{+m} + c B_{-m}
            W2[kidx(l, m)] = c * a + s * b
            W2[kidx(l, -m)] = -s * a + c * b
    g_w = oracle.f2v(v, f, L, h, W2)
    np.testing.assert_allclose(g_rot, g_w, atol=2e-6)


def test_f2v_corner_swap_flips_normal():
    v, f = mg.icosphere(1)
    _, h, W = rand_inputs(10, f.shape[0], 4, 1, 1)
    f2 = f.copy()
    f2[:, [1, 2]] = f2[:, [2, 1]]
    Wm = W.copy()
    Wm[1:] *= -1.0        # l = 1 functions are odd
    np.testing.assert_allclose(oracle.f2v(v, f2, 1, h, W), oracle.f2v(v, f, 1, h, Wm), atol=1e-12)


def test_batched_equals_concatenation():
    a, b = mg.icosphere(1), mg.tetrahedron()
    batch = mg.pack_batch([a, b, a])
    _, h, W = rand_inputs(11, batch.n_facet, 9, 3, 2)
    g = oracle.f2v(batch.vert, batch.facet, 2, h, W)
    parts = []
    for i in range(3):
        m = batch.mesh(i)
        f0, f1 = batch.facet_off[i], batch.facet_off[i + 1]
        parts.append(oracle.f2v(m.vert, m.facet, 2, h[f0:f1], W))
    np.testing.assert_array_equal(g, np.concatenate(parts, 0))


# ------------------------------------------------------------------ vertex2facet
def v2f_corner_constants(L):
    """Closed-form basis values at the three corner directions (pole / equator formulas)."""
    def dfact(n):
        return 1.0 if n <= 0 else n * dfact(n - 2)
    K = (L + 1) ** 2
    Bc = np.zeros((3, K))
    for l in range(L + 1):
        for m in range(0, l + 1):
            N = math.sqrt((2 * l + 1) / (4 * math.pi) * math.factorial(l - m) / math.factorial(l + m))
            p0 = 0.0 if (l + m) % 2 else (-1.0) ** ((l - m) // 2) * dfact(l + m - 1) / dfact(l - m)
            Bc[0, kidx(l, m)] = N * p0
            Bc[1, kidx(l, m)] = N * p0 * math.cos(m * math.pi / 2)
            if m:
                Bc[1, kidx(l, -m)] = N * p0 * math.sin(m * math.pi / 2)
            else:
                Bc[2, kidx(l, 0)] = math.sqrt((2 * l + 1) / (4 * math.pi))
    return Bc


def test_v2f_closed_form_and_conservation():
    v, f = mg.icosphere(1)
    L = 4
    _, h, W = rand_inputs(12, v.shape[0], 25, 3, 5)
    g = oracle.v2f(v.shape[0], f, L, h, W)
    Bc = v2f_corner_constants(L)
    Wj = np.einsum("jk,kio->jio", Bc, W)
    ref = sum(h[f[:, j]] @ Wj[j] for j in range(3))
    np.testing.assert_allclose(g, ref, atol=1e-12)
    rows = np.array([3, 3, 0, 79])
    np.testing.assert_array_equal(oracle.v2f(v.shape[0], f, L, h, W, rows=rows), g[rows])


def test_v2f_depends_on_corner_order_not_on_geometry():
    v, f = mg.icosphere(1)
    _, h, W = rand_inputs(13, v.shape[0], 9, 2, 2)
    g = oracle.v2f(v.shape[0], f, 2, h, W)
    f2 = f[:, [1, 2, 0]]
    assert np.abs(oracle.v2f(v.shape[0], np.ascontiguousarray(f2), 2, h, W) - g).max() > 1e-3


# ------------------------------------------------------------------ facet2facet
def test_f2f_single_corner_point_reduces_to_v2f_term():
    """R_f = 1 with xi = e_j: the facet2facet value is the j-th term of Eq. 6."""
    L = 3
    rng = np.random.default_rng(14)
    F = 6
    tex_off = np.arange(F + 1, dtype=np.int32)
    jj = rng.integers(0, 3, F)
    bary = np.eye(3, dtype=np.float32)[jj]
    h = rng.standard_normal((F, 3))
    W = rng.uniform(-1, 1, (16, 3, 4))
    g = oracle.f2f(tex_off, bary, L, h, W)
    Bc = v2f_corner_constants(L)
    ref = np.stack([h[i] @ np.einsum("k,kio->io", Bc[jj[i]], W) for i in range(F)])
    np.testing.assert_allclose(g, ref, atol=1e-12)


def test_f2f_mean_duplicates_and_empty():
    L = 2
    rng = np.random.default_rng(15)
    lat = mg.bary_lattice(2)                                 # 6 points
    tex_off = np.array([0, 6, 18, 18, 19], dtype=np.int32)   # facet 1 = facet 0's points twice; facet 2 empty
    bary = np.concatenate([lat, lat, lat, mg.bary_lattice(0)], 0)
    h0 = rng.standard_normal((6, 3))
    h = np.concatenate([h0, h0, h0, rng.standard_normal((1, 3))], 0)
    W = rng.uniform(-1, 1, (9, 3, 2))
    g = oracle.f2f(tex_off, bary, L, h, W)
    np.testing.assert_allclose(g[1], g[0], atol=1e-13)
    assert np.all(g[2] == 0)
    # brute force via the library SH
    from scipy.special import sph_harm_y
    d = bary.astype(np.float64)
    d /= np.linalg.norm(d, axis=1, keepdims=True)
    th, ph = np.arccos(d[:, 2]), np.arctan2(d[:, 1], d[:, 0])
    B = np.zeros((d.shape[0], 9))
    for l in range(3):
        for m in range(l + 1):
            Y = sph_harm_y(l, m, th, ph) * (-1.0) ** m
            B[:, kidx(l, m)] = Y.real
            if m:
                B[:, kidx(l, -m)] = Y.imag
    yp = np.einsum("pk,pi,kio->po", B, h, W)
    np.testing.assert_allclose(g[0], yp[0:6].mean(0), atol=1e-12)
    np.testing.assert_allclose(g[3], yp[18], atol=1e-12)


# ------------------------------------------------------------------ backward passes
def _fd(fun, x, dg, eps=1e-6):
    """Central finite differences of <fun(x), dg> w.r.t. a few random entries of x."""
    rng = np.random.default_rng(99)
    idx = [tuple(rng.integers(0, s) for s in x.shape) for _ in range(12)]
    out = []
    for i in idx:
        xp, xm = x.copy(), x.copy()
        xp[i] += eps
        xm[i] -= eps
        out.append(((fun(xp) - fun(xm)) * dg).sum() / (2 * eps))
    return idx, np.array(out)


def test_f2v_bwd_finite_differences_and_adjoint():
    v, f = mg.icosphere(1)
    v = np.concatenate([v, [[3, 3, 3]]], 0).astype(np.float32)
    L = 2
    rng, h, W = rand_inputs(16, f.shape[0], 9, 3, 4)
    dg = rng.standard_normal((v.shape[0], 4))
    dh, dW = oracle.f2v_bwd(v, f, L, h, W, dg)
    idx, fd = _fd(lambda x: oracle.f2v(v, f, L, x, W), h, dg)
    np.testing.assert_allclose([dh[i] for i in idx], fd, rtol=1e-7, atol=1e-9)
    idx, fd = _fd(lambda x: oracle.f2v(v, f, L, h, x), W, dg)
    np.testing.assert_allclose([dW[i] for i in idx], fd, rtol=1e-7, atol=1e-9)
    g = oracle.f2v(v, f, L, h, W)
    np.testing.assert_allclose((g * dg).sum(), (h * dh).sum(), rtol=1e-12)
    np.testing.assert_allclose((g * dg).sum(), (W * dW).sum(), rtol=1e-12)
    rows = np.array([7, 1, 1])
    dh_s, _ = oracle.f2v_bwd(v, f, L, h, W, dg, rows=rows, want_dW=False)
    np.testing.assert_array_equal(dh_s, dh[rows])


def test_v2f_bwd_finite_differences_and_adjoint():
    v, f = mg.icosphere(1)
    V = v.shape[0] + 1                      # one isolated vertex
    L = 3
    rng, h, W = rand_inputs(17, V, 16, 2, 3)
    dg = rng.standard_normal((f.shape[0], 3))
    dh, dW = oracle.v2f_bwd(V, f, L, h, W, dg)
    assert np.all(dh[-1] == 0)
    idx, fd = _fd(lambda x: oracle.v2f(V, f, L, x, W), h, dg)
    np.testing.assert_allclose([dh[i] for i in idx], fd, rtol=1e-7, atol=1e-9)
    idx, fd = _fd(lambda x: oracle.v2f(V, f, L, h, x), W, dg)
    np.testing.assert_allclose([dW[i] for i in idx], fd, rtol=1e-7, atol=1e-9)
    g = oracle.v2f(V, f, L, h, W)
    np.testing.assert_allclose((g * dg).sum(), (h * dh).sum(), rtol=1e-12)
    np.testing.assert_allclose((g * dg).sum(), (W * dW).sum(), rtol=1e-12)


def test_f2f_bwd_finite_differences_and_adjoint():
    v, f = mg.icosphere(0)
    batch = mg.pack_batch([(v * np.array([1, 2, 3], dtype=np.float32), f)])
    tex_off, bary = mg.texture_layout(batch, 3, 1)
    assert len(set(np.diff(tex_off).tolist())) > 1
    L = 2
    P = int(tex_off[-1])
    rng, h, W = rand_inputs(18, P, 9, 3, 4)
    dg = rng.standard_normal((f.shape[0], 4))
    dh, dW = oracle.f2f_bwd(tex_off, bary, L, h, W, dg)
    idx, fd = _fd(lambda x: oracle.f2f(tex_off, bary, L, x, W), h, dg)
    np.testing.assert_allclose([dh[i] for i in idx], fd, rtol=1e-7, atol=1e-9)
    idx, fd = _fd(lambda x: oracle.f2f(tex_off, bary, L, h, x), W, dg)
    np.testing.assert_allclose([dW[i] for i in idx], fd, rtol=1e-7, atol=1e-9)
    g = oracle.f2f(tex_off, bary, L, h, W)
    np.testing.assert_allclose((g * dg).sum(), (h * dh).sum(), rtol=1e-12)
    np.testing.assert_allclose((g * dg).sum(), (W * dW).sum(), rtol=1e-12)


def test_v2f_and_f2f_take_no_geometry():
    """V2F and F2F are functions of connectivity / barycentric coordinates only (rotation and
    translation invariance stated in the paper's conclusion): their oracle entry points take no
    vertex positions, so a rigid motion of the mesh cannot change their result."""
    import inspect
    assert "vert" not in inspect.signature(oracle.v2f).parameters
    assert "vert" not in inspect.signature(oracle.f2f).parameters


def test_dW_rows_equal_the_rows_of_the_full_gradients():
    """The row-wise gradient functions (used where the whole dW takes the oracle too long) against the full
    backward functions, themselves pinned above by finite differences: same sums, so bit for bit; and one row
    written out in numpy from the transposed sum of Eq. 5 with the separately pinned basis."""
    v, f = mg.icosphere(2)
    v = np.concatenate([v, [[3, 3, 3]]], 0).astype(np.float32)         # one isolated vertex
    V, F, L, K, cin, cout = v.shape[0], f.shape[0], 3, 16, 5, 7
    rng = np.random.default_rng(31)
    wrows = np.array([0, 3, K * cin - 1, 17, 17, 42], dtype=np.int64)
    h, dg, W = rng.standard_normal((F, cin)), rng.standard_normal((V, cout)), rng.uniform(-1, 1, (K, cin, cout))
    _, dW = oracle.f2v_bwd(v, f, L, h, W, dg, want_dh=False)
    got = oracle.f2v_dW_rows(v, f, L, h, dg, wrows)
    np.testing.assert_array_equal(got, dW.reshape(K * cin, cout)[wrows])
    B = oracle.sh_basis(oracle.facet_normals(v, f), L)
    deg = np.bincount(f.ravel(), minlength=V).astype(np.float64)
    dy = sum(dg[f[:, j]] / deg[f[:, j], None] for j in range(3))
    k, ci = 3, 2
    np.testing.assert_allclose(got[3], (B[:, k] * h[:, ci]) @ dy, rtol=1e-12, atol=1e-13)

    h, dg = rng.standard_normal((V, cin)), rng.standard_normal((F, cout))
    _, dW = oracle.v2f_bwd(V, f, L, h, W, dg, want_dh=False)
    np.testing.assert_array_equal(oracle.v2f_dW_rows(V, f, L, h, dg, wrows), dW.reshape(K * cin, cout)[wrows])

    batch = mg.pack_batch([(v * np.array([1, 2, 3], dtype=np.float32), f)])
    tex_off, bary = mg.texture_layout(batch, 3, 1)
    P = int(tex_off[-1])
    h, dg = rng.standard_normal((P, cin)), rng.standard_normal((F, cout))
    _, dW = oracle.f2f_bwd(tex_off, bary, L, h, W, dg, want_dh=False)
    np.testing.assert_array_equal(oracle.f2f_dW_rows(tex_off, bary, L, h, dg, wrows), dW.reshape(K * cin, cout)[wrows])

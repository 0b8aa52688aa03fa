"""fp64 CPU oracle of the SH mesh convolutions -- TEST INFRASTRUCTURE, not the product.

Thin ctypes wrappers around oracle/pm_oracle.c (plain C, fp64, naive loops written from the
paper's Eq. 3-7).  Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this package; it imports nothing from the HIP path.

Parity status: pinned by tests/test_oracle_*.py, except agreement with the authors' released
code ("parity unpinned": coefficient order and the sqrt(2) convention are this build's reading).
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build.build())
    return _lib


def num_threads() -> int:
    """Threads the OpenMP loops of the oracle will use."""
    n = os.environ.get("OMP_NUM_THREADS")
    if n:
        return int(n.split(",")[0])
    return len(os.sched_getaffinity(0))


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t)) if a is not None else None


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _rows(rows):
    if rows is None:
        return None
    return np.ascontiguousarray(rows, dtype=np.int64)


def sh_basis(dirs, L: int, norm: int = 0) -> np.ndarray:
    """Eq. 3-4: the (L+1)^2 real SH basis values at each direction (need not be unit)."""
    d = _f64(dirs).reshape(-1, 3)
    K = (L + 1) ** 2
    out = np.empty((d.shape[0], K), dtype=np.float64)
    lib().orc_sh_basis(C.c_int64(d.shape[0]), _p(d, C.c_double), C.c_int(L), C.c_int(norm), _p(out, C.c_double))
    return out


def facet_normals(vert, facet) -> np.ndarray:
    vert, facet = _f32(vert), _i32(facet)
    out = np.empty((facet.shape[0], 3), dtype=np.float64)
    lib().orc_facet_normals(C.c_int64(facet.shape[0]), _p(vert, C.c_float), _p(facet, C.c_int32), _p(out, C.c_double))
    return out


def vf_adjacency(n_vert: int, facet):
    facet = _i32(facet)
    F = facet.shape[0]
    rp = np.empty(n_vert + 1, dtype=np.int32)
    col = np.empty(3 * F, dtype=np.int32)
    lib().orc_vf_adjacency(C.c_int64(n_vert), C.c_int64(F), _p(facet, C.c_int32), _p(rp, C.c_int32), _p(col, C.c_int32))
    return rp, col


def f2v(vert, facet, L, h, W, norm: int = 0, rows=None) -> np.ndarray:
    vert, facet, h, W = _f32(vert), _i32(facet), _f64(h), _f64(W)
    K, cin, cout = W.shape
    assert K == (L + 1) ** 2 and h.shape == (facet.shape[0], cin)
    rows = _rows(rows)
    n = vert.shape[0] if rows is None else rows.shape[0]
    out = np.empty((n, cout), dtype=np.float64)
    lib().orc_f2v(C.c_int64(vert.shape[0]), C.c_int64(facet.shape[0]), _p(vert, C.c_float), _p(facet, C.c_int32),
                  C.c_int(L), C.c_int(norm), C.c_int(cin), C.c_int(cout), _p(h, C.c_double), _p(W, C.c_double),
                  C.c_int64(n), _p(rows, C.c_int64), _p(out, C.c_double))
    return out


def f2v_bwd(vert, facet, L, h, W, dg, norm: int = 0, rows=None, want_dh=True, want_dW=True):
    vert, facet, h, W, dg = _f32(vert), _i32(facet), _f64(h), _f64(W), _f64(dg)
    K, cin, cout = W.shape
    assert dg.shape == (vert.shape[0], cout)
    rows = _rows(rows)
    n = facet.shape[0] if rows is None else rows.shape[0]
    dh = np.empty((n, cin), dtype=np.float64) if want_dh else None
    dW = np.empty_like(W) if want_dW else None
    lib().orc_f2v_bwd(C.c_int64(vert.shape[0]), C.c_int64(facet.shape[0]), _p(vert, C.c_float), _p(facet, C.c_int32),
                      C.c_int(L), C.c_int(norm), C.c_int(cin), C.c_int(cout), _p(h, C.c_double), _p(W, C.c_double),
                      _p(dg, C.c_double), C.c_int64(n), _p(rows, C.c_int64), _p(dh, C.c_double), _p(dW, C.c_double))
    return dh, dW


def v2f(n_vert, facet, L, h, W, norm: int = 0, rows=None) -> np.ndarray:
    facet, h, W = _i32(facet), _f64(h), _f64(W)
    K, cin, cout = W.shape
    assert h.shape == (n_vert, cin)
    rows = _rows(rows)
    n = facet.shape[0] if rows is None else rows.shape[0]
    out = np.empty((n, cout), dtype=np.float64)
    lib().orc_v2f(C.c_int64(n_vert), C.c_int64(facet.shape[0]), _p(facet, C.c_int32), C.c_int(L), C.c_int(norm),
                  C.c_int(cin), C.c_int(cout), _p(h, C.c_double), _p(W, C.c_double), C.c_int64(n),
                  _p(rows, C.c_int64), _p(out, C.c_double))
    return out


def v2f_bwd(n_vert, facet, L, h, W, dg, norm: int = 0, rows=None, want_dh=True, want_dW=True):
    facet, h, W, dg = _i32(facet), _f64(h), _f64(W), _f64(dg)
    K, cin, cout = W.shape
    assert dg.shape == (facet.shape[0], cout)
    rows = _rows(rows)
    n = n_vert if rows is None else rows.shape[0]
    dh = np.empty((n, cin), dtype=np.float64) if want_dh else None
    dW = np.empty_like(W) if want_dW else None
    lib().orc_v2f_bwd(C.c_int64(n_vert), C.c_int64(facet.shape[0]), _p(facet, C.c_int32), C.c_int(L), C.c_int(norm),
                      C.c_int(cin), C.c_int(cout), _p(h, C.c_double), _p(W, C.c_double), _p(dg, C.c_double),
                      C.c_int64(n), _p(rows, C.c_int64), _p(dh, C.c_double), _p(dW, C.c_double))
    return dh, dW


def f2v_sep(vert, facet, L, h, alpha, P, norm: int = 0, rows=None) -> np.ndarray:
    """Depth-wise separable facet2vertex: per-channel SH coefficients alpha [K,cin], point-wise P [cin,cout]."""
    vert, facet, h, alpha, P = _f32(vert), _i32(facet), _f64(h), _f64(alpha), _f64(P)
    K, cin = alpha.shape
    cout = P.shape[1]
    assert K == (L + 1) ** 2 and P.shape[0] == cin and h.shape == (facet.shape[0], cin)
    rows = _rows(rows)
    n = vert.shape[0] if rows is None else rows.shape[0]
    out = np.empty((n, cout), dtype=np.float64)
    lib().orc_f2v_sep(C.c_int64(vert.shape[0]), C.c_int64(facet.shape[0]), _p(vert, C.c_float), _p(facet, C.c_int32),
                      C.c_int(L), C.c_int(norm), C.c_int(cin), C.c_int(cout), _p(h, C.c_double), _p(alpha, C.c_double),
                      _p(P, C.c_double), C.c_int64(n), _p(rows, C.c_int64), _p(out, C.c_double))
    return out


def f2v_sep_bwd(vert, facet, L, h, alpha, P, dg, norm: int = 0, rows=None, want_dh=True, want_dw=True):
    """Returns (dh [rows or F, cin], dalpha [K,cin], dP [cin,cout]); dalpha/dP None unless want_dw."""
    vert, facet, h, alpha, P, dg = _f32(vert), _i32(facet), _f64(h), _f64(alpha), _f64(P), _f64(dg)
    K, cin = alpha.shape
    cout = P.shape[1]
    assert dg.shape == (vert.shape[0], cout)
    rows = _rows(rows)
    n = facet.shape[0] if rows is None else rows.shape[0]
    dh = np.empty((n, cin), dtype=np.float64) if want_dh else None
    da = np.empty_like(alpha) if want_dw else None
    dP = np.empty_like(P) if want_dw else None
    lib().orc_f2v_sep_bwd(C.c_int64(vert.shape[0]), C.c_int64(facet.shape[0]), _p(vert, C.c_float),
                          _p(facet, C.c_int32), C.c_int(L), C.c_int(norm), C.c_int(cin), C.c_int(cout),
                          _p(h, C.c_double), _p(alpha, C.c_double), _p(P, C.c_double), _p(dg, C.c_double),
                          C.c_int64(n), _p(rows, C.c_int64), _p(dh, C.c_double), _p(da, C.c_double), _p(dP, C.c_double))
    return dh, da, dP


def v2f_sep(n_vert, facet, L, h, alpha, P, norm: int = 0, rows=None) -> np.ndarray:
    facet, h, alpha, P = _i32(facet), _f64(h), _f64(alpha), _f64(P)
    K, cin = alpha.shape
    cout = P.shape[1]
    assert K == (L + 1) ** 2 and h.shape == (n_vert, cin)
    rows = _rows(rows)
    n = facet.shape[0] if rows is None else rows.shape[0]
    out = np.empty((n, cout), dtype=np.float64)
    lib().orc_v2f_sep(C.c_int64(n_vert), C.c_int64(facet.shape[0]), _p(facet, C.c_int32), C.c_int(L), C.c_int(norm),
                      C.c_int(cin), C.c_int(cout), _p(h, C.c_double), _p(alpha, C.c_double), _p(P, C.c_double),
                      C.c_int64(n), _p(rows, C.c_int64), _p(out, C.c_double))
    return out


def v2f_sep_bwd(n_vert, facet, L, h, alpha, P, dg, norm: int = 0, rows=None, want_dh=True, want_dw=True):
    facet, h, alpha, P, dg = _i32(facet), _f64(h), _f64(alpha), _f64(P), _f64(dg)
    K, cin = alpha.shape
    cout = P.shape[1]
    assert dg.shape == (facet.shape[0], cout)
    rows = _rows(rows)
    n = n_vert if rows is None else rows.shape[0]
    dh = np.empty((n, cin), dtype=np.float64) if want_dh else None
    da = np.empty_like(alpha) if want_dw else None
    dP = np.empty_like(P) if want_dw else None
    lib().orc_v2f_sep_bwd(C.c_int64(n_vert), C.c_int64(facet.shape[0]), _p(facet, C.c_int32), C.c_int(L),
                          C.c_int(norm), C.c_int(cin), C.c_int(cout), _p(h, C.c_double), _p(alpha, C.c_double),
                          _p(P, C.c_double), _p(dg, C.c_double), C.c_int64(n), _p(rows, C.c_int64),
                          _p(dh, C.c_double), _p(da, C.c_double), _p(dP, C.c_double))
    return dh, da, dP


def f2f(tex_off, bary, L, h, W, norm: int = 0, rows=None) -> np.ndarray:
    tex_off, bary, h, W = _i32(tex_off), _f32(bary), _f64(h), _f64(W)
    K, cin, cout = W.shape
    F = tex_off.shape[0] - 1
    rows = _rows(rows)
    n = F if rows is None else rows.shape[0]
    out = np.empty((n, cout), dtype=np.float64)
    lib().orc_f2f(C.c_int64(F), _p(tex_off, C.c_int32), _p(bary, C.c_float), C.c_int(L), C.c_int(norm), C.c_int(cin),
                  C.c_int(cout), _p(h, C.c_double), _p(W, C.c_double), C.c_int64(n), _p(rows, C.c_int64),
                  _p(out, C.c_double))
    return out


def f2f_bwd(tex_off, bary, L, h, W, dg, norm: int = 0, rows=None, want_dh=True, want_dW=True):
    tex_off, bary, h, W, dg = _i32(tex_off), _f32(bary), _f64(h), _f64(W), _f64(dg)
    K, cin, cout = W.shape
    F = tex_off.shape[0] - 1
    P = int(tex_off[-1])
    rows = _rows(rows)
    n = P if rows is None else rows.shape[0]
    dh = np.empty((n, cin), dtype=np.float64) if want_dh else None
    dW = np.empty_like(W) if want_dW else None
    lib().orc_f2f_bwd(C.c_int64(F), _p(tex_off, C.c_int32), _p(bary, C.c_float), C.c_int(L), C.c_int(norm),
                      C.c_int(cin), C.c_int(cout), _p(h, C.c_double), _p(W, C.c_double), _p(dg, C.c_double),
                      C.c_int64(n), _p(rows, C.c_int64), _p(dh, C.c_double), _p(dW, C.c_double))
    return dh, dW


def _wrows(wrows, K, cin):
    w = np.ascontiguousarray(wrows, dtype=np.int64)
    assert w.ndim == 1 and (w.size == 0 or (w.min() >= 0 and w.max() < K * cin))
    return w


def f2v_dW_rows(vert, facet, L, h, dg, wrows, norm: int = 0) -> np.ndarray:
    """Rows dW[k, ci, :] of the facet2vertex coefficient gradient, wrows[i] = k*cin + ci (sum over all facets)."""
    vert, facet, h, dg = _f32(vert), _i32(facet), _f64(h), _f64(dg)
    cin, cout = h.shape[1], dg.shape[1]
    w = _wrows(wrows, (L + 1) ** 2, cin)
    out = np.empty((w.shape[0], cout), dtype=np.float64)
    lib().orc_f2v_dW_rows(C.c_int64(vert.shape[0]), C.c_int64(facet.shape[0]), _p(vert, C.c_float), _p(facet, C.c_int32),
                          C.c_int(L), C.c_int(norm), C.c_int(cin), C.c_int(cout), _p(h, C.c_double), _p(dg, C.c_double),
                          C.c_int64(w.shape[0]), _p(w, C.c_int64), _p(out, C.c_double))
    return out


def v2f_dW_rows(n_vert, facet, L, h, dg, wrows, norm: int = 0) -> np.ndarray:
    facet, h, dg = _i32(facet), _f64(h), _f64(dg)
    cin, cout = h.shape[1], dg.shape[1]
    w = _wrows(wrows, (L + 1) ** 2, cin)
    out = np.empty((w.shape[0], cout), dtype=np.float64)
    lib().orc_v2f_dW_rows(C.c_int64(n_vert), C.c_int64(facet.shape[0]), _p(facet, C.c_int32), C.c_int(L), C.c_int(norm),
                          C.c_int(cin), C.c_int(cout), _p(h, C.c_double), _p(dg, C.c_double), C.c_int64(w.shape[0]),
                          _p(w, C.c_int64), _p(out, C.c_double))
    return out


def f2f_dW_rows(tex_off, bary, L, h, dg, wrows, norm: int = 0) -> np.ndarray:
    tex_off, bary, h, dg = _i32(tex_off), _f32(bary), _f64(h), _f64(dg)
    cin, cout = h.shape[1], dg.shape[1]
    w = _wrows(wrows, (L + 1) ** 2, cin)
    out = np.empty((w.shape[0], cout), dtype=np.float64)
    lib().orc_f2f_dW_rows(C.c_int64(tex_off.shape[0] - 1), _p(tex_off, C.c_int32), _p(bary, C.c_float), C.c_int(L),
                          C.c_int(norm), C.c_int(cin), C.c_int(cout), _p(h, C.c_double), _p(dg, C.c_double),
                          C.c_int64(w.shape[0]), _p(w, C.c_int64), _p(out, C.c_double))
    return out


def sh_basis_bwd(dirs, L: int, dbasis, norm: int = 0) -> np.ndarray:
    """Gradient of <dbasis, B(d/|d|)> with respect to the (unnormalised) directions d.

    The basis is a smooth function of d away from the origin; its derivative is taken here by
    fourth-order central differences of `sh_basis` in fp64 (relative step 1e-3 of |d|, truncation
    error ~1e-12 relative for L <= 5), which keeps this function a direct consequence of Eq. 3-4
    with no second derivation to get wrong.  Pinned against closed-form gradients for l <= 2.
    """
    d = _f64(dirs).reshape(-1, 3)
    db = _f64(dbasis)
    out = np.zeros_like(d)
    step = 1e-3 * np.linalg.norm(d, axis=1)
    for q in range(3):
        e = np.zeros((1, 3))
        e[0, q] = 1.0
        hq = step[:, None] * e
        f1 = sh_basis(d + hq, L, norm) - sh_basis(d - hq, L, norm)
        f2 = sh_basis(d + 2 * hq, L, norm) - sh_basis(d - 2 * hq, L, norm)
        deriv = (8.0 * f1 - f2) / (12.0 * step[:, None])
        out[:, q] = np.einsum("nk,nk->n", deriv, db)
    return out

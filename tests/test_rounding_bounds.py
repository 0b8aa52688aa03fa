"""What the bf16 storage format alone implies for the two operators that chain bf16 stores (CPU only).

rounding_model evaluates the oracle's formulas with the stored tensors rounded to bf16.  Its distance from the
unrounded oracle is the error a correct bf16 data path has by construction; the GPU tests hold the HIP results to
max(2e-2, 1.25 x that distance) per case (rounding_model.derived_bound) and to a small distance from the model.
These tests pin the model itself: with the rounding switched off it IS the oracle; single stores have the size
2^-8 (half a unit of the 8-bit significand) that bf16 implies; and the numbers for the shapes the GPU tests run are the ones the documentation quotes.
"""
import numpy as np
import pytest

import rounding_model as rm
from oracle import pcloud as opc
from oracle import v2v
from paper_2112_01801_amd import meshgen as mg
from parity_util import make_features, rel_err, rel_err_rows
from test_gpu_parity import small_batch
from test_gpu_pcloud import _params as pc_params
from test_gpu_v2v import CASES as V2V_CASES, _epilogues, _params as v2v_params


def _v2v_inputs(seed, L, cin, cmid, cout, mode):
    b = small_batch(seed)
    rng = np.random.default_rng(seed + 500)
    a1, P1 = v2v_params(rng, L, cin, cmid, "bf16")
    a2, P2 = v2v_params(rng, L, cmid, cout, "bf16")
    ep1, ep2 = _epilogues(rng, cmid, cout, mode)
    h = make_features(rng, b.n_vert, cin, "bf16")
    return b, rng, (a1, P1, ep1, a2, P2, ep2), h


def test_model_without_rounding_is_the_oracle(monkeypatch):
    monkeypatch.setattr(rm, "r16", lambda x: np.asarray(x, np.float64))
    b, rng, prm, h = _v2v_inputs(31, 3, 16, 24, 8, "affine")
    ro, rg, rz = v2v.v2v_sep(b.vert, b.facet, 3, h, *prm, parts=True)
    mo, mgg, mz = rm.v2v_forward_bf16(b.vert, b.facet, 3, h, *prm)
    np.testing.assert_allclose(mo, ro, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(mgg, rg, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(mz, rz, rtol=1e-12, atol=1e-13)
    d_out = rng.standard_normal((b.n_vert, 8))
    ref = v2v.v2v_sep_bwd(b.vert, b.facet, 3, h, *prm, d_out)
    got = rm.v2v_backward_bf16(b.vert, b.facet, 3, h, *prm, rg, rz, ro, d_out)
    for x, r in zip(got, ref):
        np.testing.assert_allclose(x, r, rtol=1e-10, atol=1e-12)
    xs = rng.uniform(0, 1, (300, 3)).astype(np.float32)
    ptr, idx = mg.range_neighbors(xs, xs, 0.2)
    alpha, c0, P = pc_params(rng, 2, 8, 6, "f32")
    hh = rng.standard_normal((300, 8))
    np.testing.assert_allclose(rm.pcloud_forward_bf16(xs, xs, ptr, idx, 0.2, 2, hh, alpha, c0, P),
                               opc.pcloud_conv(xs, xs, ptr, idx, 0.2, 2, hh, alpha, c0, P), rtol=1e-12, atol=1e-13)


def test_dense_f2v_dh_model_without_rounding_is_the_oracle(monkeypatch):
    import oracle
    monkeypatch.setattr(rm, "r16", lambda x: np.asarray(x, np.float64))
    b = small_batch(33)
    rng = np.random.default_rng(533)
    L, cin, cout = 2, 6, 5
    W = rng.standard_normal(((L + 1) ** 2, cin, cout))
    h, dg = rng.standard_normal((b.n_facet, cin)), rng.standard_normal((b.n_vert, cout))
    rdh, _ = oracle.f2v_bwd(b.vert, b.facet, L, h, W, dg)
    np.testing.assert_allclose(rm.f2v_dh_bf16(b.vert, b.facet, L, W, dg), rdh, rtol=1e-11, atol=1e-12)


def test_one_store_is_half_a_bf16_ulp():
    x = np.random.default_rng(0).standard_normal(100000)
    rel = np.abs(rm.r16(x) - x) / np.abs(x)
    assert 2.0 ** -8 * 0.98 < rel.max() <= 2.0 ** -8 and 0.3 < np.sqrt(np.mean(rel ** 2)) / 2.0 ** -8 < 0.5


@pytest.mark.parametrize("L,cin,cmid,cout,dtype,mode", [c for c in V2V_CASES if c[4] == "bf16"])
def test_v2v_block_bound_from_its_bf16_stores(L, cin, cmid, cout, dtype, mode):
    """Five stores forward (folded matrices, g, g*s2, z, o) and four backward (dq, du, T, dh): between 0.4e-2 and
    3.7e-2 on these shapes, i.e. a correct data path can exceed the single-convolution bar of 2e-2."""
    b, rng, prm, h = _v2v_inputs(31, L, cin, cmid, cout, mode)
    ro, rg, rz = v2v.v2v_sep(b.vert, b.facet, L, h, *prm, parts=True)
    mo, mgg, mz = rm.v2v_forward_bf16(b.vert, b.facet, L, h, *prm, paths=rm.v2v_paths(cin, cmid, cout))
    e = [rel_err(mo, ro), rel_err(mgg, rg), rel_err(mz, rz)]
    assert 2e-3 < e[0] < 2.5e-2 and 2e-3 < e[2] < 2.5e-2, e
    assert e[1] < 1.5e-2, e                                # the first convolution alone stays under the stated bar
    b, rng, prm, h = _v2v_inputs(32, L, cin, cmid, cout, mode)
    d_out = make_features(rng, b.n_vert, cout, "bf16")
    ro, rg, rz = v2v.v2v_sep(b.vert, b.facet, L, h, *prm, parts=True)
    ref = v2v.v2v_sep_bwd(b.vert, b.facet, L, h, *prm, d_out)
    got = rm.v2v_backward_bf16(b.vert, b.facet, L, h, *prm, rm.r16(rg), rm.r16(rz), rm.r16(ro), d_out)
    eb = [rel_err(x, r) for x, r in zip(got, ref)]
    assert all(2e-3 < v < 4e-2 for v in eb), eb


def _sheet(n, L=3, cin=64, cout=64):
    v, _ = mg.heightfield(n, n, np.random.default_rng(320))
    xs = v.astype(np.float32)
    rho = 5.0 * float(xs[:, 0].max() - xs[:, 0].min()) / (n - 1)
    ptr, idx = mg.range_neighbors(xs, xs, rho)
    rng = np.random.default_rng(321)
    alpha, c0, P = pc_params(rng, L, cin, cout, "bf16")
    h = make_features(rng, xs.shape[0], cin, "bf16")
    dg = make_features(rng, xs.shape[0], cout, "bf16")
    return xs, rho, ptr, idx, alpha, c0, P, h, dg


def test_pcloud_bound_from_rows_of_different_scale():
    """The 256 x 256 sheet of the GPU test (queries = sources, 1 to ~60 neighbours per point): the depth-wise rows y
    (bf16 operand of the point-wise matrix) of border points are several times larger than the rest, and 2^-8 of
    THEIR scale, measured against the global rms, is 4.5e-2 -- while every row is within 1.1e-2 of its own rms."""
    L = 3
    xs, rho, ptr, idx, alpha, c0, P, h, dg = _sheet(256)
    ref = opc.pcloud_conv(xs, xs, ptr, idx, rho, L, h, alpha, c0, P)
    m = rm.pcloud_forward_bf16(xs, xs, ptr, idx, rho, L, h, alpha, c0, P)
    assert 4e-2 < rel_err(m, ref) < 5e-2 and rel_err_rows(m, ref) < 1.2e-2


def test_pcloud_dh_has_one_store():
    L = 3
    xs, rho, ptr, idx, alpha, c0, P, h, dg = _sheet(128)
    rdh = opc.pcloud_conv_bwd(xs, xs, ptr, idx, rho, L, h, alpha, c0, P, dg)[0]
    assert rel_err(rm.pcloud_dh_bf16(xs, xs, ptr, idx, rho, L, h, alpha, c0, P, dg), rdh) < 5e-3

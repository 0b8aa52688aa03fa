"""Separable vertex2vertex block (vertex2facet -> affine/ReLU -> facet2vertex -> affine/ReLU): HIP path vs the
fp64 oracle through the C ABI.

The backward entry point takes the saved activations as inputs.  The parity test feeds it the oracle's (rounded to
the feature dtype), so that both sides take the ReLU decisions from the same values: an element whose
pre-activation is within rounding of zero may be cut on one side and kept on the other otherwise, which is a
different (equally valid) subgradient, not an error.  The forward test checks the saved tensors themselves.

Tolerance: fp32 is held to the stated 1e-4 throughout.  In bf16 the block chains several bf16 stores (two
convolutions in sequence), so each tensor is held (a) to max(2e-2, 1.25 x the error of rounding_model) against the
oracle -- rounding_model is the oracle with exactly the stored tensors rounded to bf16, tests/test_rounding_bounds.py
pins it and the bound it gives -- and (b) to two bf16 units from that model itself.  The facet features g, the output of the
first convolution alone, keep the stated 2e-2, and so does the second convolution alone: the block's output against
the oracle's second stage applied to the g the library saved.
"""
import numpy as np
import pytest

import oracle
import rounding_model as rm
from oracle import v2v
from paper_2112_01801_amd import meshgen as mg
from parity_util import TOL, make_features, pm_dtype, rel_err, to_dev, to_host
from test_gpu_parity import small_batch

pytestmark = pytest.mark.gpu

NEAR_MODEL = 2.0 ** -6   # distance of a bf16 result from the oracle-side model of its stores: two bf16 units (a tie that
                         # fp32 accumulation order rounds the other way, on the element and on one it was computed from)


def _held(got, ref, model, dtype, name=""):
    """fp32: the stated tolerance.  bf16: the bound its stores imply, and close to the model of those stores."""
    e = rel_err(got, ref)
    if dtype != "bf16":
        assert e < TOL[dtype], (name, e)
        return
    em, d = rel_err(model, ref), rel_err(got, model)
    print("%s: err %.2e  model %.2e  from model %.2e" % (name, e, em, d))
    assert e < rm.derived_bound(TOL[dtype], em), (name, e, em)
    assert d < NEAR_MODEL, (name, d)


@pytest.fixture(scope="module")
def pm():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2112_01801_amd import binding
    binding.lib()
    return binding


def _params(rng, L, cin, cout, dtype):
    K = (L + 1) ** 2
    alpha = (rng.uniform(-1, 1, (K, cin)) / np.sqrt(K)).astype(np.float32)
    P = (rng.uniform(-1, 1, (cin, cout)) * np.sqrt(3.0 / cin)).astype(np.float32)
    return alpha, (mg.round_to_bf16(P) if dtype == "bf16" else P)


def _epilogues(rng, cmid, cout, mode):
    """mode: 'none' | 'relu' | 'affine' (affine + ReLU on both stages).  Returns the oracle's triples."""
    if mode == "none":
        return None, None
    if mode == "relu":
        return (None, None, True), (None, None, True)
    f = lambda c: (rng.uniform(0.5, 1.5, c).astype(np.float32), rng.normal(0, 0.3, c).astype(np.float32), True)
    return f(cmid), f(cout)


def _dev_ep(pm, ep):
    import torch
    if ep is None:
        return None
    a, b, relu = ep
    t = lambda x: None if x is None else torch.from_numpy(x).cuda()
    return pm.Epilogue(t(a), t(b), relu)


# (L, cin, cmid, cout, dtype, epilogues)
CASES = [
    (3, 64, 64, 64, "bf16", "affine"),     # fused facet stage and fused point-wise stage
    (3, 64, 64, 64, "bf16", "none"),
    (2, 32, 96, 64, "bf16", "relu"),       # fused facet stage; point-wise stage through the general kernel + epilogue
    (4, 64, 128, 32, "bf16", "affine"),
    (5, 32, 32, 128, "bf16", "relu"),
    (0, 64, 32, 96, "bf16", "affine"),     # K = 1: one padded basis slot
    (1, 32, 64, 20, "bf16", "affine"),     # ragged output width
    (3, 20, 24, 16, "f32", "affine"),      # general shapes: the separable kernels with element-wise epilogues
    (2, 24, 40, 8, "bf16", "relu"),
    (3, 64, 64, 64, "f32", "relu"),
]


def _setup(pm, L, cin, cmid, cout, dtype, mode, seed, batch=None):
    import torch
    b = small_batch(seed) if batch is None else batch
    rng = np.random.default_rng(seed + 500)
    a1, P1 = _params(rng, L, cin, cmid, dtype)
    a2, P2 = _params(rng, L, cmid, cout, dtype)
    ep1, ep2 = _epilogues(rng, cmid, cout, mode)
    h = make_features(rng, b.n_vert, cin, dtype)
    mesh = pm.mesh_to_device(b)
    adj = pm.pm_build_vf_adjacency(mesh)
    dev = dict(h=to_dev(h, dtype), a1=torch.from_numpy(a1).cuda(), P1=to_dev(P1, dtype), a2=torch.from_numpy(a2).cuda(),
               P2=to_dev(P2, dtype), ep1=_dev_ep(pm, ep1), ep2=_dev_ep(pm, ep2))
    return b, rng, (a1, P1, ep1, a2, P2, ep2), h, mesh, adj, dev


@pytest.mark.parametrize("L,cin,cmid,cout,dtype,mode", CASES)
def test_v2v_forward(pm, L, cin, cmid, cout, dtype, mode):
    import torch
    b, rng, (a1, P1, ep1, a2, P2, ep2), h, mesh, adj, d = _setup(pm, L, cin, cmid, cout, dtype, mode, 31)
    ro, rg, rz = v2v.v2v_sep(b.vert, b.facet, L, h, a1, P1, ep1, a2, P2, ep2, parts=True)
    mo, mgg, mz = (rm.v2v_forward_bf16(b.vert, b.facet, L, h, a1, P1, ep1, a2, P2, ep2, paths=rm.v2v_paths(cin, cmid, cout))
                   if dtype == "bf16" else (None,) * 3)
    o = pm.pm_v2v_sep(mesh, adj, L, d["h"], d["a1"], d["P1"], d["ep1"], d["a2"], d["P2"], d["ep2"], pm_dtype(dtype))
    _held(to_host(o), ro, mo, dtype, "o")
    o2, g, z = pm.pm_v2v_sep(mesh, adj, L, d["h"], d["a1"], d["P1"], d["ep1"], d["a2"], d["P2"], d["ep2"], pm_dtype(dtype),
                             save=True)
    assert torch.equal(o2, o)
    assert rel_err(to_host(g), rg) < TOL[dtype]                 # the first convolution alone: the stated tolerance
    _held(to_host(z), rz, mz, dtype, "z")
    # the second convolution alone, at the stated tolerance: the oracle's facet2vertex stage on the saved g
    o_from_g = oracle.f2v_sep(b.vert, b.facet, L, to_host(g), a2, P2)
    a, sh, relu = v2v._ep(ep2, cout)
    assert rel_err(to_host(o), v2v._act(a * o_from_g + sh, relu)) < TOL[dtype]
    if mode != "none":
        assert float(g.float().min()) >= 0 and float(o.float().min()) >= 0


@pytest.mark.parametrize("L,cin,cmid,cout,dtype,mode", CASES)
def test_v2v_backward(pm, L, cin, cmid, cout, dtype, mode):
    import torch
    b, rng, (a1, P1, ep1, a2, P2, ep2), h, mesh, adj, d = _setup(pm, L, cin, cmid, cout, dtype, mode, 32)
    d_out = make_features(rng, b.n_vert, cout, dtype)
    ro, rg, rz = v2v.v2v_sep(b.vert, b.facet, L, h, a1, P1, ep1, a2, P2, ep2, parts=True)
    ref = v2v.v2v_sep_bwd(b.vert, b.facet, L, h, a1, P1, ep1, a2, P2, ep2, d_out)
    args = (mesh, adj, L, d["h"], d["a1"], d["P1"], d["ep1"], d["a2"], d["P2"], d["ep2"], to_dev(rg.astype(np.float32), dtype),
            to_dev(rz.astype(np.float32), dtype), to_dev(ro.astype(np.float32), dtype), to_dev(d_out, dtype), pm_dtype(dtype))
    got = pm.pm_v2v_sep_bwd(*args)
    model = (rm.v2v_backward_bf16(b.vert, b.facet, L, h, a1, P1, ep1, a2, P2, ep2, rm.r16(rg), rm.r16(rz), rm.r16(ro), d_out)
             if dtype == "bf16" else (None,) * 5)
    for name, x, r, m in zip(["dh", "dalpha1", "dP1", "dalpha2", "dP2"], got, ref, model):
        _held(to_host(x), r, m, dtype, name)
    # each group alone gives the same values
    dh1, *rest = pm.pm_v2v_sep_bwd(*args, want_dw=False)
    assert all(t is None for t in rest) and torch.equal(dh1, got[0])
    none, *dw = pm.pm_v2v_sep_bwd(*args, want_dh=False)
    assert none is None and all(torch.equal(x, y) for x, y in zip(dw, got[1:]))


def test_v2v_forward_then_backward_runs_on_its_own_saved_tensors(pm):
    """End to end on the library's own saved activations: finite, and close to the oracle in the mean (single ReLU
    decisions near zero may differ, so this is a loose check beside the element-wise ones above)."""
    L, cin, cmid, cout, dtype = 3, 64, 64, 64, "bf16"
    b, rng, (a1, P1, ep1, a2, P2, ep2), h, mesh, adj, d = _setup(pm, L, cin, cmid, cout, dtype, "affine", 33)
    d_out = make_features(rng, b.n_vert, cout, dtype)
    o, g, z = pm.pm_v2v_sep(mesh, adj, L, d["h"], d["a1"], d["P1"], d["ep1"], d["a2"], d["P2"], d["ep2"], 1, save=True)
    got = pm.pm_v2v_sep_bwd(mesh, adj, L, d["h"], d["a1"], d["P1"], d["ep1"], d["a2"], d["P2"], d["ep2"], g, z, o,
                            to_dev(d_out, dtype), 1)
    ref = v2v.v2v_sep_bwd(b.vert, b.facet, L, h, a1, P1, ep1, a2, P2, ep2, d_out)
    ratio = {}
    for name, x, r in zip(["dh", "dalpha1", "dP1", "dalpha2", "dP2"], got, ref):
        x = to_host(x)
        assert np.all(np.isfinite(x)), name
        ratio[name] = float(np.sqrt(np.mean((x - r) ** 2)) / np.sqrt(np.mean(r ** 2)))
    print("rms error / rms:", ratio)
    # nothing before the first ReLU changes dalpha2 and dP2; a flipped decision moves one of the few hundred terms of
    # a dh element, and about one element in a thousand sits within rounding of zero
    assert ratio["dalpha2"] < 2e-2 and ratio["dP2"] < 2e-2, ratio
    assert all(v < 1e-1 for v in ratio.values()), ratio


@pytest.mark.parametrize("dtype,c", [("bf16", 64), ("f32", 12)])
def test_v2v_degenerate_meshes(pm, dtype, c):
    """No facets at all (every vertex isolated): the output is act2(b2); gradients of the parameters are zero."""
    import torch
    L = 2
    v = np.random.default_rng(3).standard_normal((7, 3)).astype(np.float32)
    be = mg.pack_batch([(v, np.zeros((0, 3), np.int32))])
    b, rng, (a1, P1, ep1, a2, P2, ep2), h, mesh, adj, d = _setup(pm, L, c, c, c, dtype, "affine", 34, batch=be)
    o, g, z = pm.pm_v2v_sep(mesh, adj, L, d["h"], d["a1"], d["P1"], d["ep1"], d["a2"], d["P2"], d["ep2"], pm_dtype(dtype),
                            save=True)
    ref = v2v.v2v_sep(be.vert, be.facet, L, h, a1, P1, ep1, a2, P2, ep2)
    assert g.shape == (0, c) and not z.float().abs().any()
    assert rel_err(to_host(o), ref) < TOL[dtype]                # act2(b2), rounded once
    got = pm.pm_v2v_sep_bwd(mesh, adj, L, d["h"], d["a1"], d["P1"], d["ep1"], d["a2"], d["P2"], d["ep2"], g, z, o,
                            torch.ones_like(o), pm_dtype(dtype))
    assert all(not x.float().abs().any() for x in got)


def test_v2v_config3_full_size(pm):
    """The benchmark mesh at full size, bf16, 64 channels throughout: every output row against the oracle."""
    cfg = mg.config3(1024)
    L, c, dtype = 3, 64, "bf16"
    b, rng, (a1, P1, ep1, a2, P2, ep2), h, mesh, adj, d = _setup(pm, L, c, c, c, dtype, "affine", 35, batch=cfg.batch)
    o = pm.pm_v2v_sep(mesh, adj, L, d["h"], d["a1"], d["P1"], d["ep1"], d["a2"], d["P2"], d["ep2"], 1)
    ref = v2v.v2v_sep(b.vert, b.facet, L, h, a1, P1, ep1, a2, P2, ep2)
    model = rm.v2v_forward_bf16(b.vert, b.facet, L, h, a1, P1, ep1, a2, P2, ep2)[0]
    _held(to_host(o), ref, model, dtype, "o at config 3")


def test_v2v_backward_at_a_hierarchy_level_against_the_oracle(pm):
    """The 512 x 512 level of the decimation hierarchy (522,242 facets, 64 channels, bf16, both epilogues): all five
    gradients, every element, against the oracle (the full-size test below compares the library with its own forward)."""
    cfg = mg.config5_levels()[1]
    L, c, dtype = 3, 64, "bf16"
    b, rng, (a1, P1, ep1, a2, P2, ep2), h, mesh, adj, d = _setup(pm, L, c, c, c, dtype, "affine", 39, batch=cfg.batch)
    assert b.n_facet == 522242
    d_out = make_features(rng, b.n_vert, c, dtype)
    ro, rg, rz = v2v.v2v_sep(b.vert, b.facet, L, h, a1, P1, ep1, a2, P2, ep2, parts=True)
    ref = v2v.v2v_sep_bwd(b.vert, b.facet, L, h, a1, P1, ep1, a2, P2, ep2, d_out)
    got = pm.pm_v2v_sep_bwd(mesh, adj, L, d["h"], d["a1"], d["P1"], d["ep1"], d["a2"], d["P2"], d["ep2"],
                            to_dev(rg.astype(np.float32), dtype), to_dev(rz.astype(np.float32), dtype),
                            to_dev(ro.astype(np.float32), dtype), to_dev(d_out, dtype), 1)
    model = rm.v2v_backward_bf16(b.vert, b.facet, L, h, a1, P1, ep1, a2, P2, ep2, rm.r16(rg), rm.r16(rz), rm.r16(ro), d_out)
    for name, x, r, m in zip(["dh", "dalpha1", "dP1", "dalpha2", "dP2"], got, ref, model):
        _held(to_host(x), r, m, dtype, name + " at 512x512")


def test_v2v_config3_backward_adjoint(pm):
    """Full size, no activation (the block is then linear in h and in each parameter set): every gradient against
    the forward pass through <grad, direction> = <forward(direction), d_out>."""
    import torch
    cfg = mg.config3(1024)
    L, c, dtype = 3, 64, "bf16"
    b, rng, (a1, P1, ep1, a2, P2, ep2), h, mesh, adj, d = _setup(pm, L, c, c, c, dtype, "none", 37, batch=cfg.batch)
    d_out = to_dev(make_features(rng, b.n_vert, c, dtype), dtype)
    fwd = lambda **kw: pm.pm_v2v_sep(mesh, adj, L, kw.get("h", d["h"]), kw.get("a1", d["a1"]), kw.get("P1", d["P1"]), None,
                                     kw.get("a2", d["a2"]), kw.get("P2", d["P2"]), None, 1)
    o, g, z = pm.pm_v2v_sep(mesh, adj, L, d["h"], d["a1"], d["P1"], None, d["a2"], d["P2"], None, 1, save=True)
    dh, da1, dP1, da2, dP2 = pm.pm_v2v_sep_bwd(mesh, adj, L, d["h"], d["a1"], d["P1"], None, d["a2"], d["P2"], None, g, z, o,
                                               d_out, 1)
    r2 = np.random.default_rng(38)
    h2 = to_dev(make_features(r2, b.n_vert, c, dtype), dtype)
    a1b, P1b = _params(r2, L, c, c, dtype)
    a2b, P2b = _params(r2, L, c, c, dtype)
    cases = [("h", dh, h2), ("a1", da1, torch.from_numpy(a1b).cuda()), ("P1", dP1, to_dev(P1b, dtype)),
             ("a2", da2, torch.from_numpy(a2b).cuda()), ("P2", dP2, to_dev(P2b, dtype))]
    for name, grad, direction in cases:
        od = fwd(**{name: direction})
        lhs = float((grad.double() * direction.double()).sum())
        rhs = float((od.double() * d_out.double()).sum())
        scale = float((od.double() * d_out.double()).abs().sum())
        assert abs(lhs - rhs) <= 2e-3 * scale, (name, lhs, rhs, scale)


def test_v2v_argument_errors(pm):
    import torch
    b, rng, prm, h, mesh, adj, d = _setup(pm, 2, 16, 16, 16, "f32", "none", 36)
    tiny = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(pm.PmError) as e:
        pm.pm_v2v_sep(mesh, adj, 2, d["h"], d["a1"], d["P1"], None, d["a2"], d["P2"], None, 0, ws=tiny)
    assert e.value.status == -3
    assert pm.lib().pm_v2v_sep_ws_bytes(0, 10, 10, 9, 16, 16, 16, 0) == 0      # degree out of range

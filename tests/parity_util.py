"""Shared helpers of the GPU parity tests: seeded inputs, the error metric, oracle <-> HIP plumbing."""
from __future__ import annotations

import numpy as np

from paper_2112_01801_amd import meshgen as mg

TOL = {"f32": 1e-4, "bf16": 2e-2}
NW = 48            # sampled rows dW[k, ci, :] of the weight gradient
ADJ_TOL = {"bf16": 1e-2, "f32": 2e-5}


def rel_err_rows(got: np.ndarray, ref: np.ndarray) -> float:
    """Like rel_err, with a row whose own rms exceeds the global one measured against its own rms.

    For operators whose output rows differ widely in scale (a point with one neighbour beside points that
    average thirty): a bf16 operand carries 2^-9 of its row's scale, whatever the scale of the other rows."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape and ref.ndim == 2, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    assert np.all(np.isfinite(got)), "non-finite values in the HIP result"
    rms = float(np.sqrt(np.mean(ref ** 2)))
    row = np.sqrt(np.mean(ref ** 2, axis=1, keepdims=True))
    den = np.maximum(np.abs(ref), np.maximum(row, rms if rms > 0 else 1.0))
    return float(np.max(np.abs(got - ref) / den))


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max_i |got_i - ref_i| / max(|ref_i|, rms(ref))   (the tolerance of 1e-4 / 2e-2 applies to this)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    assert np.all(np.isfinite(got)), "non-finite values in the HIP result"
    rms = float(np.sqrt(np.mean(ref ** 2)))
    den = np.maximum(np.abs(ref), rms if rms > 0 else 1.0)
    return float(np.max(np.abs(got - ref) / den))


def make_features(rng, n, c, dtype):
    x = mg.normal_features(rng, n, c)
    return mg.round_to_bf16(x) if dtype == "bf16" else x


def make_coeffs(rng, K, cin, cout, dtype):
    w = mg.glorot_coeffs(rng, K, cin, cout)
    return mg.round_to_bf16(w) if dtype == "bf16" else w


def to_dev(x: np.ndarray, dtype: str):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def to_host(t) -> np.ndarray:
    return t.float().cpu().numpy().astype(np.float64)


def pm_dtype(dtype: str) -> int:
    return 1 if dtype == "bf16" else 0


def sample_rows(rng, n, k):
    if n <= k:
        return np.arange(n, dtype=np.int64)
    return np.sort(rng.choice(n, size=k, replace=False)).astype(np.int64)


N_PROBE = 6        # independent random W' of the adjoint identity


def _adjoint_gap(probes, dW, dg_d):
    """rms over the probes (W', g' = conv(h; W')) of <W', dW> - <g', dg>, over the 2-norm of the terms g'*dg (the size
    of each side: a sum of terms of random sign).  One probe alone can have a small <W', dW> by chance and then sees
    little of a wrong dW; the rms over several does not."""
    import torch
    num, den = 0.0, 0.0
    for Wp, gp in probes:
        lhs = float((torch.from_numpy(Wp).cuda().double() * dW.double()).sum())
        terms = gp.double() * dg_d.double()
        num += (lhs - float(terms.sum())) ** 2
        den += float(terms.pow(2).sum())
    return (num / den) ** 0.5


def adjoint_ok(fwd, make_w, first, dW, dg_d, dtype):
    """first = (W', g') already computed (and sample-checked) by the caller; fwd(W' on the device) gives further g';
    make_w() draws a fresh W' (numpy).  bf16: g' carries two roundings of relative size 2^-8 at most per element,
    independent between elements, so the gap is about 2e-3 of the 2-norm; fp32: accumulation error only."""
    probes = [first]
    for _ in range(N_PROBE - 1):
        Wp = make_w()
        probes.append((Wp, fwd(to_dev(Wp, dtype))))
    gap = _adjoint_gap(probes, dW, dg_d)
    assert gap <= ADJ_TOL[dtype], gap
    # negative controls: the identity has to see a wrong dW
    bad = dW.clone()
    bad[dW.shape[0] // 2] = 0
    assert _adjoint_gap(probes, bad, dg_d) > 3 * ADJ_TOL[dtype]
    assert _adjoint_gap(probes, dW * 1.1, dg_d) > 3 * ADJ_TOL[dtype]


def sample_wrows(rng, K, cin):
    w = np.sort(rng.choice(K * cin, size=min(NW, K * cin), replace=False)).astype(np.int64)
    w[0], w[-1] = 0, K * cin - 1
    return w

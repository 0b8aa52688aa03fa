"""The entry point that allocates nothing (pm_v2f_noalloc) against pm_v2f, through the C ABI: two calls in a row,
the second with a smaller input and other channel counts, so the static scratch array holds the first call's
image when the second starts; then the refusal of a shape whose image does not fit."""
import numpy as np
import pytest

import oracle
from paper_2112_01801_amd import meshgen as mg
from parity_util import TOL, make_coeffs, make_features, pm_dtype, rel_err, to_dev, to_host
from test_gpu_parity import small_batch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pm():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2112_01801_amd import binding
    binding.lib()
    return binding


def test_two_calls_in_a_row_match_the_workspace_entry_point(pm):
    import torch
    big = mg.pack_batch([mg.heightfield(90, 70, np.random.default_rng(1), random_diag=True)])      # 12,282 facets
    cases = [(big, 3, 64, 128, "bf16", 71), (small_batch(72), 2, 24, 40, "f32", 73), (small_batch(74), 3, 64, 64, "bf16", 75)]
    for b, L, cin, cout, dtype, seed in cases:
        rng = np.random.default_rng(seed)
        K = (L + 1) ** 2
        W = make_coeffs(rng, K, cin, cout, dtype)
        h = make_features(rng, b.n_vert, cin, dtype)
        mesh = pm.mesh_to_device(b)
        h_d, W_d, dt = to_dev(h, dtype), to_dev(W, dtype), pm_dtype(dtype)
        ref = pm.pm_v2f(mesh, L, h_d, W_d, dt)
        out = torch.full_like(ref, float("nan"))
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        pm.pm_v2f_noalloc(mesh, L, h_d, W_d, dt, out)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(out, ref)                                     # same kernels, same image: bit for bit
        assert rel_err(to_host(out), oracle.v2f(b.n_vert, b.facet, L, h, W)) < TOL[dtype]


def test_shape_beyond_the_static_array_is_refused(pm):
    import torch
    b = small_batch(76)
    mesh = pm.mesh_to_device(b)
    cin = cout = 1024                                    # 3 * 1024 * 1024 * 4 bytes of image > 4 MiB
    W = torch.zeros((1, cin, cout), device="cuda")
    h = torch.zeros((b.n_vert, cin), device="cuda")
    out = torch.zeros((b.n_facet, cout), device="cuda")
    with pytest.raises(pm.PmError) as e:
        pm.pm_v2f_noalloc(mesh, 0, h, W, 0, out)
    assert e.value.status == -3 and "scratch" in str(e.value)

"""The allocation-free potential (swarm_potential_static) against swarm_potential and the oracle:
two calls in a row on one GPU, the second over a smaller matrix, so that whatever the first call
left in the library's static scratch array must not leak into the second result."""
import numpy as np
import pytest
import torch

import workloads as wl
from helpers import TOL_ELEMENTWISE, assert_close, force_state, make_both

pytestmark = pytest.mark.gpu


def filled(gpu, n, d, seed):
    g, c = make_both(gpu, n, d, wl.complete_graph(n), 8, 1.0, 0, 0.0)
    gen = np.random.Generator(np.random.PCG64(seed))
    c.X[:] = (gen.standard_normal((n, d)) * gen.uniform(0.1, 3.0, size=(n, 1)) + 50.0).astype(np.float32)
    force_state(gpu, g, c)
    return g, c


def test_static_scratch_potential_equals_the_handle_entry_point_twice_in_a_row(gpu):
    big = filled(gpu, 12, 8 * 40001, 1)          # 313 workgroups of partial sums, ragged last one
    small = filled(gpu, 5, 8 * 333, 2)           # 3 workgroups: reads only what it wrote
    for g, c in (big, small):
        n, d = c.n, c.d
        mu_handle = torch.empty(d, dtype=torch.float32, device="cuda")
        gamma_handle = g.potential(mu_handle)
        X = g.models_view(gpu.COMM)
        gamma_dev = torch.full((1,), -1.0, dtype=torch.float64, device="cuda")
        mu_static = torch.full((d,), -1.0, dtype=torch.float32, device="cuda")
        gpu.potential_static(X, gamma_dev, mu_static)
        torch.cuda.synchronize()
        assert gamma_dev.item() == gamma_handle                    # same kernels, same order of sums
        assert torch.equal(mu_static, mu_handle)
        assert gamma_dev.item() == pytest.approx(c.potential(), rel=1e-9)
        assert_close(mu_static.cpu().numpy(), c.mean(), TOL_ELEMENTWISE, "mean model")
    # a sub-matrix of the big swarm (first 7 nodes), without the mean output
    g, c = big
    gamma_dev = torch.zeros(1, dtype=torch.float64, device="cuda")
    gpu.potential_static(g.models_view(gpu.COMM)[:7], gamma_dev)
    x = c.X[:7].astype(np.float64)
    assert gamma_dev.item() == pytest.approx(float(((x - x.mean(axis=0)) ** 2).sum()), rel=1e-9)


def test_static_scratch_potential_rejects_what_it_cannot_hold(gpu):
    gamma_dev = torch.zeros(1, dtype=torch.float64, device="cuda")
    X = torch.zeros((2, 16), dtype=torch.float32, device="cuda")
    lib = gpu.lib()
    import ctypes
    too_wide = (1 << 27) + 4                                         # one workgroup of partial sums too many
    rc = lib.swarm_potential_static(ctypes.c_void_p(X.data_ptr()), 2, too_wide, ctypes.c_void_p(gamma_dev.data_ptr()),
                                    None, None)
    assert rc == gpu.EINVAL and b"134217728" in lib.swarm_last_error(None)
    assert lib.swarm_potential_static(ctypes.c_void_p(X.data_ptr()), 2, 18, ctypes.c_void_p(gamma_dev.data_ptr()),
                                      None, None) == gpu.EINVAL        # d not a multiple of 4
    assert lib.swarm_potential_static(None, 2, 16, ctypes.c_void_p(gamma_dev.data_ptr()), None, None) == gpu.EINVAL

"""Parity at the benchmark's full size and launch configuration (n = 64, d = 25.6 M, 4-bit
codes, reads one round stale): the oracle evaluates column windows (every step is
per-coordinate and the random streams are counter-based), the GPU runs the whole rows."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle.objectives import DiagQuadratic
from oracle.swarm import SwarmOracle
from helpers import TOL_ELEMENTWISE, assert_close

pytestmark = pytest.mark.gpu


def test_config4_full_size_sampled_windows(gpu):
    cfg = wl.CONFIGS[4]
    n, d, bits, H, lr, S, sigma = cfg["n"], cfg["d"], cfg["bits"], cfg["H"], cfg["lr"], cfg["stale_max"], cfg["sigma"]
    eps, seed = 0.5, 0
    edges = wl.random_regular_graph(n, 4, 0)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1)
    a = torch.empty((n, d), dtype=torch.float32, device="cuda").uniform_(0.5, 2.0, generator=gen)
    c = torch.empty((n, d), dtype=torch.float32, device="cuda").normal_(0.0, 1.0, generator=gen)
    c += torch.randn(n, 1, generator=gen, device="cuda")
    g = gpu.Swarm(n, d, edges, bits, eps, H, lr, S, seed)
    g.set_objective_diag(a, c, sigma)
    g.models_view(gpu.COMM).normal_(0.0, 0.7, generator=gen)        # any state: start away from zero
    torch.cuda.synchronize()
    width = 6 * 512 + 8                                             # several tiles and a ragged edge
    starts = [0, 8 * 1234567, d - width]                            # first, an unaligned middle, last columns
    oracles = []
    for k0 in starts:
        o = SwarmOracle(n, d, edges, bits, eps, H, lr, S, seed, k0=k0, k1=k0 + width)
        o.objective = DiagQuadratic(a[:, k0:k0 + width].cpu().numpy(), c[:, k0:k0 + width].cpu().numpy(), sigma, k0=k0)
        oracles.append(o)
    for r in range(3):
        for o, k0 in zip(oracles, starts):                           # same state on both sides
            o.X[:] = g.read_models(gpu.COMM, k0=k0, length=width)
        pairs = g.sample_matching()
        assert np.array_equal(pairs, oracles[0].sample_matching().astype(np.uint32))
        stale = np.full(n, 1, dtype=np.uint8)
        g.local_steps()
        g.gossip_round(None, stale)                                  # the launch configuration bench.py times
        for o, k0 in zip(oracles, starts):
            o.local_steps()
            assert_close(g.read_models(gpu.LIVE, k0=k0, length=width), o.W, TOL_ELEMENTWISE, f"W window {k0} round {r}")
            o.gossip_round(pairs, stale)
            for node in (0, 17, n - 1):
                got = g.read_codes(node, byte0=k0 * bits // 8, length=width * bits // 8)
                assert np.array_equal(got, o.ring[r % (S + 1)][node]), f"codes window {k0} node {node} round {r}"
            assert_close(g.read_models(gpu.COMM, k0=k0, length=width), o.X, 2 * TOL_ELEMENTWISE,
                         f"X window {k0} round {r}")
    cnt = g.counters()
    assert cnt["rounds"] == 3 and cnt["interactions"] == oracles[0].interactions
    assert cnt["bits_communicated"] == oracles[0].bits_communicated
    # a property that holds at any size: the mean model moves only by the applied updates and the
    # quantization error, so after the rounds it stays finite and the potential is positive
    assert np.isfinite(g.potential()) and g.potential() > 0

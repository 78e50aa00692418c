"""Parity at the full sizes of the workload configurations, in the launch configuration the
benchmark times.  For the per-coordinate objectives the oracle evaluates column windows (every
step is per-coordinate and the random streams are counter-based) while the GPU runs whole rows;
for the MLP the oracle evaluates a few whole nodes."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle.objectives import DiagQuadratic, MixtureMLP
from oracle.swarm import SwarmOracle
from helpers import TOL_ELEMENTWISE, TOL_TWO_STAGE, TOL_GEMM, assert_close, disjoint_prefix

pytestmark = pytest.mark.gpu


def graph_of(cfg):
    n = cfg["n"]
    return {"regular4": lambda: wl.random_regular_graph(n, 4, 0), "regular8": lambda: wl.random_regular_graph(n, 8, 0),
            "torus8x8": lambda: wl.torus_graph(8, 8), "complete": lambda: wl.complete_graph(n)}[cfg["graph"]]()


def register_window(g, gpu, node, k0, width, bits, prefix, d):
    """Bytes of a node's last published register that cover columns [k0, k0 + width)."""
    if not prefix:
        return g.read_codes(node, byte0=k0 * bits // 8, length=width * bits // 8)
    return np.concatenate([g.read_codes(node, byte0=k0 // 2, length=width // 2),               # bits 0-3
                           g.read_codes(node, byte0=d // 2 + k0 // 2, length=width // 2),      # bits 4-7
                           g.read_codes(node, byte0=d + k0, length=width),                     # bits 8-15
                           g.read_codes(node, byte0=2 * d + 8 * (k0 // 512), length=8 * (width // 512))])


@pytest.mark.parametrize("cfg_id,eps,mode", [(2, 2.0 ** -4, "two calls"), (4, 0.5, "two calls"), (5, 0.25, "two calls"),
                                             (4, 0.5, "one pass"), (5, 0.25, "one pass"), (4, 0.5, "one pass, prefix")])
def test_diag_configs_full_size_sampled_windows(gpu, cfg_id, eps, mode):
    """mode: the two entry points (swarm_local_steps + swarm_gossip_round) or the one-pass round the
    benchmark times by default; "prefix": 16-bit multi-resolution registers instead of the fixed b bits."""
    cfg = wl.CONFIGS[cfg_id]
    n, d, bits, H, lr, S, sigma = cfg["n"], cfg["d"], cfg["bits"], cfg["H"], cfg["lr"], cfg["stale_max"], cfg["sigma"]
    one_pass, prefix = mode.startswith("one pass"), mode.endswith("prefix")
    if prefix:
        bits = 16
    seed = cfg_id
    edges = graph_of(cfg)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(cfg_id)
    a = torch.empty((n, d), dtype=torch.float32, device="cuda").uniform_(0.0, 1.0, generator=gen)
    if cfg["a_law"] == "uniform":
        a.mul_(cfg["a_hi"] - cfg["a_lo"]).add_(cfg["a_lo"])
    else:
        a.mul_(float(np.log(cfg["a_hi"] / cfg["a_lo"]))).add_(float(np.log(cfg["a_lo"]))).exp_()
    c = torch.empty((n, d), dtype=torch.float32, device="cuda").normal_(0.0, 1.0, generator=gen)
    c += cfg["shift_sigma"] * torch.randn(n, 1, generator=gen, device="cuda")
    g = gpu.Swarm(n, d, edges, bits, eps, H, lr, S, seed, codec=gpu.CODEC_PREFIX if prefix else gpu.CODEC_FIXED)
    g.set_objective_diag(a, c, sigma)
    g.models_view(gpu.COMM).normal_(0.0, 0.7, generator=gen)        # any state: start away from zero
    torch.cuda.synchronize()
    width = 6 * 512 + 8                                             # several tiles and a ragged edge
    starts = [0, 8 * (d // 24) + 8, d - width]                      # first, an unaligned middle, last columns
    if prefix:                                                      # whole checksum tiles
        width = 6 * 512
        starts = [0, 512 * (d // 1536), 512 * ((d - width) // 512)]
    oracles = []
    for k0 in starts:
        o = SwarmOracle(n, d, edges, bits, eps, H, lr, S, seed, k0=k0, k1=k0 + width, codec="prefix" if prefix else "fixed")
        o.objective = DiagQuadratic(a[:, k0:k0 + width].cpu().numpy(), c[:, k0:k0 + width].cpu().numpy(), sigma, k0=k0)
        oracles.append(o)
    for o, k0 in zip(oracles, starts):                               # the seeded initial state, read once
        o.X[:] = g.read_models(gpu.COMM, k0=k0, length=width)
    for r in range(4):
        for o, k0 in zip(oracles, starts):                           # the oracle's state is forced into the device
            g.write_models(gpu.COMM, o.X, k0=k0)
        pairs = g.sample_matching()
        assert np.array_equal(pairs, oracles[0].sample_matching().astype(np.uint32))
        if cfg.get("stale") == "fixed1":
            stale = np.full(n, 1, dtype=np.uint8)
        elif cfg.get("stale") == "uniform":
            stale = g.sample_stale()
            assert np.array_equal(stale, oracles[0].sample_stale().astype(np.uint8))
        else:
            stale = None
        if one_pass:                                                 # the launch configurations bench.py times
            g.round_fused(None, stale)
        else:
            g.local_steps()
            g.gossip_round(None, stale)
        for o, k0 in zip(oracles, starts):
            o.local_steps()
            if not one_pass:
                assert_close(g.read_models(gpu.LIVE, k0=k0, length=width), o.W, TOL_ELEMENTWISE, f"W window {k0} round {r}")
            o.gossip_round(pairs, stale)
            for node in (0, n // 3, n - 1):
                got = register_window(g, gpu, node, k0, width, bits, prefix, d)
                assert np.array_equal(got, o.ring[r % (S + 1)][node]), f"codes window {k0} node {node} round {r}"
            assert_close(g.read_models(gpu.COMM, k0=k0, length=width), o.X, TOL_TWO_STAGE,
                         f"X window {k0} round {r}")
    cnt = g.counters()
    assert cnt["rounds"] == 4 and cnt["interactions"] == oracles[0].interactions
    if not prefix:                                                   # prefix reads: the bits depend on every tile of the row
        assert cnt["bits_communicated"] == oracles[0].bits_communicated
    assert np.isfinite(g.potential()) and g.potential() > 0


@pytest.mark.parametrize("arithmetic", ["float32", "three bf16 products"])
def test_mlp_config_full_size_sampled_nodes(gpu, arithmetic):
    """n = 256 nodes, 1024-4096-1024 perceptron (d = 8.4 M), batch 128, H = 2, 8-bit codes: the oracle
    recomputes the local steps of two whole nodes and one matched pair of the gossip round."""
    cfg = wl.CONFIGS[3]
    n, d, bits, H, lr = cfg["n"], cfg["d"], cfg["bits"], cfg["H"], cfg["lr"]
    eps, seed = 2.0 ** -10, 3
    edges = graph_of(cfg)
    means, cdf = wl.mixture_data(n, cfg["n_in"], cfg["n_out"], 0, cfg["alpha"])
    gen = torch.Generator(device="cuda")
    gen.manual_seed(3)
    g = gpu.Swarm(n, d, edges, bits, eps, H, lr, 0, seed)
    g.set_objective_mlp(cfg["n_in"], cfg["n_hid"], cfg["n_out"], torch.from_numpy(means).cuda(),
                        torch.from_numpy(cdf).cuda(), cfg["data_sigma"], cfg["batch"])
    if arithmetic != "float32":
        g.set_mlp_arithmetic(gpu.MLP_BF16X3)
    g.models_view(gpu.COMM).normal_(0.0, 0.02, generator=gen)
    torch.cuda.synchronize()
    pairs = g.sample_matching()
    i, j = (int(v) for v in pairs[len(pairs) // 2])                 # one matched pair in the middle of the list
    obj = MixtureMLP(cfg["n_in"], cfg["n_hid"], cfg["n_out"], means, cdf, cfg["data_sigma"], cfg["batch"])
    X = {u: g.read_models(gpu.COMM, node0=u, count=1)[0] for u in (i, j)}
    g.local_steps()
    g.gossip_round(None)
    W = {}
    for u in (i, j):
        w = X[u].astype(np.float64)
        for q in range(H):
            w = w - float(np.float32(lr)) * obj.gradient(u, w, seed, 0, q)
        W[u] = w
        assert_close(g.read_models(gpu.LIVE, node0=u, count=1)[0], w, TOL_GEMM, f"W of node {u}")
    # the pair's gossip step written with the oracle's quantizer, from the same X and the oracle's own W
    from oracle import quantizer as qz, rng
    z = {u: qz.stochastic_round(X[u], eps, rng.sr_halves(seed, u, 0, 0, d)) for u in (i, j)}
    for u, v in ((i, j), (j, i)):
        seen = qz.decode(qz.code(z[v], bits), X[u], eps, bits)
        want = (z[u] + seen) * (0.5 * eps) + (W[u] - X[u].astype(np.float64))
        assert np.array_equal(g.read_codes(u), qz.pack(qz.code(z[u], bits), bits)), f"codes of node {u}"
        assert_close(g.read_models(gpu.COMM, node0=u, count=1)[0], want, TOL_GEMM, f"X of node {u}")


def test_algorithm1_run_config4_shape_full_size(gpu):
    """Algorithm 1 at config 4's shape with fresh reads, the run `bench.py --sequential` times.  Teacher-forced on
    column windows: from the oracle's state, the next interactions that touch disjoint nodes -- one launch of the
    batched run, local steps inside -- against the oracle taking them one after the other (codes bit-exact: nothing
    quantized there depends on the device's own float32 steps).  Then a longer run with dependent interactions on
    whole rows against one swarm_sample_pair + swarm_interact per step on a second handle, bit for bit."""
    cfg = wl.CONFIGS[4]
    n, d, bits, H, lr, sigma, eps, seed = cfg["n"], cfg["d"], cfg["bits"], cfg["H"], cfg["lr"], cfg["sigma"], 0.5, 4
    edges = graph_of(cfg)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(44)
    a = torch.empty((n, d), dtype=torch.float32, device="cuda").uniform_(cfg["a_lo"], cfg["a_hi"], generator=gen)
    c = torch.empty((n, d), dtype=torch.float32, device="cuda").normal_(0.0, 1.0, generator=gen)
    g = gpu.Swarm(n, d, edges, bits, eps, H, lr, 0, seed)
    g.set_objective_diag(a, c, sigma)
    g.models_view(gpu.COMM).normal_(0.0, 0.7, generator=gen)
    g.models_view(gpu.SNAP).copy_(g.models_view(gpu.COMM)).add_(0.01 * torch.randn(n, 1, generator=gen, device="cuda"))
    torch.cuda.synchronize()
    width = 6 * 512 + 8
    starts = [0, 8 * (d // 24) + 8, d - width]
    oracles = []
    for k0 in starts:
        o = SwarmOracle(n, d, edges, bits, eps, H, lr, 0, seed, k0=k0, k1=k0 + width)
        o.objective = DiagQuadratic(a[:, k0:k0 + width].cpu().numpy(), c[:, k0:k0 + width].cpu().numpy(), sigma, k0=k0)
        o.X[:] = g.read_models(gpu.COMM, k0=k0, length=width)
        o.Xhat[:] = g.read_models(gpu.SNAP, k0=k0, length=width)
        oracles.append(o)
    widest = 0
    for rep in range(4):
        for o, k0 in zip(oracles, starts):
            g.write_models(gpu.COMM, o.X, k0=k0)
            g.write_models(gpu.SNAP, o.Xhat, k0=k0)
        k = disjoint_prefix(oracles[0], n // 2)
        widest = max(widest, k)
        pairs, launches = g.run_sequential(k)
        assert launches == 1
        for o, k0 in zip(oracles, starts):
            steps = [o.step_sequential() for _ in range(k)]
            assert [tuple(p) for p in pairs.tolist()] == steps
            for i, j in steps:
                for node in (i, j):
                    got = g.read_codes(node, byte0=k0 * bits // 8, length=width * bits // 8)
                    assert np.array_equal(got, o.ring[0][node]), f"register of node {node}, window {k0}, launch {rep}"
            assert_close(g.read_models(gpu.COMM, k0=k0, length=width), o.X, TOL_TWO_STAGE, f"X window {k0} launch {rep}")
            assert_close(g.read_models(gpu.SNAP, k0=k0, length=width), o.Xhat, TOL_TWO_STAGE, f"snapshots window {k0}")
        cnt = g.counters()
        assert cnt["interactions"] == oracles[0].interactions
    assert widest >= 2
    g.close()
    # dependent interactions, whole rows: the batched run against one call per interaction
    T = 48
    twins = []
    for _ in range(2):
        t = gpu.Swarm(n, d, edges, bits, eps, H, lr, 0, seed)
        t.set_objective_diag(a, c, sigma)
        gen.manual_seed(45)
        t.models_view(gpu.COMM).normal_(0.0, 0.7, generator=gen)
        t.models_view(gpu.SNAP).copy_(t.models_view(gpu.COMM)).add_(0.01 * torch.randn(n, 1, generator=gen, device="cuda"))
        twins.append(t)
    g1, g2 = twins
    torch.cuda.synchronize()
    assert torch.equal(g1.models_view(gpu.COMM), g2.models_view(gpu.COMM))
    drawn = []
    for t in range(T):
        i, j = g1.sample_pair()
        drawn.append((i, j))
        g1.interact(i, j)
    pairs, launches = g2.run_sequential(T)
    assert [tuple(p) for p in pairs.tolist()] == drawn and 1 < launches < T
    torch.cuda.synchronize()
    assert torch.equal(g1.models_view(gpu.COMM), g2.models_view(gpu.COMM))
    assert torch.equal(g1.models_view(gpu.SNAP), g2.models_view(gpu.SNAP))
    for node in sorted({v for p in drawn for v in p})[:8]:
        assert np.array_equal(g1.read_codes(node), g2.read_codes(node)), f"register of node {node}"
    assert g1.counters() == g2.counters()

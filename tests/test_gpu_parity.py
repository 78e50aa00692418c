"""GPU parity: the HIP library against the CPU oracle on identical seeded inputs.
Integer work (codes, matchings, random streams) must be bit-exact; float32 results are
within 1e-6 * max(1, |oracle|) for averaging and elementwise updates."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import quantizer as qz
from oracle import rng
from oracle.objectives import DiagQuadratic
from helpers import TOL_ELEMENTWISE, TOL_TWO_STAGE, assert_close, force_state, make_both, ring_row

pytestmark = pytest.mark.gpu

D_RAGGED = 8 * 5231          # 81.7 tiles of 512 coordinates: several workgroups and a ragged tail


def models(gen, n, d, scale=1.0):
    return (gen.standard_normal((n, d)) * scale).astype(np.float32)


# ------------------------------------------------------------------ stateless codec
@pytest.mark.parametrize("bits", [2, 4, 8, 16])
@pytest.mark.parametrize("d", [8, 512, D_RAGGED])
def test_quantize_codes_bit_exact(gpu, bits, d):
    gen = np.random.Generator(np.random.PCG64(bits * 1000 + d))
    x = (gen.standard_normal(d) * 3).astype(np.float32)
    x[:: 7] *= -1
    if d > 100:
        x[5], x[6], x[17], x[18] = 0.0, -0.0, 1e-40, -1e-40
    for eps in (2.0 ** -5, 0.01):
        seed, node, event = 0x1234567890ABCDEF, 3, 77
        got = gpu.quantize(torch.from_numpy(x).cuda(), eps, bits, seed, node, event).cpu().numpy()
        want = qz.quantize(x, eps, bits, rng.sr_halves(seed, node, event, 0, d))
        assert np.array_equal(got, want), f"bits={bits} d={d} eps={eps}"


@pytest.mark.parametrize("bits", [2, 4, 8, 16])
def test_dequantize_against_key(gpu, bits):
    gen = np.random.Generator(np.random.PCG64(bits))
    d, eps = D_RAGGED, 2.0 ** -4
    x = models(gen, 1, d)[0]
    key = (x + gen.uniform(-1, 1, d) * eps * (1 << bits)).astype(np.float32)     # some inside, some outside the radius
    codes = qz.quantize(x, eps, bits, rng.sr_halves(1, 0, 0, 0, d))
    got = gpu.dequantize(torch.from_numpy(codes).cuda(), torch.from_numpy(key).cuda(), eps, bits).cpu().numpy()
    want = qz.dequantize(codes, key, eps, bits)
    assert np.array_equal(got.astype(np.float64), want)      # eps is a power of two: exact


def test_stateless_codec_rejects_misaligned_pointers(gpu):
    x = torch.zeros(64 + 4, dtype=torch.float32, device="cuda")
    codes = torch.zeros(64 + 8, dtype=torch.uint8, device="cuda")
    with pytest.raises(gpu.SwarmError):
        gpu.quantize(x[1:65], 1.0, 8, 0, 0, 0)                          # 4-byte aligned input
    with pytest.raises(gpu.SwarmError):
        gpu.dequantize(codes[1:65], x[:64], 1.0, 8)                     # odd code address
    with pytest.raises(gpu.SwarmError):
        gpu.dequantize(codes[:64], x[2:66], 1.0, 8)                     # 8-byte aligned key
    assert gpu.dequantize(codes[:64], x[4:68], 1.0, 8).shape == (64,)


def test_quantize_clamps_like_the_oracle(gpu):
    x = np.zeros(64, dtype=np.float32)
    x[3], x[9] = 3e9, -3e9
    eps = 1.0
    got = gpu.quantize(torch.from_numpy(x).cuda(), eps, 8, 0, 0, 0).cpu().numpy()
    assert np.array_equal(got, qz.quantize(x, eps, 8, rng.sr_halves(0, 0, 0, 0, 64)))


# ------------------------------------------------------------------ fused gossip pass
@pytest.mark.parametrize("bits", [2, 4, 8, 16])
def test_gossip_round_teacher_forced_fresh(gpu, bits):
    """Three rounds, fresh reads; local-step deltas absent / on every node / on some."""
    n, d, eps = 8, D_RAGGED, 2.0 ** -4
    edges = wl.complete_graph(n)
    g, c = make_both(gpu, n, d, edges, bits, eps, 0, 0.0, 0, seed=bits)
    gen = np.random.Generator(np.random.PCG64(bits))
    spread = {2: 0.01, 4: 0.1, 8: 1.0, 16: 3.0}[bits]
    for rnd, pend in enumerate([[], list(range(n)), [0, 3, 4, 6]]):
        base = models(gen, 1, d)
        c.X[:] = base + models(gen, n, d, spread)
        c.pending[:] = False
        for i in pend:
            c.W[i] = c.X[i] + models(gen, 1, d, 0.05)[0]
            c.pending[i] = True
        force_state(gpu, g, c)
        pairs = [(0, 5), (2, 3), (7, 1)]
        c.gossip_round(pairs)
        g.gossip_round(pairs)
        for i in range(n):
            assert np.array_equal(g.read_codes(i), ring_row(c, i)), f"codes of node {i}, round {rnd}"
        assert_close(g.read_models(gpu.COMM), c.X, TOL_ELEMENTWISE, f"X after round {rnd}")
    cnt = g.counters()
    assert cnt["rounds"] == 3 and cnt["interactions"] == 9
    assert cnt["bits_communicated"] == c.bits_communicated
    assert cnt["decode_failures"] == c.decode_failures


@pytest.mark.parametrize("bits", [4, 8])
def test_gossip_round_teacher_forced_stale(gpu, bits):
    """Ring of 3 slots; reads 0, 1 or 2 rounds old, uniform and mixed within a pair."""
    n, d, eps, S = 6, D_RAGGED, 2.0 ** -3, 2
    edges = wl.complete_graph(n)
    g, c = make_both(gpu, n, d, edges, bits, eps, 0, 0.0, S, seed=40 + bits)
    gen = np.random.Generator(np.random.PCG64(40 + bits))
    base = models(gen, 1, d)
    spread = 0.05 if bits == 4 else 1.0
    plans = [([(0, 1), (2, 3)], [0] * n), ([(0, 2), (1, 5)], [1] * n), ([(3, 4), (0, 5)], [2, 2, 2, 2, 2, 2]),
             ([(1, 2), (4, 5)], [0, 1, 2, 0, 0, 1]), ([(0, 3)], [2, 0, 0, 1, 0, 0]), ([(2, 5), (1, 4)], [1] * n)]
    for rnd, (pairs, stale) in enumerate(plans):
        c.X[:] = base + models(gen, n, d, spread)
        c.pending[:] = False
        for i in range(0, n, 2):
            c.W[i] = c.X[i] + models(gen, 1, d, 0.02)[0]
            c.pending[i] = True
        force_state(gpu, g, c)
        c.gossip_round(pairs, stale)
        g.gossip_round(pairs, stale)
        for i in range(n):
            for age in range(min(S, rnd) + 1):
                assert np.array_equal(g.read_codes(i, age=age), ring_row(c, i, age)), (rnd, i, age)
        assert_close(g.read_models(gpu.COMM), c.X, TOL_ELEMENTWISE, f"X after round {rnd}")
    assert g.counters()["decode_failures"] == c.decode_failures


def test_decode_failures_wrap_identically(gpu):
    """Rows farther apart than the radius: both sides land on the same wrong lattice point."""
    n, d, eps, bits = 4, 1024, 0.5, 4
    g, c = make_both(gpu, n, d, wl.complete_graph(n), bits, eps, 0, 0.0, 0, seed=1)
    gen = np.random.Generator(np.random.PCG64(1))
    c.X[:] = models(gen, n, d, 4.0)
    force_state(gpu, g, c)
    c.gossip_round([(0, 1), (2, 3)])
    g.gossip_round([(0, 1), (2, 3)])
    assert c.decode_failures > 0
    assert g.counters()["decode_failures"] == c.decode_failures
    assert_close(g.read_models(gpu.COMM), c.X, TOL_ELEMENTWISE, "wrapped averages")


def test_identity_quantizer_round_preserves_the_mean(gpu):
    n, d = 8, D_RAGGED
    g, c = make_both(gpu, n, d, wl.torus_graph(2, 4), 0, 0.0, 0, 0.0, 0)
    gen = np.random.Generator(np.random.PCG64(2))
    c.X[:] = models(gen, n, d)
    force_state(gpu, g, c)
    mean0 = c.X.astype(np.float64).mean(axis=0)
    pairs = [(0, 1), (2, 6), (3, 7)]
    c.gossip_round(pairs)
    g.gossip_round(pairs)
    X = g.read_models(gpu.COMM)
    assert_close(X, c.X, TOL_ELEMENTWISE, "plain averages")
    assert np.abs(X.astype(np.float64).mean(axis=0) - mean0).max() < 1e-6
    assert np.array_equal(X[0], X[1]) and np.array_equal(X[4], c.X[4])


@pytest.mark.parametrize("form", ["pairs, fresh reads", "nodes, stale reads", "prefix registers", "unmatched node"])
def test_range_clamp_is_reported(gpu, form):
    """|x / eps| beyond 2^29 is clamped and flagged by every kernel form, as in the oracle; the clamped
    codes and models still agree."""
    n, d = 3, 64
    prefix = form == "prefix registers"
    g, c = make_both(gpu, n, d, wl.complete_graph(n), 16 if prefix else 8, 2.0 ** -20, 0, 0.0, 1, prefix=prefix)
    c.X[:] = 0.001
    force_state(gpu, g, c)
    c.gossip_round([(0, 1)])
    g.gossip_round([(0, 1)])                                # round 0: gives round 1 something stale to read
    assert not c.range_clamped and g.counters()["rounds"] == 1
    c.X[:] = 0.001
    c.X[2 if form == "unmatched node" else 0, 5] = 1e6
    force_state(gpu, g, c)
    stale = [0, 0, 0] if form == "pairs, fresh reads" else [1, 1, 1]
    c.gossip_round([(0, 1)], stale)
    g.gossip_round([(0, 1)], stale)
    for i in range(n):
        assert np.array_equal(g.read_codes(i), ring_row(c, i))
    assert_close(g.read_models(gpu.COMM), c.X, TOL_ELEMENTWISE, form)
    assert c.range_clamped and g.counters(raise_on_range=False)["range_clamped"]
    with pytest.raises(gpu.SwarmError):
        g.counters()


@pytest.mark.parametrize("value", [np.nan, np.inf, -np.inf])
@pytest.mark.parametrize("form", ["pairs, fresh reads", "nodes, stale reads", "prefix registers", "unmatched node"])
def test_values_that_are_not_numbers_are_flagged(gpu, form, value):
    """A diverged coordinate (NaN, +-inf) is flagged like an overflow by every kernel form and sent as the
    same saturated code on both sides; it cannot reach a partner as a plausible finite value unnoticed."""
    n, d = 3, 64
    prefix = form == "prefix registers"
    g, c = make_both(gpu, n, d, wl.complete_graph(n), 16 if prefix else 8, 2.0 ** -4, 0, 0.0, 1, prefix=prefix)
    c.X[:] = 0.25
    force_state(gpu, g, c)
    c.gossip_round([(0, 1)])
    g.gossip_round([(0, 1)])
    assert not c.range_clamped and not g.counters()["range_clamped"]
    c.X[:] = 0.25
    c.X[2 if form == "unmatched node" else 0, 9] = value
    force_state(gpu, g, c)
    stale = [0, 0, 0] if form == "pairs, fresh reads" else [1, 1, 1]
    c.gossip_round([(0, 1)], stale)
    g.gossip_round([(0, 1)], stale)
    for i in range(n):
        assert np.array_equal(g.read_codes(i), ring_row(c, i))
    assert c.range_clamped and g.counters(raise_on_range=False)["range_clamped"]
    got = g.read_models(gpu.COMM)
    finite = np.isfinite(c.X)
    assert np.array_equal(np.isfinite(got), finite)
    assert_close(got[finite], c.X[finite], TOL_ELEMENTWISE, form)


# ------------------------------------------------------------------ local steps, diagonal quadratics
@pytest.mark.parametrize("sigma", [0.0, 0.1])
def test_local_steps_diag_quadratic(gpu, sigma):
    n, d, H, lr = 6, D_RAGGED, 3, 0.1
    a, cc = wl.diag_quadratic_data(n, d, 5)
    g, c = make_both(gpu, n, d, wl.complete_graph(n), 8, 2.0 ** -4, H, lr, 0, seed=9)
    c.objective = DiagQuadratic(a, cc, sigma)
    g.set_objective_diag(torch.from_numpy(a).cuda(), torch.from_numpy(cc).cuda(), sigma)
    gen = np.random.Generator(np.random.PCG64(3))
    c.X[:] = models(gen, n, d)
    force_state(gpu, g, c)
    c.local_steps()
    g.local_steps()
    assert_close(g.read_models(gpu.LIVE), c.W, TOL_ELEMENTWISE, "W after local steps")
    assert np.array_equal(g.read_models(gpu.COMM), c.X)            # not applied yet
    # the pending update reaches X through the gossip pass, and unmatched nodes apply their own
    pairs = [(0, 1), (2, 3)]
    c.gossip_round(pairs)
    g.gossip_round(pairs)
    assert_close(g.read_models(gpu.COMM), c.X, TOL_TWO_STAGE, "X after the round")
    # a subset of nodes, next round's random stream
    force_state(gpu, g, c)
    c.local_steps([4, 1])
    g.local_steps([4, 1])
    W = g.read_models(gpu.LIVE)
    assert_close(W[[4, 1]], c.W[[4, 1]], TOL_ELEMENTWISE, "W of the chosen nodes")


# ------------------------------------------------------------------ pair selection
@pytest.mark.parametrize("graph", ["torus", "regular4", "regular8", "complete"])
def test_matching_identical_to_oracle(gpu, graph):
    n, edges = {"torus": (64, wl.torus_graph(8, 8)), "regular4": (64, wl.random_regular_graph(64, 4, 2)),
                "regular8": (256, wl.random_regular_graph(256, 8, 3)), "complete": (33, wl.complete_graph(33))}[graph]
    g, c = make_both(gpu, n, 8, edges, 8, 1.0, 0, 0.0, 0, seed=123)
    for r in range(12):
        want = c.sample_matching()
        got = g.sample_matching()
        assert np.array_equal(got, want.astype(np.uint32)), f"round {r}"
        c.gossip_round(want)
        g.gossip_round(None)                   # samples the same matching internally
        assert g.counters()["interactions"] == c.interactions


def test_stale_and_pair_draws_identical_to_oracle(gpu):
    n = 32
    g, c = make_both(gpu, n, 8, wl.random_regular_graph(n, 4, 4), 8, 1.0, 0, 0.0, 2, seed=77)
    for r in range(6):
        assert np.array_equal(g.sample_stale(), c.sample_stale().astype(np.uint8))
        c.gossip_round([])
        g.gossip_round([])
    g2, c2 = make_both(gpu, n, 8, wl.random_regular_graph(n, 4, 4), 0, 0.0, 0, 0.0, 0, seed=78)
    for t in range(40):
        pair = c2.sample_pair()
        assert g2.sample_pair() == pair
        c2.interact(*pair)
        g2.interact(*pair)


# ------------------------------------------------------------------ reductions
def test_potential_mean_and_pair_linf(gpu):
    n, d = 12, D_RAGGED
    g, c = make_both(gpu, n, d, wl.complete_graph(n), 8, 1.0, 0, 0.0)
    gen = np.random.Generator(np.random.PCG64(8))
    c.X[:] = models(gen, n, d) + 100.0          # large common offset: the shifted sums must not cancel badly
    force_state(gpu, g, c)
    mu = torch.empty(d, dtype=torch.float32, device="cuda")
    gamma = g.potential(mu)
    assert gamma == pytest.approx(c.potential(), rel=1e-9)
    assert_close(mu.cpu().numpy(), c.mean(), TOL_ELEMENTWISE, "mean model")
    pairs = [(0, 1), (5, 2), (11, 7)]
    want = [np.abs(c.X[i] - c.X[j]).max() for i, j in pairs]
    assert np.array_equal(g.pair_linf(pairs), np.array(want, dtype=np.float32))


# ------------------------------------------------------------------ boundary errors
def test_boundary_rejects_bad_arguments(gpu):
    edges = wl.torus_graph(2, 4)
    with pytest.raises(gpu.SwarmError):
        gpu.Swarm(8, 12, edges, 8, 1.0, 0, 0.0)                       # d not a multiple of 8
    with pytest.raises(gpu.SwarmError):
        gpu.Swarm(8, 64, edges, 3, 1.0, 0, 0.0)                       # unsupported code width
    with pytest.raises(gpu.SwarmError):
        gpu.Swarm(8, 64, edges, 0, 1.0, 0, 0.0, stale_max=1)          # stale reads need codes
    with pytest.raises(gpu.SwarmError):
        gpu.Swarm(8, 64, [(0, 0)], 8, 1.0, 0, 0.0)                    # self loop
    g = gpu.Swarm(8, 64, edges, 8, 1.0, 1, 0.1, stale_max=1)
    for bad in ([(0, 5)], [(0, 1), (1, 2)], [(0, 9)]):                 # not an edge / node twice / out of range
        with pytest.raises(gpu.SwarmError) as err:
            g.gossip_round(bad)
        assert err.value.status == gpu.EINVAL
    with pytest.raises(gpu.SwarmError):
        g.gossip_round([(0, 1)], stale=[2] * 8)                        # beyond stale_max
    with pytest.raises(gpu.SwarmError) as err:
        g.local_steps()                                                # no objective set
    assert err.value.status == gpu.ESTATE
    with pytest.raises(gpu.SwarmError):
        g.interact(0, 1)                                               # Algorithm 1 needs stale_max = 0
    assert g.counters()["rounds"] == 0                                 # rejected calls change nothing
    g.gossip_round([])                                                 # an empty round is legal
    assert g.counters()["rounds"] == 1


# ------------------------------------------------------------------ Algorithm 1 with least-squares objectives
def test_algorithm1_least_squares_teacher_forced(gpu):
    """The sequential model on the small workload's shape: n=8, d=4096, 256x4096 least squares per
    node, batch 32, H=2, 8-bit codes; every step starts from the oracle's state."""
    from oracle.objectives import LeastSquares
    from helpers import TOL_GEMM
    n, d, m, batch, H, lr, bits, eps = 8, 4096, 256, 32, 2, 0.05, 8, 2.0 ** -6
    edges = wl.complete_graph(n)
    A, b, _ = wl.least_squares_data(n, d, m, 0)
    g, c = make_both(gpu, n, d, edges, bits, eps, H, lr, 0, seed=0)
    c.objective = LeastSquares(A, b, batch)
    g.set_objective_lsq(torch.from_numpy(A).cuda(), torch.from_numpy(b).cuda(), m, batch)
    for t in range(25):
        g.write_models(gpu.COMM, c.X)
        g.write_models(gpu.SNAP, c.Xhat)
        i, j = c.sample_pair()
        assert g.sample_pair() == (i, j)
        c.interact(i, j)
        g.interact(i, j)
        assert np.array_equal(g.read_codes(i), c.ring[0][i]) and np.array_equal(g.read_codes(j), c.ring[0][j])
        assert_close(g.read_models(gpu.LIVE, i, 1), c.W[i:i + 1], TOL_GEMM, f"W_i after local steps, t={t}")
        X = g.read_models(gpu.COMM)
        assert_close(X[j], c.X[j], TOL_ELEMENTWISE, f"responder model, t={t}")
        assert_close(X[i], c.X[i], TOL_GEMM, f"initiator model, t={t}")
        assert_close(g.read_models(gpu.SNAP), c.Xhat, TOL_GEMM, f"snapshots, t={t}")
        others = [k for k in range(n) if k not in (i, j)]
        assert np.array_equal(X[others], c.X[others])
    assert g.counters()["bits_communicated"] == c.bits_communicated


def test_algorithm1_free_running_matches_statistically(gpu):
    """200 sequential interactions without forcing: a last-bit difference can flip a rounding
    decision, so the runs are compared through the potential and the distance to the optimum."""
    from oracle.objectives import LeastSquares
    n, d, m, batch, H, lr, bits, eps = 8, 4096, 256, 32, 2, 0.05, 8, 2.0 ** -6
    edges = wl.complete_graph(n)
    A, b, xstar = wl.least_squares_data(n, d, m, 1)
    g, c = make_both(gpu, n, d, edges, bits, eps, H, lr, 0, seed=0)
    c.objective = LeastSquares(A, b, batch)
    g.set_objective_lsq(torch.from_numpy(A).cuda(), torch.from_numpy(b).cuda(), m, batch)
    for t in range(200):
        pair = c.sample_pair()
        assert g.sample_pair() == pair
        c.interact(*pair)
        g.interact(*pair)
    X = g.read_models(gpu.COMM).astype(np.float64)
    assert np.abs(X - c.X).max() <= 8 * eps
    assert (np.abs(X - c.X) > 1e-4).mean() < 0.05
    assert g.potential() == pytest.approx(c.potential(), rel=0.05)
    assert g.counters()["decode_failures"] == c.decode_failures == 0
    # both moved from 0 toward the least-squares solution's neighbourhood
    d0, d1 = np.linalg.norm(xstar), np.linalg.norm(X.mean(axis=0) - xstar)
    assert d1 < d0


@pytest.mark.parametrize("mode", ["fixed scale", "per-round scale, stale reads", "prefix registers, stale reads, one pass"])
def test_round_mode_free_running_matches_statistically(gpu, mode):
    """40 rounds on a torus with noisy diagonal quadratics, matching and staleness sampled on the device,
    nothing forced: the potential follows the oracle's to 2 %, the models stay within a few lattice
    steps, and the integer bookkeeping that does not depend on last-bit differences is equal."""
    n, d, H, lr, eps = 16, 8192, 3, 0.1, 2.0 ** -4
    edges = wl.torus_graph(4, 4)
    a, cc = wl.diag_quadratic_data(n, d, 2)
    bits, S = (16, 2) if mode.startswith("prefix") else (8, 2 if "stale" in mode else 0)
    g, c = make_both(gpu, n, d, edges, bits, eps, H, lr, S, seed=3, global_scale=mode.startswith("per-round"),
                     prefix=mode.startswith("prefix"))
    c.objective = DiagQuadratic(a, cc, 0.1)
    g.set_objective_diag(torch.from_numpy(a).cuda(), torch.from_numpy(cc).cuda(), 0.1)
    gam_g, gam_c = [], []
    for r in range(40):
        stale = c.sample_stale() if S else None
        c.local_steps()
        c.gossip_round(c.sample_matching(), stale)
        if mode.endswith("one pass"):
            g.round_fused(None, None if stale is None else g.sample_stale())
        else:
            g.local_steps()
            g.gossip_round(None, None if stale is None else g.sample_stale())
        gam_g.append(g.potential())
        gam_c.append(c.potential())
    assert np.allclose(gam_g, gam_c, rtol=0.02)
    assert g.counters()["interactions"] == c.interactions
    X = g.read_models(gpu.COMM).astype(np.float64)
    assert np.abs(X - c.X).max() <= 8 * max(eps, float(c.eps_cur))
    if mode.startswith("per-round"):
        assert g.scale()[0] == float(c.eps_cur)              # a power of two: robust to last-bit differences
    if mode.startswith("prefix"):
        tiles, unconfirmed = g.prefix_stats()
        assert unconfirmed == 0 == c.prefix_unconfirmed and sum(tiles) == int(c.prefix_levels.sum())
        assert abs(tiles[0] - int(c.prefix_levels[0])) <= 0.02 * sum(tiles)


# ------------------------------------------------------------------ MLP local steps (MFMA GEMMs)
@pytest.mark.parametrize("arithmetic", ["float32", "three bf16 products"])
# the last shape has a batch taller than one 128-row tile: ragged second tile row, ten K slabs in the update GEMMs,
# and the hidden-layer bias updated by its own kernel instead of inside the backward GEMM
@pytest.mark.parametrize("shape", [(64, 96, 32, 32), (256, 384, 128, 128), (64, 96, 32, 160)])
def test_local_steps_mlp(gpu, shape, arithmetic):
    """Two local steps of the two-layer perceptron on the Gaussian mixture: data generation,
    forward, softmax-CE gradient, backward GEMMs and fused SGD updates against the float64 oracle."""
    from oracle.objectives import MixtureMLP
    from helpers import TOL_GEMM
    n_in, n_hid, n_out, batch = shape
    n, H, lr = 5, 2, 0.02
    d = n_hid * n_in + n_hid + n_out * n_hid + n_out
    means, cdf = wl.mixture_data(n, n_in, n_out, 3)
    g, c = make_both(gpu, n, d, wl.complete_graph(n), 8, 2.0 ** -8, H, lr, 0, seed=21)
    c.objective = MixtureMLP(n_in, n_hid, n_out, means, cdf, 0.5, batch)
    g.set_objective_mlp(n_in, n_hid, n_out, torch.from_numpy(means).cuda(), torch.from_numpy(cdf).cuda(), 0.5, batch)
    if arithmetic != "float32":
        g.set_mlp_arithmetic(gpu.MLP_BF16X3)
    gen = np.random.Generator(np.random.PCG64(5))
    c.X[:] = models(gen, n, d, 0.1)
    force_state(gpu, g, c)
    c.local_steps()
    g.local_steps()
    W = g.read_models(gpu.LIVE)
    assert_close(W, c.W, TOL_GEMM, "weights after two local steps")
    # the summed gradient itself: -(W - X) / eta
    grad_gpu = (c.X.astype(np.float64) - W) / lr
    grad_cpu = (c.X.astype(np.float64) - c.W) / lr
    assert_close(grad_gpu, grad_cpu, TOL_GEMM, "summed stochastic gradient")
    assert np.abs(grad_cpu).max() > 1e-3                                   # the comparison is not vacuous
    # subset of nodes, then a gossip round on top
    force_state(gpu, g, c)
    c.local_steps([3, 0])
    g.local_steps([3, 0])
    assert_close(g.read_models(gpu.LIVE)[[3, 0]], c.W[[3, 0]], TOL_GEMM, "subset")
    pairs = [(0, 3), (1, 2)]
    c.gossip_round(pairs)
    g.gossip_round(pairs)
    assert_close(g.read_models(gpu.COMM), c.X, TOL_GEMM, "models after the round")


# ------------------------------------------------------------------ in-place apply mode
@pytest.mark.parametrize("registers", ["fixed", "per-round scale", "prefix"])
def test_inplace_apply_mode_rounds(gpu, registers):
    """One matrix: the local steps update the exchanged model, the averaging acts on the result."""
    n, d, H, lr, bits, eps, S = 8, D_RAGGED, 3, 0.1, 16 if registers == "prefix" else 8, 2.0 ** -4, 1
    edges = wl.torus_graph(2, 4)
    a, cc = wl.diag_quadratic_data(n, d, 7)
    g, c = make_both(gpu, n, d, edges, bits, eps, H, lr, S, seed=31, inplace=True,
                     global_scale=registers == "per-round scale", prefix=registers == "prefix")
    c.objective = DiagQuadratic(a, cc, 0.05)
    g.set_objective_diag(torch.from_numpy(a).cuda(), torch.from_numpy(cc).cuda(), 0.05)
    gen = np.random.Generator(np.random.PCG64(31))
    c.X[:] = models(gen, n, d)
    for r in range(4):
        g.write_models(gpu.COMM, c.X)
        c.local_steps()
        g.local_steps()
        assert_close(g.read_models(gpu.COMM), c.X, TOL_ELEMENTWISE, f"X after local steps, round {r}")
        g.write_models(gpu.COMM, c.X)                      # same input to the gossip pass on both sides
        pairs = c.sample_matching()
        stale = [min(r, 1)] * n
        c.gossip_round(pairs, stale)
        g.gossip_round(None, stale)
        for i in range(n):
            assert np.array_equal(g.read_codes(i), ring_row(c, i)), (r, i)
        assert_close(g.read_models(gpu.COMM), c.X, TOL_ELEMENTWISE, f"X after round {r}")
        if registers == "per-round scale":
            assert g.scale() == (float(c.eps_cur), float(c.max_disagreement))
        if registers == "prefix":
            assert g.prefix_stats() == (c.prefix_levels.tolist(), c.prefix_unconfirmed)
    with pytest.raises(gpu.SwarmError):
        g.interact(0, 1)


# ------------------------------------------------------------------ fused round (local steps inside the gossip pass)
@pytest.mark.parametrize("inplace", [False, True])
@pytest.mark.parametrize("bits,S", [(4, 1), (8, 2)])
def test_fused_round_equals_two_calls_and_oracle(gpu, inplace, bits, S):
    n, d, H, lr, eps, sigma = 10, D_RAGGED, 3, 0.1, 2.0 ** -3, 0.05
    edges = wl.random_regular_graph(n, 3, 1)
    a, cc = wl.diag_quadratic_data(n, d, 11)
    ad, cd = torch.from_numpy(a).cuda(), torch.from_numpy(cc).cuda()
    fused, c = make_both(gpu, n, d, edges, bits, eps, H, lr, S, seed=17, inplace=inplace)
    split, _ = make_both(gpu, n, d, edges, bits, eps, H, lr, S, seed=17, inplace=inplace)
    c.objective = DiagQuadratic(a, cc, sigma)
    fused.set_objective_diag(ad, cd, sigma)
    split.set_objective_diag(ad, cd, sigma)
    gen = np.random.Generator(np.random.PCG64(17))
    c.X[:] = models(gen, n, d, 0.3)
    for r in range(5):
        fused.write_models(gpu.COMM, c.X)
        split.write_models(gpu.COMM, c.X)
        pairs = c.sample_matching()
        stale = fused.sample_stale()
        assert np.array_equal(stale, c.sample_stale().astype(np.uint8))
        c.local_steps()
        c.gossip_round(pairs, stale)
        split.local_steps()
        split.gossip_round(None, stale)
        fused.round_fused(None, stale)
        Xf, Xs = fused.read_models(gpu.COMM), split.read_models(gpu.COMM)
        assert np.array_equal(Xf, Xs), f"fused and two-call rounds differ, round {r}"
        for i in range(n):
            assert np.array_equal(fused.read_codes(i), ring_row(c, i)), (r, i)
        assert_close(Xf, c.X, TOL_TWO_STAGE, f"X after fused round {r}")
    assert fused.counters() == split.counters()
    fused.local_steps()
    if not inplace:
        with pytest.raises(gpu.SwarmError) as err:
            fused.round_fused(None)                        # steps already pending
        assert err.value.status == gpu.ESTATE


# ------------------------------------------------------------------ geometric number of local steps
def test_geometric_local_steps(gpu):
    """H_i drawn per node and interaction: identical draws on both sides, used by the stand-alone
    local steps, by the one-pass round and by Algorithm 1's initiator."""
    n, d, H, lr, bits, eps = 12, D_RAGGED, 3, 0.05, 8, 2.0 ** -4
    edges = wl.random_regular_graph(n, 3, 2)
    a, cc = wl.diag_quadratic_data(n, d, 13)
    ad, cd = torch.from_numpy(a).cuda(), torch.from_numpy(cc).cuda()
    g, c = make_both(gpu, n, d, edges, bits, eps, H, lr, 0, seed=23, geometric=True)
    f, _ = make_both(gpu, n, d, edges, bits, eps, H, lr, 0, seed=23, geometric=True)
    c.objective = DiagQuadratic(a, cc, 0.02)
    g.set_objective_diag(ad, cd, 0.02)
    f.set_objective_diag(ad, cd, 0.02)
    gen = np.random.Generator(np.random.PCG64(23))
    c.X[:] = models(gen, n, d, 0.5)
    seen = set()
    for r in range(4):
        g.write_models(gpu.COMM, c.X)
        f.write_models(gpu.COMM, c.X)
        steps = g.sample_steps()
        assert np.array_equal(steps, c.sample_steps().astype(np.uint8))
        seen |= set(steps.tolist())
        pairs = c.sample_matching()
        c.local_steps()
        g.local_steps()
        assert_close(g.read_models(gpu.LIVE), c.W, TOL_ELEMENTWISE, f"W, round {r}")
        c.gossip_round(pairs)
        g.gossip_round(None)
        f.round_fused(None)
        assert np.array_equal(f.read_models(gpu.COMM), g.read_models(gpu.COMM))
        assert_close(g.read_models(gpu.COMM), c.X, TOL_TWO_STAGE, f"X, round {r}")
    assert len(seen) > 1
    # sequential model: the initiator's H_i is drawn for the interaction number
    g2, c2 = make_both(gpu, n, d, edges, bits, eps, H, lr, 0, seed=29, geometric=True)
    c2.objective = DiagQuadratic(a, cc, 0.0)
    g2.set_objective_diag(ad, cd, 0.0)
    c2.X[:] = models(gen, n, d, 0.5)
    c2.Xhat[:] = c2.X
    g2.write_models(gpu.COMM, c2.X)
    g2.write_models(gpu.SNAP, c2.Xhat)
    for t in range(6):
        pair = c2.sample_pair()
        c2.interact(*pair)
        g2.interact(*pair)
        g2.write_models(gpu.COMM, c2.X)
        g2.write_models(gpu.SNAP, c2.Xhat)
        assert_close(g2.read_models(gpu.LIVE, pair[0], 1), c2.W[pair[0]:pair[0] + 1], TOL_ELEMENTWISE, f"W_i, t={t}")


# ------------------------------------------------------------------ per-pair lattice scale
@pytest.mark.parametrize("bits", [4, 8])
def test_pair_linf_scale_policy(gpu, bits):
    """Each matched pair quantizes at the smallest power-of-two scale that keeps it inside the decoding
    radius: codes and models match the oracle, and no decode ever fails however far apart the rows are."""
    n, d, H, lr = 8, D_RAGGED, 2, 0.1
    edges = wl.complete_graph(n)
    a, cc = wl.diag_quadratic_data(n, d, 3, shift_sigma=2.0)
    g, c = make_both(gpu, n, d, edges, bits, 1.0, H, lr, 0, seed=41, pair_scale=True)
    c.objective = DiagQuadratic(a, cc, 0.05)
    g.set_objective_diag(torch.from_numpy(a).cuda(), torch.from_numpy(cc).cuda(), 0.05)
    gen = np.random.Generator(np.random.PCG64(41))
    for r, spread in enumerate([1e-3, 0.3, 5.0, 40.0]):
        c.X[:] = models(gen, 1, d) + models(gen, n, d, spread)
        c.pending[:] = False
        force_state(gpu, g, c)
        c.local_steps([0, 1, 2, 5])
        g.local_steps([0, 1, 2, 5])
        force_state(gpu, g, c)
        pairs = [(0, 4), (6, 1), (2, 3)]                       # 5 and 7 unmatched; 5 has pending steps
        want = [np.abs(c.X[i] - c.X[j]).max() for i, j in pairs]
        assert np.array_equal(g.pair_linf(pairs), np.array(want, dtype=np.float32))
        c.gossip_round(pairs)
        g.gossip_round(pairs)
        for i in (0, 4, 6, 1, 2, 3):
            assert np.array_equal(g.read_codes(i), c.ring[0][i]), (r, i)
        assert_close(g.read_models(gpu.COMM), c.X, TOL_ELEMENTWISE, f"X after round {r}")
    assert c.decode_failures == 0 and g.counters()["decode_failures"] == 0
    with pytest.raises(gpu.SwarmError):
        g.round_fused(None)
    with pytest.raises(gpu.SwarmError):
        gpu.Swarm(n, d, edges, 2, 1.0, H, lr, 0, 0, scale_policy=gpu.SCALE_PAIR_LINF)


# ------------------------------------------------------------------ edge cases and limits
@pytest.mark.parametrize("case", ["complete64", "ring1500", "regular3_2000", "star"])
def test_matching_large_graphs(gpu, case):
    """More edges and more nodes than the matching workgroup has threads; a star (every edge shares
    one node, exactly one pair) as the degenerate case."""
    if case == "complete64":
        n, edges = 64, wl.complete_graph(64)                       # 2016 edges
    elif case == "ring1500":
        n = 1500
        edges = np.array([(i, (i + 1) % n) for i in range(n)], dtype=np.uint32)
    elif case == "regular3_2000":
        n, edges = 2000, wl.random_regular_graph(2000, 3, 9)       # 3000 edges
    else:
        n = 300
        edges = np.array([(0, i) for i in range(1, n)], dtype=np.uint32)
    g, c = make_both(gpu, n, 8, edges, 8, 1.0, 0, 0.0, 0, seed=5)
    for r in range(4):
        want = c.sample_matching()
        assert np.array_equal(g.sample_matching(), want.astype(np.uint32)), (case, r)
        c.gossip_round(want)
        g.gossip_round(None)
    if case == "star":
        assert len(want) == 1
    assert g.counters()["interactions"] == c.interactions


def test_largest_swarm_and_one_node_more(gpu):
    """n = 4096, the most the boundary takes (the matching of a round runs in one workgroup), on a random
    4-regular graph: matching, codes and models of a one-pass round against the oracle; n = 4097 is refused."""
    n, d, H, lr, bits, eps = 4096, 16, 2, 0.1, 8, 2.0 ** -4
    edges = wl.random_regular_graph(n, 4, 21)
    a, cc = wl.diag_quadratic_data(n, d, 13, shift_sigma=0.2)
    g, c = make_both(gpu, n, d, edges, bits, eps, H, lr, 1, seed=99)
    c.objective = DiagQuadratic(a, cc, 0.05)
    g.set_objective_diag(torch.from_numpy(a).cuda(), torch.from_numpy(cc).cuda(), 0.05)
    gen = np.random.Generator(np.random.PCG64(99))
    for r in range(2):
        c.X[:] = models(gen, 1, d) + models(gen, n, d, 0.05)
        c.pending[:] = False
        force_state(gpu, g, c)
        pairs, stale = c.sample_matching(), c.sample_stale()
        assert np.array_equal(g.sample_matching(), pairs.astype(np.uint32)) and len(pairs) > 1500
        c.local_steps()
        c.gossip_round(pairs, stale)
        g.round_fused(None, stale.astype(np.uint8))
        for i in (0, 1, n // 2, n - 2, n - 1):
            assert np.array_equal(g.read_codes(i), ring_row(c, i)), f"register of node {i}, round {r}"
        assert_close(g.read_models(gpu.COMM), c.X, TOL_TWO_STAGE, f"X after round {r}")
    assert g.counters()["interactions"] == c.interactions
    ring = np.array([(i, (i + 1) % (n + 1)) for i in range(n + 1)], dtype=np.uint32)
    with pytest.raises(gpu.SwarmError) as err:
        gpu.Swarm(n + 1, d, ring, bits, eps, H, lr, 1, 99)
    assert "EINVAL" in str(err.value)


def test_smallest_swarm_and_empty_rounds(gpu):
    """n = 2, d = 8 (one Philox call per row), rounds with no pair, H = 0."""
    g, c = make_both(gpu, 2, 8, [(0, 1)], 8, 0.25, 0, 0.0, 1, seed=1)
    c.X[:] = np.array([[0.1, -0.2, 0.3, 5.0, -5.0, 0.0, 1.0, 2.0], [0.2, -0.1, 0.1, 4.0, -4.5, 0.5, 1.5, 2.5]], dtype=np.float32)
    force_state(gpu, g, c)
    for pairs, stale in [([], None), ([(1, 0)], [1, 1]), ([(0, 1)], [1, 0])]:
        c.gossip_round(pairs, stale)
        g.gossip_round(pairs, stale)
        assert np.array_equal(g.read_codes(0), ring_row(c, 0)) and np.array_equal(g.read_codes(1), ring_row(c, 1))
        assert_close(g.read_models(gpu.COMM), c.X, TOL_ELEMENTWISE, "two-node swarm")
    with pytest.raises(gpu.SwarmError):
        g.local_steps()                                   # no objective set
    a, cc = wl.diag_quadratic_data(2, 8, 0)
    g.set_objective_diag(torch.from_numpy(a).cuda(), torch.from_numpy(cc).cuda(), 0.0)
    g.local_steps()                                       # H = 0: nothing becomes pending
    before = g.read_models(gpu.COMM)
    g.gossip_round([])
    assert np.array_equal(g.read_models(gpu.COMM), before) and g.counters()["rounds"] == 4


def test_windows_of_models_and_codes(gpu):
    n, d, bits = 5, 4096, 4
    g, c = make_both(gpu, n, d, wl.complete_graph(n), bits, 0.5, 0, 0.0)
    gen = np.random.Generator(np.random.PCG64(3))
    c.X[:] = models(gen, n, d)
    force_state(gpu, g, c)
    patch = models(gen, 2, 100)
    g.write_models(gpu.COMM, patch, node0=2, k0=1000)
    c.X[2:4, 1000:1100] = patch
    assert np.array_equal(g.read_models(gpu.COMM), c.X)
    assert np.array_equal(g.read_models(gpu.COMM, node0=3, count=2, k0=8, length=24), c.X[3:5, 8:32])
    c.gossip_round([(0, 1)])
    g.gossip_round([(0, 1)])
    assert np.array_equal(g.read_codes(2, byte0=16, length=64), ring_row(c, 2)[16:80])
    for bad in (dict(node0=4, count=2), dict(k0=4090, length=10), dict(count=0)):
        with pytest.raises(gpu.SwarmError):
            g.read_models(gpu.COMM, **bad)
    with pytest.raises(gpu.SwarmError):
        g.read_codes(0, age=1)                           # deeper than the ring
    view = g.models_view(gpu.COMM)
    assert view.shape == (n, d) and np.array_equal(view.cpu().numpy(), g.read_models(gpu.COMM))


def test_deep_stale_ring(gpu):
    """Ring of 6 slots with reads up to 5 rounds old, staleness drawn from the STALE stream."""
    n, d, bits, eps, S = 6, 2048 + 8, 8, 2.0 ** -3, 5
    g, c = make_both(gpu, n, d, wl.complete_graph(n), bits, eps, 0, 0.0, S, seed=77)
    gen = np.random.Generator(np.random.PCG64(77))
    base = models(gen, 1, d)
    for r in range(9):
        c.X[:] = base + models(gen, n, d, 0.5)
        force_state(gpu, g, c)
        stale = g.sample_stale()
        assert np.array_equal(stale, c.sample_stale().astype(np.uint8)) and stale.max() <= min(r, S)
        pairs = c.sample_matching()
        c.gossip_round(pairs, stale)
        g.gossip_round(None, stale)
        for i in range(n):
            assert np.array_equal(g.read_codes(i), ring_row(c, i)), (r, i)
        assert_close(g.read_models(gpu.COMM), c.X, TOL_ELEMENTWISE, f"round {r}")
    assert g.counters()["decode_failures"] == c.decode_failures


@pytest.mark.parametrize("bits", [0, 2, 4, 16])
def test_algorithm1_all_code_widths_and_decode_failure(gpu, bits):
    """Sequential steps with diagonal objectives for every code width; some rows are placed farther
    apart than the decoding radius so that the initiator averages with a wrapped value."""
    n, d, H, lr, eps = 6, 8 * 300 + 8, 2, 0.1, 0.25
    edges = wl.complete_graph(n)
    a, cc = wl.diag_quadratic_data(n, d, 4)
    g, c = make_both(gpu, n, d, edges, bits, eps if bits else 0.0, H, lr, 0, seed=61)
    c.objective = DiagQuadratic(a, cc, 0.05)
    g.set_objective_diag(torch.from_numpy(a).cuda(), torch.from_numpy(cc).cuda(), 0.05)
    gen = np.random.Generator(np.random.PCG64(61))
    c.X[:] = models(gen, n, d, 0.1)
    c.X[3] += 5.0                                         # far from everyone: beyond the 2- and 4-bit radius
    c.Xhat[:] = c.X + models(gen, n, d, 0.05)
    for t, (i, j) in enumerate([(0, 1), (3, 2), (4, 3), (1, 0), (5, 3)]):
        g.write_models(gpu.COMM, c.X)
        g.write_models(gpu.SNAP, c.Xhat)
        c.interact(i, j)
        g.interact(i, j)
        if bits:
            assert np.array_equal(g.read_codes(i), c.ring[0][i]) and np.array_equal(g.read_codes(j), c.ring[0][j])
        assert_close(g.read_models(gpu.COMM), c.X, TOL_TWO_STAGE, f"X, t={t}")
        assert_close(g.read_models(gpu.SNAP), c.Xhat, TOL_TWO_STAGE, f"snapshots, t={t}")
    cnt = g.counters()
    assert cnt["decode_failures"] == c.decode_failures and cnt["interactions"] == 5
    if bits in (2, 4):
        assert c.decode_failures > 0


def test_copy_measurement_aids(gpu):
    """The copy kernels the bandwidth figures are compared with move what they claim: stream_copy is a
    copy; stream_mix sums its read streams (float32, in order) into every write stream, plus the
    stream's number; an unsupported shape is an error, not a launch."""
    gen = np.random.Generator(np.random.PCG64(5))
    m = 4 * 1000 + 4                                       # floats per stream: several workgroups and a tail
    src = gen.standard_normal(6 * m).astype(np.float32)
    s = torch.from_numpy(src).cuda()
    out = torch.zeros(2 * m, dtype=torch.float32, device="cuda")
    gpu.stream_copy(out, s[:2 * m])
    assert np.array_equal(out.cpu().numpy(), src[:2 * m])
    for n_read, n_write in [(2, 1), (3, 1), (2, 2), (4, 2), (6, 2)]:
        out.zero_()
        gpu.stream_mix(out, s, 4 * m, n_read, n_write)
        want = np.zeros(m, dtype=np.float32)
        for r in range(n_read):
            want = want + src[r * m:(r + 1) * m]
        got = out.cpu().numpy()
        for w in range(n_write):
            assert np.array_equal(got[w * m:(w + 1) * m], want + np.float32(w)), (n_read, n_write, w)
        assert not got[n_write * m:].any()
    with pytest.raises(gpu.SwarmError):
        gpu.stream_mix(out, s, 4 * m, 5, 1)


# ------------------------------------------------------------------ one lattice scale per round
@pytest.mark.parametrize("fused", [False, True])
@pytest.mark.parametrize("bits", [8, 16])
def test_global_linf_scale_policy(gpu, bits, fused):
    """The scale follows the disagreement the previous round saw: too small at first (decodes wrap, the
    scale grows), then tracking a spread that shrinks and widens again, with reads up to two rounds
    old decoded at the scale they were written with.  Codes, the scale and the disagreement match the
    oracle exactly in every round, models to the elementwise tolerance."""
    n, d, H, lr, S = 10, D_RAGGED, 2, 0.1, 2
    edges = wl.complete_graph(n)
    a, cc = wl.diag_quadratic_data(n, d, 3, shift_sigma=0.2)
    g, c = make_both(gpu, n, d, edges, bits, 2.0 ** -12, H, lr, S, seed=77, global_scale=True)
    c.objective = DiagQuadratic(a, cc, 0.05)
    g.set_objective_diag(torch.from_numpy(a).cuda(), torch.from_numpy(cc).cuda(), 0.05)
    gen = np.random.Generator(np.random.PCG64(77 + bits))
    assert g.scale() == (2.0 ** -12, 0.0)
    matchings = [[(0, 4), (6, 1), (2, 3), (8, 9)], [(1, 2), (3, 4), (5, 6)], [], [(0, 9), (7, 1), (2, 8)],
                 [(0, 1), (2, 3), (4, 5), (6, 7), (8, 9)], [(9, 1), (2, 7)], [(0, 5), (3, 6), (4, 8)], [(1, 5), (2, 6)],
                 [(0, 2), (1, 3), (4, 6), (5, 7)], [(0, 3), (1, 2), (8, 5)], [(0, 4), (6, 1), (2, 3), (8, 9)],
                 [(1, 2), (3, 4), (5, 6)], [(0, 9), (7, 1), (2, 8)], [(0, 3), (1, 2), (8, 5)]]
    rounds = list(zip([0.02] * 6 + [0.0005] * 5 + [0.3] * 3, matchings))
    base = models(gen, 1, d)                               # the models stay near one point: stale codes stay meaningful
    scales = []
    for r, (spread, pairs) in enumerate(rounds):
        c.X[:] = base + models(gen, n, d, spread)
        c.pending[:] = False
        force_state(gpu, g, c)
        stale = np.minimum(gen.integers(0, S + 1, n), r).astype(np.uint8)
        if fused:
            c.local_steps()
            c.gossip_round(pairs, stale)
            g.round_fused(pairs, stale)
        else:
            c.local_steps([0, 1, 2, 5])
            g.local_steps([0, 1, 2, 5])
            force_state(gpu, g, c)
            c.gossip_round(pairs, stale)
            g.gossip_round(pairs, stale)
        for i in range(n):
            assert np.array_equal(g.read_codes(i), ring_row(c, i)), f"codes of node {i}, round {r}"
        assert g.scale() == (float(c.eps_cur), float(c.max_disagreement)), f"scale after round {r}"
        assert_close(g.read_models(gpu.COMM), c.X, TOL_TWO_STAGE, f"X after round {r}")
        assert g.counters()["decode_failures"] == c.decode_failures
        scales.append(float(c.eps_cur))
    assert scales[2] == scales[1]                                      # nobody matched
    if bits == 8:
        assert scales[0] == 2.0 ** -10 and c.decode_failures > 0       # wrapped decodes: fourfold growth
        assert scales[10] < scales[5] and scales[13] >= 8 * scales[10]  # follows the spread down and up again
    else:
        assert scales[0] == 2.0 ** -13 and scales[10] < scales[5]       # 16 bits reach at first: the scale refines
    with pytest.raises(gpu.SwarmError):
        g.interact(0, 1)
    with pytest.raises(gpu.SwarmError):
        gpu.Swarm(n, d, edges, bits, 0.3, H, lr, 0, 0, scale_policy=gpu.SCALE_GLOBAL_LINF)   # not a power of two
    with pytest.raises(gpu.SwarmError):
        gpu.Swarm(n, d, edges, 4, 0.25, H, lr, 0, 0, scale_policy=gpu.SCALE_GLOBAL_LINF)     # too few bits


# ------------------------------------------------------------------ multi-resolution registers
@pytest.mark.parametrize("fused", [False, True])
def test_prefix_codec_rounds(gpu, fused):
    """Registers hold 16 bits per coordinate in three planes plus tile checksums; readers fetch the
    shortest confirmed prefix.  The models drift by tens of lattice cells per round, so stale reads
    escalate to 8 bits; one node sits hundreds of cells away (16 bits) and in one round one coordinate is
    beyond even that (a tile nobody can confirm).  Register images, levels, unconfirmed tiles, bits read
    and decode failures equal the oracle's; models to the elementwise tolerance."""
    n, d, H, lr, S, eps = 10, D_RAGGED, 2, 0.1, 2, 2.0 ** -5
    edges = wl.complete_graph(n)
    a, cc = wl.diag_quadratic_data(n, d, 3, shift_sigma=0.2)
    g, c = make_both(gpu, n, d, edges, 16, eps, H, lr, S, seed=91, prefix=True)
    c.objective = DiagQuadratic(a, cc, 0.05)
    g.set_objective_diag(torch.from_numpy(a).cuda(), torch.from_numpy(cc).cuda(), 0.05)
    gen = np.random.Generator(np.random.PCG64(91))
    base = models(gen, 1, d)
    matchings = [[(0, 4), (6, 1), (2, 3), (8, 9)], [(1, 2), (3, 4), (5, 6)], [], [(0, 9), (7, 1), (2, 8)],
                 [(0, 1), (2, 3), (4, 5), (6, 7), (8, 9)], [(9, 1), (2, 7)]]
    stales = [np.zeros(n), np.ones(n), np.ones(n), np.array([2, 0, 1, 2, 0, 1, 2, 0, 1, 2]),
              np.array([0, 0, 1, 1, 2, 0, 0, 2, 1, 0]), np.full(n, 2)]
    for r, (pairs, stale) in enumerate(zip(matchings, stales)):
        c.X[:] = base + 0.4 * r + models(gen, n, d, 0.02)          # 12.8 cells per round
        c.X[9] += 20.0                                             # 640 cells from everyone: needs 16 bits
        if r == 3:
            c.X[7, 1000] += 3000.0                                 # 96000 cells: beyond the 16-bit radius
        c.pending[:] = False
        force_state(gpu, g, c)
        stale = np.minimum(stale, r).astype(np.uint8)
        if fused:
            c.local_steps()
            c.gossip_round(pairs, stale)
            g.round_fused(pairs, stale)
        else:
            c.local_steps([0, 1, 2, 5])
            g.local_steps([0, 1, 2, 5])
            force_state(gpu, g, c)
            c.gossip_round(pairs, stale)
            g.gossip_round(pairs, stale)
        for i in range(n):
            assert np.array_equal(g.read_codes(i), ring_row(c, i)), f"register of node {i}, round {r}"
        assert_close(g.read_models(gpu.COMM), c.X, TOL_TWO_STAGE, f"X after round {r}")
        tiles, unconfirmed = g.prefix_stats()
        assert tiles == c.prefix_levels.tolist() and unconfirmed == c.prefix_unconfirmed, f"levels after round {r}"
        cnt = g.counters()
        assert cnt["decode_failures"] == c.decode_failures and cnt["bits_communicated"] == c.bits_communicated
    assert c.prefix_levels[1] > 0 and c.prefix_levels[2] > 0 and c.prefix_unconfirmed > 0
    with pytest.raises(gpu.SwarmError):
        g.interact(0, 1)
    with pytest.raises(gpu.SwarmError):
        gpu.Swarm(n, d, edges, 8, eps, H, lr, 0, 0, codec=gpu.CODEC_PREFIX)


def test_local_steps_computed_by_the_caller(gpu):
    """Gradients from outside the library: the caller writes W = X - eta * (its own gradients) into the
    live matrix on the device and declares the steps pending; the round treats them like its own."""
    n, d, bits, eps, S = 6, D_RAGGED, 8, 2.0 ** -5, 1
    edges = wl.complete_graph(n)
    g, c = make_both(gpu, n, d, edges, bits, eps, 0, 0.0, S, seed=13)
    gen = np.random.Generator(np.random.PCG64(13))
    for r, (nodes, pairs) in enumerate([([0, 2, 3], [(0, 1), (2, 5)]), (None, [(4, 0), (1, 3)]), ([5], [])]):
        c.X[:] = models(gen, 1, d) + models(gen, n, d, 0.05)
        c.pending[:] = False
        force_state(gpu, g, c)
        live = g.models_view(gpu.LIVE)
        ids = list(range(n)) if nodes is None else nodes
        for i in ids:                                             # a gradient step of the caller's own making
            step = models(gen, 1, d, 0.01)[0]
            c.W[i] = c.X[i] - step
            c.pending[i] = True
            live[i].copy_(torch.from_numpy(c.W[i]).cuda())
        g.mark_pending(nodes)
        stale = np.minimum(1, r) * np.ones(n, dtype=np.uint8)
        c.gossip_round(pairs, stale)
        g.gossip_round(pairs, stale)
        for i in range(n):
            assert np.array_equal(g.read_codes(i), ring_row(c, i))
        assert_close(g.read_models(gpu.COMM), c.X, TOL_ELEMENTWISE, f"X after round {r}")
    with pytest.raises(gpu.SwarmError):
        g.mark_pending([0, 0])
    with pytest.raises(gpu.SwarmError):
        gpu.Swarm(n, d, edges, bits, eps, 0, 0.0, 0, 0, apply_mode=gpu.INPLACE).mark_pending()


@pytest.mark.parametrize("kind", ["prefix", "global"])
def test_smallest_swarm_with_prefix_registers_and_per_round_scale(gpu, kind):
    """n = 2, d = 8: a row shorter than one lane group, one checksum tile of 8 coordinates; an empty
    round, stale and mixed reads."""
    bits = 16 if kind == "prefix" else 8
    g, c = make_both(gpu, 2, 8, [(0, 1)], bits, 0.25, 0, 0.0, 1, seed=1, prefix=kind == "prefix",
                     global_scale=kind == "global")
    X = np.array([[0.1, -0.2, 0.3, 5.0, -5.0, 0.0, 1.0, 2.0], [0.2, -0.1, 0.1, 4.0, -4.5, 0.5, 1.5, 30.0]], dtype=np.float32)
    for r, (pairs, stale) in enumerate([([], None), ([(1, 0)], [1, 1]), ([(0, 1)], [1, 0]), ([(0, 1)], None)]):
        c.X[:] = X + np.float32(0.05 * r)
        force_state(gpu, g, c)
        c.gossip_round(pairs, stale)
        g.gossip_round(pairs, stale)
        assert np.array_equal(g.read_codes(0), ring_row(c, 0)) and np.array_equal(g.read_codes(1), ring_row(c, 1))
        assert_close(g.read_models(gpu.COMM), c.X, TOL_ELEMENTWISE, f"two-node swarm, round {r}")
        if kind == "prefix":
            assert g.prefix_stats() == (c.prefix_levels.tolist(), c.prefix_unconfirmed)
            assert g.counters()["bits_communicated"] == c.bits_communicated
        else:
            assert g.scale() == (float(c.eps_cur), float(c.max_disagreement))
    assert g.counters()["decode_failures"] == c.decode_failures


@pytest.mark.parametrize("d", [8, 16, 504, 512, 520, 1032])
def test_row_lengths_around_the_tile_edges(gpu, d):
    """Rows shorter than a lane group, one short of / exactly / just over one 512-coordinate tile and
    two tiles plus 8: local steps with noise, the gossip pass with fresh and stale reads, the one-pass
    round and the multi-resolution registers all agree with the oracle."""
    n, H, lr, S, eps = 4, 2, 0.1, 1, 2.0 ** -4
    edges = wl.complete_graph(n)
    a, cc = wl.diag_quadratic_data(n, d, 3, shift_sigma=0.2)
    ad, cd = torch.from_numpy(a).cuda(), torch.from_numpy(cc).cuda()
    gen = np.random.Generator(np.random.PCG64(d))
    for bits, prefix in [(4, False), (8, False), (16, True)]:
        two, c2 = make_both(gpu, n, d, edges, bits, eps, H, lr, S, seed=d, prefix=prefix)
        one, c1 = make_both(gpu, n, d, edges, bits, eps, H, lr, S, seed=d, prefix=prefix)
        for g, c in ((two, c2), (one, c1)):
            c.objective = DiagQuadratic(a, cc, 0.05)
            g.set_objective_diag(ad, cd, 0.05)
        for r, (pairs, stale) in enumerate([([(0, 1), (2, 3)], [0, 0, 0, 0]), ([(1, 2)], [1, 1, 1, 1]), ([(3, 0), (2, 1)], [0, 1, 1, 0])]):
            X = models(gen, 1, d) + models(gen, n, d, 0.05)
            for g, c in ((two, c2), (one, c1)):
                c.X[:] = X
                c.pending[:] = False
                force_state(gpu, g, c)
                c.local_steps()
            two.local_steps()
            assert_close(two.read_models(gpu.LIVE), c2.W, TOL_ELEMENTWISE, f"W, bits {bits}, round {r}")
            force_state(gpu, two, c2)
            c2.gossip_round(pairs, stale)
            two.gossip_round(pairs, stale)
            c1.gossip_round(pairs, stale)
            one.round_fused(pairs, stale)
            for g, c, what in ((two, c2, "two calls"), (one, c1, "one pass")):
                for i in range(n):
                    assert np.array_equal(g.read_codes(i), ring_row(c, i)), f"{what}: codes of node {i}, bits {bits}, round {r}"
                assert_close(g.read_models(gpu.COMM), c.X, TOL_TWO_STAGE, f"{what}: X, bits {bits}, round {r}")
                assert g.counters()["decode_failures"] == c.decode_failures


@pytest.mark.parametrize("kind", ["fixed", "per-round scale", "prefix", "algorithm 1"])
def test_saved_state_resumes_bit_for_bit(gpu, kind):
    """Three steps, save, three more; a fresh handle of the same configuration loads the image and
    takes the same three steps: models, registers, counters and the scale are identical."""
    n, d, H, lr, eps = 8, D_RAGGED, 2, 0.1, 2.0 ** -4
    edges = wl.torus_graph(2, 4)
    a, cc = wl.diag_quadratic_data(n, d, 9)
    ad, cd = torch.from_numpy(a).cuda(), torch.from_numpy(cc).cuda()
    sequential = kind == "algorithm 1"
    bits, S = (16 if kind == "prefix" else 8), (0 if sequential else 2)
    kw = dict(scale_policy=gpu.SCALE_GLOBAL_LINF if kind == "per-round scale" else gpu.SCALE_FIXED,
              codec=gpu.CODEC_PREFIX if kind == "prefix" else gpu.CODEC_FIXED)

    def fresh():
        s = gpu.Swarm(n, d, edges, bits, eps, H, lr, S, 21, **kw)
        s.set_objective_diag(ad, cd, 0.05)
        return s

    def step(s, r):
        if sequential:
            s.interact(*s.sample_pair())
        elif r % 2:
            s.round_fused(None, s.sample_stale())
        else:
            s.local_steps([0, 3, 5])                          # leaves pending marks behind when saved mid-way
            s.gossip_round(None, s.sample_stale())

    first = fresh()
    first.write_models(gpu.COMM, models(np.random.Generator(np.random.PCG64(21)), n, d, 0.3))
    for r in range(3):
        step(first, r)
    first.local_steps([1, 2]) if not sequential else None      # pending steps are part of the state
    image = first.save_state()
    second = fresh()
    second.load_state(image)
    for s in (first, second):
        if not sequential:
            s.gossip_round(None, s.sample_stale())
        for r in range(3):
            step(s, r + 1)
    for which in (gpu.COMM, gpu.LIVE) + ((gpu.SNAP,) if sequential else ()):
        assert np.array_equal(first.read_models(which), second.read_models(which))
    for i in range(n):
        for age in range(S + 1):
            assert np.array_equal(first.read_codes(i, age), second.read_codes(i, age))
    assert first.counters() == second.counters() and first.scale() == second.scale()
    assert first.prefix_stats() == second.prefix_stats()
    if sequential:
        # an image saved before any step of Algorithm 1 carries no snapshots: loading it into a handle
        # that has taken steps must bring the snapshots back to the loaded models
        start, used = fresh(), fresh()
        start.write_models(gpu.COMM, models(np.random.Generator(np.random.PCG64(5)), n, d, 0.3))
        early = start.save_state()
        for r in range(3):
            step(used, r)
        used.load_state(early)
        for s in (start, used):
            for r in range(3):
                step(s, r)
        for which in (gpu.COMM, gpu.SNAP):
            assert np.array_equal(start.read_models(which), used.read_models(which))
    with pytest.raises(gpu.SwarmError):
        gpu.Swarm(n, d, edges, bits, eps, H, lr, S, 22, **kw).load_state(image)      # another seed
    with pytest.raises(gpu.SwarmError):
        second.load_state(image[:100])


def test_algorithm1_with_prefix_registers(gpu):
    """Sequential steps where the initiator reads the responder's multi-resolution register; node 3 sits
    tens of cells away (8 bits), node 5 hundreds (16 bits).  Registers, models, snapshots, levels and
    the bits read and written back equal the oracle's."""
    n, d, H, lr, eps = 6, D_RAGGED, 2, 0.1, 2.0 ** -6
    edges = wl.complete_graph(n)
    a, cc = wl.diag_quadratic_data(n, d, 4)
    g, c = make_both(gpu, n, d, edges, 16, eps, H, lr, 0, seed=63, prefix=True)
    c.objective = DiagQuadratic(a, cc, 0.05)
    g.set_objective_diag(torch.from_numpy(a).cuda(), torch.from_numpy(cc).cuda(), 0.05)
    gen = np.random.Generator(np.random.PCG64(63))
    c.X[:] = models(gen, 1, d) + models(gen, n, d, 0.02)
    c.X[3] += 0.5                                          # 32 cells: beyond 4 bits
    c.X[5] += 4.0                                          # 256 cells: beyond 8 bits
    c.Xhat[:] = c.X + models(gen, n, d, 0.01)
    for t, (i, j) in enumerate([(0, 1), (3, 2), (4, 5), (1, 0), (5, 3), (2, 4)]):
        g.write_models(gpu.COMM, c.X)
        g.write_models(gpu.SNAP, c.Xhat)
        c.interact(i, j)
        g.interact(i, j)
        assert np.array_equal(g.read_codes(i), c.ring[0][i]) and np.array_equal(g.read_codes(j), c.ring[0][j])
        assert_close(g.read_models(gpu.COMM), c.X, TOL_TWO_STAGE, f"X, t={t}")
        assert_close(g.read_models(gpu.SNAP), c.Xhat, TOL_TWO_STAGE, f"snapshots, t={t}")
        assert g.prefix_stats() == (c.prefix_levels.tolist(), c.prefix_unconfirmed), f"levels, t={t}"
        cnt = g.counters()
        assert cnt["bits_communicated"] == c.bits_communicated and cnt["decode_failures"] == c.decode_failures
    assert c.prefix_levels[1] > 0 and c.prefix_levels[2] > 0 and g.counters()["interactions"] == 6


def ring_graph(n):
    return [(i, (i + 1) % n) for i in range(n)] if n > 2 else [(0, 1)]


@pytest.mark.parametrize("case", range(48))
def test_random_configurations(gpu, case):
    """Seeded random draws of everything a round can be configured with -- swarm size, row length,
    code width, staleness depth, apply mode, step law, scale policy, register format, one pass or two
    calls, who has pending steps, who is matched -- each checked round by round against the oracle."""
    gen = np.random.Generator(np.random.PCG64(1000 + case))
    n = int(gen.integers(2, 10))
    d = 8 * int(gen.integers(1, 200)) if case % 3 else 8 * int(gen.integers(500, 1600))   # a third spans workgroups
    bits = int(gen.choice([2, 4, 8, 16]))
    S = int(gen.integers(0, 4))
    H = int(gen.integers(1, 4))
    sigma = float(gen.choice([0.0, 0.05]))
    inplace = bool(gen.integers(0, 2))
    geometric = bool(gen.integers(0, 2))
    prefix = bits == 16 and bool(gen.integers(0, 2))
    global_scale = bits >= 8 and not prefix and bool(gen.integers(0, 2))
    # in-place apply in one pass rounds the kernel's own float32 step result, which may differ from the
    # oracle's in the last bit; that pairing is compared elsewhere (one pass against two calls, bit for bit)
    one_pass = bool(gen.integers(0, 2)) and not inplace
    eps = 2.0 ** -int(gen.integers(2, 7))
    edges = wl.complete_graph(n) if gen.integers(0, 2) else ring_graph(n)
    a, cc = wl.diag_quadratic_data(n, d, case, shift_sigma=0.2)
    g, c = make_both(gpu, n, d, edges, bits, eps, H, 0.1, S, seed=case, inplace=inplace, geometric=geometric,
                     global_scale=global_scale, prefix=prefix)
    c.objective = DiagQuadratic(a, cc, sigma)
    g.set_objective_diag(torch.from_numpy(a).cuda(), torch.from_numpy(cc).cuda(), sigma)
    what = dict(n=n, d=d, bits=bits, S=S, H=H, sigma=sigma, inplace=inplace, geometric=geometric, prefix=prefix,
                global_scale=global_scale, one_pass=one_pass, eps=eps)
    base = models(gen, 1, d)
    for r in range(4):
        c.X[:] = base + models(gen, n, d, float(gen.choice([0.02, 0.3])))
        c.pending[:] = False
        force_state(gpu, g, c)
        pairs = c.sample_matching()
        pairs = pairs[: int(gen.integers(0, len(pairs) + 1))]              # sometimes fewer pairs, sometimes none
        stale = np.minimum(gen.integers(0, S + 1, n), r).astype(np.uint8)
        if one_pass:
            c.local_steps()
            c.gossip_round(pairs, stale)
            g.round_fused(pairs, stale)
        else:
            nodes = sorted(gen.choice(n, int(gen.integers(1, n + 1)), replace=False).tolist())
            c.local_steps(nodes)
            g.local_steps(nodes)
            force_state(gpu, g, c)
            c.gossip_round(pairs, stale)
            g.gossip_round(pairs, stale)
        for i in range(n):
            assert np.array_equal(g.read_codes(i), ring_row(c, i)), f"{what}: register of node {i}, round {r}"
        assert_close(g.read_models(gpu.COMM), c.X, TOL_TWO_STAGE, f"{what}: X after round {r}")
        cnt = g.counters(raise_on_range=False)
        assert cnt["decode_failures"] == c.decode_failures and cnt["bits_communicated"] == c.bits_communicated, what
        if global_scale:
            assert g.scale() == (float(c.eps_cur), float(c.max_disagreement)), what
        if prefix:
            assert g.prefix_stats() == (c.prefix_levels.tolist(), c.prefix_unconfirmed), what


@pytest.mark.parametrize("one_pass", [False, True])
def test_many_nodes_few_coordinates(gpu, one_pass):
    """n = 1024 nodes on a random 6-regular graph, d = 64: hundreds of pairs per launch (grid rows),
    matching sampled on the device, stale and fresh reads mixed."""
    n, d, H, lr, bits, eps, S = 1024, 64, 2, 0.1, 8, 2.0 ** -4, 1
    edges = wl.random_regular_graph(n, 6, 3)
    a, cc = wl.diag_quadratic_data(n, d, 12, shift_sigma=0.2)
    g, c = make_both(gpu, n, d, edges, bits, eps, H, lr, S, seed=77)
    c.objective = DiagQuadratic(a, cc, 0.05)
    g.set_objective_diag(torch.from_numpy(a).cuda(), torch.from_numpy(cc).cuda(), 0.05)
    gen = np.random.Generator(np.random.PCG64(77))
    for r in range(3):
        c.X[:] = models(gen, 1, d) + models(gen, n, d, 0.05)
        c.pending[:] = False
        force_state(gpu, g, c)
        pairs, stale = c.sample_matching(), c.sample_stale()
        assert np.array_equal(g.sample_matching(), pairs.astype(np.uint32)) and len(pairs) > 400
        c.local_steps()
        c.gossip_round(pairs, stale)
        if one_pass:
            g.round_fused(None, stale.astype(np.uint8))
        else:
            g.local_steps()
            g.gossip_round(None, stale.astype(np.uint8))
        codes = np.stack([g.read_codes(i) for i in range(0, n, 37)])
        assert np.array_equal(codes, np.stack([ring_row(c, i) for i in range(0, n, 37)]))
        assert_close(g.read_models(gpu.COMM), c.X, TOL_TWO_STAGE, f"X after round {r}")
    assert g.counters()["interactions"] == c.interactions

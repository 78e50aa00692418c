"""Algorithm 1 as batched launches (swarm_run_sequential): the same result, bit for bit, as one
swarm_sample_pair + swarm_interact per step, and the oracle's step_sequential to tolerance."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle.objectives import DiagQuadratic, LeastSquares
from helpers import TOL_ELEMENTWISE, TOL_TWO_STAGE, TOL_GEMM, assert_close, disjoint_prefix, make_both

pytestmark = pytest.mark.gpu

D_RAGGED = 8 * 5231


def models(gen, n, d, scale=1.0):
    return (gen.standard_normal((n, d)) * scale).astype(np.float32)


def build(gpu, kind, seed):
    """Two identical device swarms and the oracle for one of the sequential workloads."""
    geometric = kind == "diag, geometric steps"
    prefix = kind == "diag, prefix registers"
    if kind == "least squares":
        n, d, m, batch, H, lr, bits, eps = 8, 4096, 256, 32, 2, 0.05, 8, 2.0 ** -6      # the small workload's shape
        edges = wl.complete_graph(n)
        A, b, _ = wl.least_squares_data(n, d, m, 0)
        Ad, bd = torch.from_numpy(A).cuda(), torch.from_numpy(b).cuda()
        def objective(g, c):
            g.set_objective_lsq(Ad, bd, m, batch)
            if c is not None:
                c.objective = LeastSquares(A, b, batch)
    else:
        n, d, H, lr = 64, D_RAGGED, 3, 0.1
        bits, eps = (16, 2.0 ** -6) if prefix else (0, 0.0) if kind == "diag, identity quantizer" else (8, 2.0 ** -4)
        edges = wl.random_regular_graph(n, 4, 0)
        a, cc = wl.diag_quadratic_data(n, d, 3)
        ad, cd = torch.from_numpy(a).cuda(), torch.from_numpy(cc).cuda()
        sigma = 0.0 if kind == "diag, no noise" else 0.05
        def objective(g, c):
            if kind == "no objective, caller's steps":
                return
            g.set_objective_diag(ad, cd, sigma)
            if c is not None:
                c.objective = DiagQuadratic(a, cc, sigma)
    pair = [make_both(gpu, n, d, edges, bits, eps, H, lr, 0, seed=seed, geometric=geometric, prefix=prefix) for _ in range(2)]
    (g1, c), (g2, _) = pair
    objective(g1, c)
    objective(g2, None)
    gen = np.random.Generator(np.random.PCG64(seed))
    c.X[:] = models(gen, 1, d) + models(gen, n, d, 0.05)
    if prefix:
        c.X[3] += 0.5                                       # tens of cells away: reads go to 8 bits
    c.Xhat[:] = c.X + models(gen, n, d, 0.01)
    for g in (g1, g2):
        g.write_models(gpu.COMM, c.X)
        g.write_models(gpu.SNAP, c.Xhat)
    if kind == "no objective, caller's steps":
        c.W[:] = c.Xhat + models(gen, n, d, 0.02)
        c.pending[:] = True
        for g in (g1, g2):
            g.write_models(gpu.LIVE, c.W)                   # marks every node pending
    return g1, g2, c


KINDS = ["least squares", "diag", "diag, no noise", "diag, geometric steps", "diag, prefix registers",
         "diag, identity quantizer", "no objective, caller's steps"]


@pytest.mark.parametrize("kind", KINDS)
def test_batched_run_equals_one_interaction_per_call_bit_for_bit(gpu, kind):
    T = 60 if kind == "least squares" else 150
    g1, g2, c = build(gpu, kind, seed=7 + len(kind))
    drawn = []
    for t in range(T):
        i, j = g1.sample_pair()
        drawn.append((i, j))
        g1.interact(i, j)
    # two calls, so that the second starts from a state with interactions behind it
    pairs_a, launches_a = g2.run_sequential(T // 3)
    pairs_b, launches_b = g2.run_sequential(T - T // 3)
    assert np.array_equal(np.concatenate([pairs_a, pairs_b]), np.array(drawn, dtype=np.uint32))
    assert 0 < launches_a + launches_b < T                   # several interactions share a launch
    assert np.array_equal(g2.read_models(gpu.COMM), g1.read_models(gpu.COMM))
    assert np.array_equal(g2.read_models(gpu.SNAP), g1.read_models(gpu.SNAP))
    if c.bits:
        for node in range(c.n):
            assert np.array_equal(g2.read_codes(node), g1.read_codes(node)), f"register of node {node}"
    assert g2.counters() == g1.counters()
    assert g2.prefix_stats() == g1.prefix_stats()
    assert g2.sample_pair() == g1.sample_pair()              # both stand at the same interaction number
    if kind in ("least squares", "no objective, caller's steps"):   # the steps are a kernel of their own: same live copies
        assert np.array_equal(g2.read_models(gpu.LIVE), g1.read_models(gpu.LIVE))


@pytest.mark.parametrize("kind", ["least squares", "diag", "diag, geometric steps", "diag, prefix registers",
                                  "diag, identity quantizer", "no objective, caller's steps"])
def test_one_launch_of_disjoint_interactions_against_the_oracle(gpu, kind):
    """Teacher-forced: from the oracle's state, as many steps of Algorithm 1 as touch disjoint nodes --
    one launch on the device -- against the oracle taking them one after the other.  Nothing the
    device quantizes depends on its own float32 local steps here, so codes are bit-exact."""
    g, _, c = build(gpu, kind, seed=31 + len(kind))
    tol = TOL_GEMM if kind == "least squares" else TOL_TWO_STAGE
    widths = []
    for rep in range(6):
        g.write_models(gpu.COMM, c.X)
        g.write_models(gpu.SNAP, c.Xhat)
        if kind == "no objective, caller's steps":
            gen = np.random.Generator(np.random.PCG64(rep))
            c.W[:] = c.Xhat + models(gen, c.n, c.d, 0.02)
            c.pending[:] = True
            g.write_models(gpu.LIVE, c.W)
        k = disjoint_prefix(c, c.n // 2)
        widths.append(k)
        steps = [c.step_sequential() for _ in range(k)]
        pairs, launches = g.run_sequential(k)
        assert [tuple(p) for p in pairs.tolist()] == steps and launches == 1
        if c.bits:
            for i, j in steps:
                assert np.array_equal(g.read_codes(i), c.ring[0][i]) and np.array_equal(g.read_codes(j), c.ring[0][j])
        assert_close(g.read_models(gpu.COMM), c.X, tol, f"X after {k} interactions in one launch")
        assert_close(g.read_models(gpu.SNAP), c.Xhat, tol, "snapshots")
        cnt = g.counters()
        assert cnt["interactions"] == c.interactions and cnt["bits_communicated"] == c.bits_communicated
        assert cnt["decode_failures"] == c.decode_failures
        if kind == "diag, prefix registers":
            assert g.prefix_stats() == (c.prefix_levels.tolist(), c.prefix_unconfirmed)
    assert max(widths) >= 2


def test_long_batched_run_follows_the_oracle(gpu):
    """200 steps on the small least-squares workload without forcing: a last-bit difference of the
    float32 path can flip a rounding decision later on, so all but a few entries agree to tolerance
    and those few stay within a couple of lattice cells."""
    g, _, c = build(gpu, "least squares", seed=0)
    pairs, launches = g.run_sequential(200)
    for t in range(200):
        assert c.step_sequential() == tuple(int(v) for v in pairs[t])
    X = g.read_models(gpu.COMM).astype(np.float64)
    diff = np.abs(X - c.X)
    assert diff.max() <= 8 * c.eps
    assert (diff > 1e-4).mean() < 0.05
    assert g.potential() == pytest.approx(c.potential(), rel=0.05)
    cnt = g.counters()
    assert cnt["interactions"] == 200 and cnt["bits_communicated"] == c.bits_communicated
    assert launches < 120


def test_batched_run_rejects_what_algorithm_1_does_not_cover(gpu):
    edges = wl.complete_graph(4)
    s = gpu.Swarm(4, 64, edges, 8, 1.0, 0, 0.0, stale_max=1)
    with pytest.raises(gpu.SwarmError):
        s.run_sequential(3)                                  # stale reads are a round-mode notion
    s = gpu.Swarm(4, 64, edges, 8, 1.0, 0, 0.0, apply_mode=gpu.INPLACE)
    with pytest.raises(gpu.SwarmError):
        s.run_sequential(3)
    s = gpu.Swarm(4, 64, edges, 8, 1.0, 0, 0.0)
    pairs, launches = s.run_sequential(0)
    assert len(pairs) == 0 and launches == 0 and s.counters()["interactions"] == 0

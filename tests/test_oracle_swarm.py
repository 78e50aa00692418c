"""Pins for the oracle's interaction rules: the invariants and exact identities
the paper's analysis states (appendix, potential-bound lemmas) and brute force."""
import itertools
import math

import numpy as np
import pytest

import workloads as wl
from oracle import quantizer as qz
from oracle import rng
from oracle.objectives import DiagQuadratic, LeastSquares, MixtureMLP
from oracle.swarm import SwarmOracle


def make(n, d, edges, bits=0, eps=1.0, H=0, lr=0.0, S=0, seed=0, dtype=np.float64, X=None):
    o = SwarmOracle(n, d, edges, bits, eps, H, lr, S, seed, state_dtype=dtype)
    if X is not None:
        o.X[:] = X
        o.W[:] = X
        o.Xhat[:] = X
    return o


def gamma(X):
    return float(((X - X.mean(axis=0)) ** 2).sum())


# ---------------------------------------------------------------- averaging without quantization
def test_mean_preserved_and_potential_drop_identity_single_interaction():
    """With Q = identity and no local steps: mu is unchanged and
    Gamma_{t+1} - Gamma_t = -|X_i - X_j|^2 / 2 (per-step potential lemma, S = 0)."""
    gen = np.random.Generator(np.random.PCG64(0))
    n, d = 6, 8
    X = gen.standard_normal((n, d))
    for i, j in [(0, 1), (4, 2), (5, 0)]:
        o = make(n, d, wl.complete_graph(n), X=X)
        o.interact(i, j)
        assert np.allclose(o.mean(), X.mean(axis=0), atol=1e-15)
        assert o.potential() - gamma(X) == pytest.approx(-((X[i] - X[j]) ** 2).sum() / 2, rel=1e-12)
        assert np.array_equal(o.X[i], o.X[j]) and np.allclose(o.X[i], (X[i] + X[j]) / 2)
        others = [k for k in range(n) if k not in (i, j)]
        assert np.array_equal(o.X[others], X[others])


def test_round_of_disjoint_pairs_is_a_sum_of_interactions():
    gen = np.random.Generator(np.random.PCG64(1))
    n, d = 8, 16
    X = gen.standard_normal((n, d))
    pairs = [(0, 3), (5, 1), (2, 7)]
    o = make(n, d, wl.complete_graph(n), X=X)
    o.gossip_round(pairs)
    assert np.allclose(o.mean(), X.mean(axis=0), atol=1e-15)
    drop = sum(((X[i] - X[j]) ** 2).sum() / 2 for i, j in pairs)
    assert gamma(X) - o.potential() == pytest.approx(drop, rel=1e-12)
    assert o.round == 1 and o.interactions == 3


def test_complete_graph_expected_contraction_by_enumeration():
    """Complete graph (lambda_2 = n): over all n(n-1) ordered (initiator, responder)
    choices, E[Gamma_{t+1}] = Gamma_t (1 - 1/(n-1)) exactly."""
    gen = np.random.Generator(np.random.PCG64(2))
    for n in (3, 5):
        X = gen.standard_normal((n, 8))
        total = 0.0
        for i, j in itertools.permutations(range(n), 2):
            o = make(n, 8, wl.complete_graph(n), X=X)
            o.interact(i, j)
            total += o.potential()
        assert total / (n * (n - 1)) == pytest.approx(gamma(X) * (1 - 1 / (n - 1)), rel=1e-12)
        assert wl.laplacian_lambda2(n, wl.complete_graph(n)) == pytest.approx(n)


@pytest.mark.parametrize("graph", ["torus", "regular"])
def test_laplacian_inequality_and_per_step_contraction(graph):
    """sum_E |X_i - X_j|^2 >= lambda_2 Gamma, and enumerating Algorithm 1's sampling
    law (initiator uniform, responder uniform among neighbours) the expected
    potential contracts at least by the factor 1 - lambda_2 / (2 n rho_max)."""
    n, d = (16, 8) if graph == "torus" else (12, 8)
    edges = wl.torus_graph(4, 4) if graph == "torus" else wl.random_regular_graph(12, 3, 5)
    adj = wl.adjacency(n, edges)
    lam2 = wl.laplacian_lambda2(n, edges)
    rho_max = max(len(a) for a in adj)
    X = np.random.Generator(np.random.PCG64(3)).standard_normal((n, d))
    o = make(n, d, edges, X=X)
    edge_sum = sum(((X[u] - X[v]) ** 2).sum() for u, v in edges.tolist())
    assert edge_sum >= lam2 * o.potential() * (1 - 1e-12)
    expect = 0.0
    for i in range(n):
        for j in adj[i]:
            o = make(n, d, edges, X=X)
            o.interact(i, j)
            expect += o.potential() / (n * len(adj[i]))
    exact = gamma(X) - sum(((X[i] - X[j]) ** 2).sum() / (2 * n * len(adj[i])) for i in range(n) for j in adj[i])
    assert expect == pytest.approx(exact, rel=1e-12)
    assert expect <= (1 - lam2 / (2 * n * rho_max)) * gamma(X)


# ---------------------------------------------------------------- quantized interaction
def test_quantized_interaction_matches_the_exact_potential_identity():
    """Algorithm 1 with quantization: X_i' = (X_i+X_j)/2 + S_i, X_j' = (X_i+X_j)/2 + S_j with
    S_j = (Q(X_i)-X_i)/2 + (Q(X_j)-X_j)/2, mu' = mu + (S_i+S_j)/n, |S_j|^2 <= the two
    quantization errors' half-sum, and the potential change equals the closed expression
    of the per-step lemma's proof."""
    gen = np.random.Generator(np.random.PCG64(4))
    n, d, eps, bits = 5, 64, 2.0 ** -3, 8
    X = gen.standard_normal((n, d)).astype(np.float32).astype(np.float64)
    i, j = 3, 1
    o = make(n, d, wl.complete_graph(n), bits=bits, eps=eps, seed=9, X=X)
    o.interact(i, j)
    Qi = qz.stochastic_round(X[i], eps, rng.sr_halves(9, i, 0, 0, d)) * eps
    Qj = qz.stochastic_round(X[j], eps, rng.sr_halves(9, j, 0, 0, d)) * eps
    assert np.all(np.abs(Qi - X[i]) < eps) and np.all(np.abs(Qj - X[j]) < eps)
    S = (Qi - X[i]) / 2 + (Qj - X[j]) / 2
    assert np.allclose(o.X[i], (X[i] + X[j]) / 2 + S, atol=1e-14)
    assert np.array_equal(o.X[i], o.X[j])
    assert np.allclose(o.mean(), X.mean(axis=0) + 2 * S / n, atol=1e-14)
    assert (S ** 2).sum() <= ((Qi - X[i]) ** 2).sum() / 2 + ((Qj - X[j]) ** 2).sum() / 2 + 1e-15
    mu = X.mean(axis=0)
    closed = (-((X[i] - X[j]) ** 2).sum() / 2 + ((X[i] - mu + X[j] - mu) * 2 * S).sum()
              + (n - 2) / n ** 2 * ((2 * S) ** 2).sum() + 2 * (((n - 2) / n * S) ** 2).sum())
    assert o.potential() - gamma(X) == pytest.approx(closed, rel=1e-10)
    assert o.decode_failures == 0 and o.bits_communicated == 2 * d * bits


def test_round_mode_pair_holds_the_same_average_when_decodes_succeed():
    gen = np.random.Generator(np.random.PCG64(5))
    n, d, eps, bits = 6, 128, 2.0 ** -4, 8
    X = (gen.standard_normal((n, d)) * 0.5).astype(np.float32)
    o = make(n, d, wl.complete_graph(n), bits=bits, eps=eps, seed=1, X=X, dtype=np.float32)
    o.gossip_round([(0, 5), (2, 3)])
    assert o.decode_failures == 0
    assert np.array_equal(o.X[0], o.X[5]) and np.array_equal(o.X[2], o.X[3])
    assert np.array_equal(o.X[1], X[1]) and np.array_equal(o.X[4], X[4])
    assert np.all(np.abs(o.X[0].astype(np.float64) - (X[0].astype(np.float64) + X[5]) / 2) < eps)
    lattice = o.X[0].astype(np.float64) / (eps / 2)                 # averages live on the half lattice
    assert np.array_equal(lattice, np.rint(lattice))


def test_decode_failure_wraps_identically_and_is_counted():
    """Rows farther apart than the decoding radius: the receiver lands on another member of
    the residue class (off by a multiple of 2^b eps), and the simulation counts it."""
    n, d, eps, bits = 2, 16, 1.0, 4
    X = np.zeros((n, d), dtype=np.float32)
    X[1] = 20.0                                                      # 20 eps apart, radius is 5.5 eps
    o = make(n, d, wl.complete_graph(n), bits=bits, eps=eps, X=X, dtype=np.float32)
    o.gossip_round([(0, 1)])
    assert o.decode_failures == 2 * d
    # node 0 sees 20 as 20 - 16 = 4 ; node 1 sees 0 as 16
    assert np.all(o.X[0] == 2.0) and np.all(o.X[1] == 18.0)


def test_stale_reads_use_the_code_published_s_rounds_earlier():
    gen = np.random.Generator(np.random.PCG64(6))
    n, d, eps, bits, S = 4, 32, 2.0 ** -3, 8, 2
    X0 = (gen.standard_normal((n, d)) * 0.3).astype(np.float32)
    o = make(n, d, wl.complete_graph(n), bits=bits, eps=eps, S=S, seed=2, X=X0, dtype=np.float32)
    hist = []
    for r in range(3):
        hist.append(o.X.copy())
        o.gossip_round([(0, 1), (2, 3)], stale=[0] * n)
    Xr = o.X.copy()
    o.gossip_round([(0, 2)], stale=[2, 1, 1, 0])                       # round 3: 0 reads 2 from round 1, 2 reads 0 fresh
    z0 = qz.stochastic_round(Xr[0], eps, rng.sr_halves(2, 0, 3, 0, d))
    z2_old = qz.stochastic_round(hist[1][2], eps, rng.sr_halves(2, 2, 1, 0, d))
    z2_now = qz.stochastic_round(Xr[2], eps, rng.sr_halves(2, 2, 3, 0, d))
    assert np.allclose(o.X[0], (z0 + z2_old) * eps / 2)
    assert np.allclose(o.X[2], (z2_now + z0) * eps / 2)
    # staleness is limited to the rounds that exist
    o2 = make(n, d, wl.complete_graph(n), bits=bits, eps=eps, S=S, seed=2, X=X0, dtype=np.float32)
    o3 = make(n, d, wl.complete_graph(n), bits=bits, eps=eps, S=S, seed=2, X=X0, dtype=np.float32)
    o2.gossip_round([(0, 1)], stale=[2, 2, 0, 0])
    o3.gossip_round([(0, 1)], stale=[0, 0, 0, 0])
    assert np.array_equal(o2.X, o3.X)


def test_algorithm1_snapshot_and_responder_rules():
    """Initiator applies its steps (computed at its snapshot) on top of the average and
    refreshes its snapshot; the responder gets the plain average and keeps its snapshot."""
    gen = np.random.Generator(np.random.PCG64(7))
    n, d = 4, 8
    a = gen.uniform(0.5, 2, (n, d)).astype(np.float32)
    c = gen.standard_normal((n, d)).astype(np.float32)
    X = gen.standard_normal((n, d))
    o = make(n, d, wl.complete_graph(n), H=2, lr=0.1, X=X)
    o.objective = DiagQuadratic(a, c, 0.0)
    o.interact(0, 1)
    avg = (X[0] + X[1]) / 2
    w = X[0].copy()
    for _ in range(2):
        w = w - np.float64(np.float32(0.1)) * a[0] * (w - c[0])
    assert np.allclose(o.X[1], avg) and np.allclose(o.X[0], avg + (w - X[0]))
    assert np.array_equal(o.Xhat[0], o.X[0]) and np.array_equal(o.Xhat[1], X[1])
    # responder 1 now initiates: its gradient is taken at its old snapshot X[1], not at the average
    o.interact(1, 2)
    w1 = X[1].copy()
    for _ in range(2):
        w1 = w1 - np.float64(np.float32(0.1)) * a[1] * (w1 - c[1])
    assert np.allclose(o.X[1], (avg + X[2]) / 2 + (w1 - X[1]))


def test_potential_of_the_snapshots_by_hand_and_against_its_bound():
    """Gamma-hat = sum_i |Xhat_i - mu|^2 with mu the mean of the CURRENT models (appendix, "Potential
    Functions").  By hand on three nodes; then the appendix's inequality Gamma-hat <= 2 A + 2 B along a
    run, A = sum_i |X^i - mu|^2 and B = sum_i |mu_now - mu_then|^2 taken when node i last initiated."""
    o = make(3, 8, wl.complete_graph(3))
    o.X[:] = np.array([1.0, 2.0, 6.0])[:, None]          # mean 3 in every coordinate
    o.Xhat[:] = np.array([0.0, 2.0, 4.0])[:, None]
    assert o.potential_hat() == pytest.approx(8 * (9 + 1 + 1))
    assert o.potential() == pytest.approx(8 * (4 + 1 + 9))
    gen = np.random.Generator(np.random.PCG64(12))
    n, d = 6, 16
    a = gen.uniform(0.5, 2, (n, d)).astype(np.float32)
    c = gen.standard_normal((n, d)).astype(np.float32)
    o = make(n, d, wl.complete_graph(n), H=2, lr=0.1, seed=4, X=gen.standard_normal((n, d)))
    o.objective = DiagQuadratic(a, c, 0.05)
    then_x = [o.X[i].copy() for i in range(n)]            # X^i and mu at node i's last initiation (the start, before any)
    then_mu = [o.mean() for _ in range(n)]
    strict = 0
    for t in range(60):
        i, _ = o.step_sequential()
        then_x[i], then_mu[i] = o.X[i].copy(), o.mean()
        assert all(np.array_equal(o.Xhat[k], then_x[k]) for k in range(n))
        mu = o.mean()
        A = sum(((then_x[k] - then_mu[k]) ** 2).sum() for k in range(n))
        B = sum(((mu - then_mu[k]) ** 2).sum() for k in range(n))
        direct = sum(((then_x[k] - mu) ** 2).sum() for k in range(n))
        assert o.potential_hat() == pytest.approx(direct, rel=1e-12)
        assert o.potential_hat() <= 2 * A + 2 * B + 1e-12
        strict += o.potential_hat() != pytest.approx(o.potential(), rel=1e-6)
    assert strict > 30                                      # the snapshots really lag behind the current models


def test_staleness_clock_second_moment_bound():
    """tau_i resets when i initiates, else grows by one; sum_i E[tau_i^2] <= 5 n^3
    (clock-bound lemma); sampled initiators come from the PICK stream."""
    n = 8
    o = make(n, 8, wl.complete_graph(n), seed=3)
    tau = np.zeros(n)
    acc, T = 0.0, 4000
    counts = np.zeros(n)
    for t in range(T):
        i, j = o.sample_pair()
        assert j in o.adj[i]
        o.interactions += 1
        counts[i] += 1
        tau += 1
        tau[i] = 0
        if t >= 500:
            acc += (tau ** 2).sum()
    mean_sq = acc / (T - 500)
    assert mean_sq <= 5 * n ** 3
    assert mean_sq == pytest.approx(n * (2 * n * n - 3 * n + 1), rel=0.2)   # geometric waiting time, p = 1/n
    assert np.all(np.abs(counts - T / n) < 5 * math.sqrt(T / n))


# ---------------------------------------------------------------- matching
def greedy_reference(n, edges, prio):
    free, out = set(range(n)), []
    for e in sorted(range(len(edges)), key=lambda e: prio[e]):
        u, v = edges[e]
        if u in free and v in free:
            free -= {u, v}
            out.append(e)
    return sorted(out)


def test_matching_is_valid_maximal_and_greedy():
    for name, n, edges in [("torus", 64, wl.torus_graph(8, 8)), ("reg", 64, wl.random_regular_graph(64, 4, 1)),
                           ("complete", 9, wl.complete_graph(9))]:
        o = make(n, 8, edges, seed=4)
        for r in range(20):
            o.round = r
            pairs = o.sample_matching()
            nodes = pairs.reshape(-1).tolist()
            assert len(set(nodes)) == len(nodes)
            eset = {tuple(e) for e in edges.tolist()}
            assert all(tuple(p) in eset for p in pairs.tolist())
            used = set(nodes)
            assert all(u in used or v in used for u, v in edges.tolist())         # maximal
            prio = o.edge_priorities().tolist()
            want = greedy_reference(n, edges.tolist(), prio)
            assert [tuple(edges[e]) for e in want] == [tuple(p) for p in pairs.tolist()]
            assert len(set(prio)) == len(prio)


def test_perfect_matchings_of_k4_are_equally_likely():
    edges = wl.complete_graph(4)
    o = make(4, 8, edges, seed=5)
    counts = {}
    trials = 3000
    for r in range(trials):
        o.round = r
        key = tuple(map(tuple, o.sample_matching().tolist()))
        counts[key] = counts.get(key, 0) + 1
    assert len(counts) == 3
    chi2 = sum((c - trials / 3) ** 2 / (trials / 3) for c in counts.values())
    assert chi2 < 13.8                                                             # chi^2_2 at 0.001


def test_stale_draw_is_uniform_and_limited():
    o = make(32, 8, wl.complete_graph(32), bits=8, eps=1.0, S=2, seed=6)
    assert o.sample_stale().tolist() == [0] * 32                                    # round 0: nothing older exists
    o.round = 1
    assert set(o.sample_stale().tolist()) <= {0, 1}
    hist = np.zeros(3)
    for r in range(2, 302):
        o.round = r
        hist += np.bincount(o.sample_stale(), minlength=3)
    assert np.all(np.abs(hist / hist.sum() - 1 / 3) < 0.02)


# ---------------------------------------------------------------- local steps
def test_diag_quadratic_closed_form_and_noise_statistics():
    gen = np.random.Generator(np.random.PCG64(8))
    n, d, H, lr = 3, 32768, 3, 0.1      # 98304 draws: the sample variance has std 0.0045
    a, c = wl.diag_quadratic_data(n, d, 0)
    X = gen.standard_normal((n, d))
    o = make(n, d, wl.complete_graph(n), H=H, lr=lr, X=X)
    o.objective = DiagQuadratic(a, c, 0.0)
    o.local_steps()
    eta = np.float64(np.float32(lr))
    closed = c + (1 - eta * a.astype(np.float64)) ** H * (X - c)
    assert np.allclose(o.W, closed, rtol=0, atol=1e-13)
    assert o.pending.all() and np.array_equal(o.X, X)                               # not yet applied
    sigma = 0.1
    o.objective = DiagQuadratic(a, c, sigma)
    o.local_steps()
    dev = o.W - closed                   # = -eta sigma sum_q (1 - eta a)^(H-1-q) N_q
    var = (eta * float(np.float32(sigma))) ** 2 * sum((1 - eta * a.astype(np.float64)) ** (2 * p) for p in range(H))
    zscore = dev / np.sqrt(var)
    assert abs(zscore.mean()) < 5 / math.sqrt(zscore.size)
    assert zscore.var() == pytest.approx(1.0, abs=0.03)
    o.gossip_round([])                   # unmatched nodes apply their own steps
    assert np.array_equal(o.X, o.W) and not o.pending.any()


def test_diag_quadratic_window_equals_slice_of_full_row():
    n, d = 2, 256
    a, c = wl.diag_quadratic_data(n, d, 1)
    full = SwarmOracle(n, d, wl.complete_graph(n), 8, 2.0 ** -5, 3, 0.1, 1, 7)
    win = SwarmOracle(n, d, wl.complete_graph(n), 8, 2.0 ** -5, 3, 0.1, 1, 7, k0=64, k1=192)
    full.objective = DiagQuadratic(a, c, 0.05)
    win.objective = DiagQuadratic(a[:, 64:192], c[:, 64:192], 0.05, k0=64)
    for r in range(3):
        for o in (full, win):
            o.local_steps()
            o.gossip_round([(0, 1)], stale=[min(r, 1)] * 2)
        assert np.array_equal(full.X[:, 64:192], win.X)
        assert np.array_equal(full.ring[r % 2][0][64:192], win.ring[r % 2][0])


def test_least_squares_gradient_against_numpy_and_unbiasedness():
    n, d, m, batch = 2, 64, 32, 8
    A, b, _ = wl.least_squares_data(n, d, m, 0)
    obj = LeastSquares(A, b, batch)
    w = np.random.Generator(np.random.PCG64(9)).standard_normal(d)
    rows = obj.batch_rows(1, 3, 4, 0)
    assert rows.shape == (batch,) and rows.min() >= 0 and rows.max() < m
    g = obj.gradient(1, w, 3, 4, 0)
    want = np.zeros(d)
    for r in rows:                                       # per-sample definition
        want += (m / batch) * A[1, r].astype(np.float64) * (A[1, r].astype(np.float64) @ w - float(b[1, r]))
    assert np.allclose(g, want, rtol=1e-12, atol=1e-12)
    full = A[1].astype(np.float64).T @ (A[1].astype(np.float64) @ w - b[1])
    mean = np.mean([obj.gradient(1, w, 3, ev, 0) for ev in range(3000)], axis=0)
    assert np.linalg.norm(mean - full) < 0.1 * np.linalg.norm(full)
    hist = np.bincount(np.concatenate([obj.batch_rows(0, 1, ev, q) for ev in range(500) for q in range(2)]), minlength=m)
    assert np.all(np.abs(hist - hist.sum() / m) < 5 * math.sqrt(hist.sum() / m))


def test_mlp_gradient_against_autograd_float64():
    import torch
    n, n_in, n_hid, n_out, batch = 2, 16, 24, 8, 12
    means, cdf = wl.mixture_data(n, n_in, n_out, 0)
    obj = MixtureMLP(n_in, n_hid, n_out, means, cdf, 0.5, batch)
    w = np.random.Generator(np.random.PCG64(10)).standard_normal(obj.d) * 0.2
    x, y = obj.batch_data(1, 5, 6, 1)
    loss, g = obj.loss_and_gradient(w, x, y)
    wt = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    p = 0
    W1 = wt[p:p + n_hid * n_in].reshape(n_hid, n_in); p += n_hid * n_in
    b1 = wt[p:p + n_hid]; p += n_hid
    W2 = wt[p:p + n_out * n_hid].reshape(n_out, n_hid); p += n_out * n_hid
    b2 = wt[p:p + n_out]
    hid = torch.relu(torch.tensor(x) @ W1.T + b1)
    lt = torch.nn.functional.cross_entropy(hid @ W2.T + b2, torch.tensor(y))
    lt.backward()
    assert loss == pytest.approx(float(lt.detach()), rel=1e-12)
    assert np.allclose(g, wt.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_mlp_batch_follows_the_node_label_law_and_mixture():
    n, n_in, n_out, batch = 2, 8, 4, 64
    means, cdf = wl.mixture_data(n, n_in, n_out, 1, alpha=0.5)
    obj = MixtureMLP(n_in, 8, n_out, means, cdf, 0.5, batch)
    ys, res = [], []
    for ev in range(200):
        x, y = obj.batch_data(0, 2, ev, 0)
        ys.append(y)
        res.append(x - means[y])
    ys, res = np.concatenate(ys), np.concatenate(res)
    law = np.diff(np.concatenate([[0.0], cdf[0].astype(np.float64)]))
    freq = np.bincount(ys, minlength=n_out) / ys.size
    assert np.all(np.abs(freq - law) < 5 * np.sqrt(law * (1 - law) / ys.size) + 1e-3)
    assert res.std() == pytest.approx(0.5, rel=0.02) and abs(res.mean()) < 0.01


def test_swarm_converges_to_the_global_minimiser_neighbourhood():
    """Diagonal quadratics have the closed-form minimiser x* = sum_i a_i c_i / sum_i a_i;
    the swarm mean approaches it and Gamma stays bounded (does not grow with t)."""
    n, d = 8, 64
    edges = wl.complete_graph(n)
    a, c = wl.diag_quadratic_data(n, d, 3)
    o = SwarmOracle(n, d, edges, 8, 2.0 ** -4, 3, 0.1, 0, 11)
    o.objective = DiagQuadratic(a, c, 0.05)
    xstar = (a.astype(np.float64) * c).sum(axis=0) / a.astype(np.float64).sum(axis=0)
    gam = []
    for r in range(150):
        o.local_steps()
        o.gossip_round(o.sample_matching())
        gam.append(o.potential())
    assert o.decode_failures == 0
    assert np.sqrt(((o.mean() - xstar) ** 2).mean()) < 0.25
    assert np.mean(gam[100:]) < 1.5 * np.mean(gam[50:100]) + 1e-9


def test_oracle_inplace_mode_is_average_of_updated_models():
    """CPU pin of the in-place rule: with Q = identity, X_i' = (w_i + w_j)/2 where w = X - eta h~(X)."""
    n, d, H, lr = 4, 16, 2, 0.1
    a, cc = wl.diag_quadratic_data(n, d, 1)
    o = SwarmOracle(n, d, wl.complete_graph(n), 0, 0.0, H, lr, 0, 0, state_dtype=np.float64, apply_mode="inplace")
    o.objective = DiagQuadratic(a, cc, 0.0)
    X = np.random.Generator(np.random.PCG64(0)).standard_normal((n, d))
    o.X[:] = X
    o.local_steps()
    w = cc + (1 - np.float64(np.float32(lr)) * a.astype(np.float64)) ** H * (X - cc)
    assert np.allclose(o.X, w, atol=1e-13) and not o.pending.any()
    o.gossip_round([(0, 1)])
    assert np.allclose(o.X[0], (w[0] + w[1]) / 2) and np.array_equal(o.X[0], o.X[1])


def test_geometric_steps_have_the_stated_moments():
    """Geometric H_i of mean H: E[H_i] = H and E[H_i^2] = 2H^2 - H (appendix, properties of the
    local steps); draws are >= 1, fresh per node and per interaction."""
    for H in (2, 3, 5):
        o = SwarmOracle(64, 8, wl.complete_graph(64), 0, 0.0, H, 0.1, 0, 5, steps_law="geometric")
        draws = []
        for r in range(150):
            o.round = r
            draws.append(o.sample_steps())
        k = np.concatenate(draws).astype(np.float64)
        assert k.min() >= 1
        se1 = math.sqrt((H * H - H) / k.size)
        assert abs(k.mean() - H) < 5 * se1 + 1e-3
        assert (k ** 2).mean() == pytest.approx(2 * H * H - H, rel=0.08)
        assert not np.array_equal(draws[0], draws[1])
    one = SwarmOracle(4, 8, wl.complete_graph(4), 0, 0.0, 1, 0.1, 0, 5, steps_law="geometric")
    assert one.sample_steps().tolist() == [1, 1, 1, 1]
    const = SwarmOracle(4, 8, wl.complete_graph(4), 0, 0.0, 3, 0.1, 0, 5)
    assert const.sample_steps().tolist() == [3, 3, 3, 3]


def test_geometric_steps_are_used_by_the_local_steps():
    n, d, H, lr = 6, 16, 3, 0.1
    a, cc = wl.diag_quadratic_data(n, d, 2)
    o = SwarmOracle(n, d, wl.complete_graph(n), 0, 0.0, H, lr, 0, 9, state_dtype=np.float64, steps_law="geometric")
    o.objective = DiagQuadratic(a, cc, 0.0)
    X = np.random.Generator(np.random.PCG64(1)).standard_normal((n, d))
    o.X[:] = X
    o.local_steps()
    steps = o.sample_steps()
    assert len(set(steps.tolist())) > 1
    for i in range(n):
        closed = cc[i] + (1 - np.float64(np.float32(lr)) * a[i].astype(np.float64)) ** int(steps[i]) * (X[i] - cc[i])
        assert np.allclose(o.W[i], closed, atol=1e-13)


def test_sequential_sampling_law_initiator_and_responder_independent():
    """Algorithm 1's sampling lines: every ordered edge (i, j) has probability 1 / (n deg(i))."""
    edges = wl.torus_graph(4, 4)
    n = 16
    o = make(n, 8, edges, seed=12)
    counts = {}
    T = 6400
    for t in range(T):
        o.interactions = t
        ij = o.sample_pair()
        counts[ij] = counts.get(ij, 0) + 1
    adj = wl.adjacency(n, edges)
    assert set(counts) == {(i, j) for i in range(n) for j in adj[i]}      # all 64 ordered edges occur
    expected = T / 64
    chi2 = sum((c - expected) ** 2 / expected for c in counts.values())
    assert chi2 < 63 + 5 * math.sqrt(2 * 63)


def test_algorithm1_initiator_uses_the_decoded_partner_model():
    """Rows farther apart than the radius: the initiator averages with what it decodes (another
    member of the residue class), and writes that average to the responder too."""
    n, d, eps, bits = 2, 8, 1.0, 4
    X = np.zeros((n, d))
    X[1] = 20.0
    o = make(n, d, wl.complete_graph(n), bits=bits, eps=eps, X=X)
    o.interact(0, 1)
    assert np.all(o.X[0] == 2.0) and np.all(o.X[1] == 2.0)          # 20 is read as 20 - 16 = 4
    assert o.decode_failures == d


# ---------------------------------------------------------------- one lattice scale per round
def global_oracle(n, d, bits, eps, S=0, seed=0, X=None):
    o = SwarmOracle(n, d, wl.complete_graph(n), bits, eps, 0, 0.0, S, seed, state_dtype=np.float32,
                    scale_policy="global_linf")
    if X is not None:
        o.X[:] = X
        o.W[:] = X
    return o


def lattice_points(o, slot, node, key, eps):
    """Decode a published code by hand: plain Python integers, nearest member of the residue class."""
    codes = qz.unpack(o.ring[slot][node], o.bits, o.d)
    out = []
    for c, y in zip(codes.tolist(), key.tolist()):
        k = round(float(np.float32(y) * np.float32(1.0 / eps)))           # eps is a power of two: exact
        cands = [c + w * (1 << o.bits) for w in range((k >> o.bits) - 2, (k >> o.bits) + 3)]
        out.append(min(cands, key=lambda v: (abs(v - k), v > k)))          # window [k - 2^(b-1), k + 2^(b-1) - 1]
    return np.array(out, dtype=np.int64)


@pytest.mark.parametrize("bits", [8, 16])
def test_global_scale_equals_the_fixed_scale_rule_while_the_scale_stands_still(bits):
    """With every code written and read at one scale the update is the fixed-scale one,
    eps (z_i + z_j') / 2, and the pair's sum is eps (z_i + z_j) exactly."""
    n, d, eps = 6, 64, 2.0 ** -3
    gen = np.random.Generator(np.random.PCG64(bits))
    X = (gen.standard_normal((n, d)) * 0.1).astype(np.float32)
    pairs = [(0, 3), (4, 1)]
    g = global_oracle(n, d, bits, eps, X=X)
    f = SwarmOracle(n, d, wl.complete_graph(n), bits, eps, 0, 0.0, 0, 0, state_dtype=np.float32)
    f.X[:] = X
    g.gossip_round(pairs)
    f.gossip_round(pairs)
    assert np.array_equal(g.X, f.X)                    # eps z / 2 is exact in float32 here
    assert g.decode_failures == 0 and [bytes(a) for a in g.ring[0]] == [bytes(a) for a in f.ring[0]]
    for i, j in pairs:
        zi = lattice_points(g, 0, i, X[i], eps)
        zj = lattice_points(g, 0, j, X[j], eps)
        assert np.array_equal(g.X[i].astype(np.float64) + g.X[j].astype(np.float64), eps * (zi + zj))


def test_global_scale_update_rule_by_hand():
    """eps_(r+1) = max(2^ceil(log2(2 m / (2^(b-1) - 3))), eps_r / 2) with m recomputed from the
    published codes in plain Python; unmatched rounds leave the scale alone."""
    n, d, bits, eps = 4, 32, 8, 2.0 ** -6
    gen = np.random.Generator(np.random.PCG64(11))
    X = (gen.standard_normal((n, d)) * 0.2).astype(np.float32)
    o = global_oracle(n, d, bits, eps, X=X)
    o.gossip_round([])                                  # nobody matched
    assert o.eps_cur == np.float32(eps) and o.round == 1
    before = o.X.copy()
    pairs = [(0, 1), (2, 3)]
    o.gossip_round(pairs)
    m = 0.0
    for i, j in pairs:
        for me, other in ((i, j), (j, i)):
            theirs = lattice_points(o, 0, other, before[me], eps)
            m = max(m, float(np.abs(before[me].astype(np.float64) - eps * theirs).max()))
    assert float(o.max_disagreement) == m
    want = 2.0 ** math.ceil(math.log2(2 * m / (2 ** (bits - 1) - 3)))
    assert want > eps / 2                                # this case exercises the first branch
    assert float(o.eps_cur) == want
    # a pair in full agreement: the scale halves, no faster
    o.X[:] = 0.25
    o.W[:] = 0.25
    e = float(o.eps_cur)
    o.gossip_round(pairs)
    assert float(o.max_disagreement) == 0.0 and float(o.eps_cur) == e / 2


def test_global_scale_recovers_from_a_scale_that_is_too_small_or_too_large():
    """Too small: decodes wrap, the disagreement reads as about the decoding radius and the scale
    grows fourfold per round until the failures stop.  Too large: it halves per round.  Either
    way it settles at the power of two next above 2 (D + eps) / (2^(b-1) - 3), D the largest
    distance between two models (the decoded partner is within eps of the partner)."""
    n, d, bits = 8, 256, 8
    gen = np.random.Generator(np.random.PCG64(5))
    base = gen.standard_normal(d).astype(np.float32)
    spread = 0.5
    for eps0 in (2.0 ** -12, 2.0 ** 6):
        o = global_oracle(n, d, bits, eps0, seed=3)
        history, fails = [], []
        for r in range(22):
            X = (base + gen.uniform(-spread, spread, (n, d))).astype(np.float32)
            o.X[:] = X                                    # keep the spread alive: only the scale moves
            o.W[:] = X
            f0 = o.decode_failures
            o.gossip_round(o.sample_matching())
            history.append(float(o.eps_cur))
            fails.append(o.decode_failures - f0)
        ratios = [b / a for a, b in zip(history, history[1:])]
        if eps0 < 1e-3:
            assert fails[0] > 0 and ratios[0] == 4.0 and ratios[1] == 4.0
        else:
            assert fails[0] == 0 and ratios[0] == 0.5 and ratios[1] == 0.5
        assert all(f == 0 for f in fails[8:])
        D, levels = 2 * spread, 2 ** (bits - 1) - 3
        for e in history[14:]:                            # 2^6 needs 11 halvings to come down
            assert 2 * 0.8 * D / levels <= e <= 2 * 2 * (D + e) / levels


def test_global_scale_stale_read_uses_the_scale_the_code_was_written_with():
    """Round 1 reads the codes of round 0 (age 1) after the scale has moved: the partner's lattice
    point is decoded on the old lattice and averaged with the own point on the new one."""
    n, d, bits, S = 2, 16, 8, 1
    gen = np.random.Generator(np.random.PCG64(2))
    X0 = (gen.standard_normal((n, d)) * 0.05).astype(np.float32)
    o = global_oracle(n, d, bits, 2.0 ** -4, S=S, X=X0)
    o.gossip_round([(0, 1)], stale=[0, 0])
    e0, e1 = 2.0 ** -4, float(o.eps_cur)
    assert e1 == e0 / 2 and o.eps_ring[0] == np.float32(e0)
    X1 = o.X.copy()
    o.gossip_round([(0, 1)], stale=[1, 1])
    assert o.eps_ring[1] == np.float32(e1)
    for me, other in ((0, 1), (1, 0)):
        mine = lattice_points(o, 1, me, X1[me], e1)          # published this round, new scale
        theirs = lattice_points(o, 0, other, X1[me], e0)     # last round's code, its own scale
        assert np.array_equal(o.X[me].astype(np.float64), (e1 * mine + e0 * theirs) / 2)


# ---------------------------------------------------------------- multi-resolution registers
def prefix_oracle(n, d, eps, S=0, seed=0):
    return SwarmOracle(n, d, wl.complete_graph(n), 16, eps, 0, 0.0, S, seed, state_dtype=np.float32, codec="prefix")


def test_prefix_codec_matches_the_short_code_where_it_decodes_and_succeeds_where_it_fails():
    """Close pairs: same update as the fixed 4-bit codec at 4 bits per coordinate read (+ one checksum
    per tile).  A pair too far apart for 4 bits: the fixed codec averages with a wrapped value, the
    prefix reader goes on to 8 bits for those tiles and decodes the sender's point."""
    n, d, eps = 4, 2048, 2.0 ** -4
    gen = np.random.Generator(np.random.PCG64(21))
    X = (gen.standard_normal((1, d)) + gen.uniform(-0.1, 0.1, (n, d))).astype(np.float32)
    X[3, 512:1024] += 1.5                                     # 24 cells away on one tile
    pairs = [(0, 1), (2, 3)]
    p, f = prefix_oracle(n, d, eps), SwarmOracle(n, d, wl.complete_graph(n), 4, eps, 0, 0.0, 0, 0, state_dtype=np.float32)
    for o in (p, f):
        o.X[:] = X
        o.gossip_round(pairs)
    assert np.array_equal(p.X[:2], f.X[:2]) and f.decode_failures > 0 and p.decode_failures == 0
    assert not np.array_equal(p.X[2], f.X[2])
    assert np.array_equal(p.X[2], p.X[3])                     # both decodes right: the pair agrees
    assert p.prefix_levels.tolist() == [14, 2, 0] and p.prefix_unconfirmed == 0
    assert p.bits_communicated == 14 * 512 * 4 + 2 * 512 * 8 + 16 * 64
    assert f.bits_communicated == 4 * d * 4


def test_prefix_codec_stale_reads_decode_after_the_models_moved():
    """Reads two rounds old of models that drifted by tens of cells: 4 bits would wrap, the reader
    confirms at 8 bits; nothing is left unconfirmed and the levels account for every tile read."""
    n, d, eps, S = 6, 1024, 2.0 ** -5, 2
    gen = np.random.Generator(np.random.PCG64(22))
    o = prefix_oracle(n, d, eps, S=S, seed=5)
    base = gen.standard_normal(d).astype(np.float32)
    published = []
    for r in range(5):
        X = (base + r * 0.4 + gen.uniform(-0.05, 0.05, (n, d))).astype(np.float32)     # 12.8 cells per round
        o.X[:] = X
        published.append(X.copy())
        pairs = [(0, 1), (2, 3), (4, 5)] if r % 2 == 0 else [(1, 2), (3, 4)]
        stale = np.full(n, min(r, S))
        before = o.prefix_levels.copy()
        o.gossip_round(pairs, stale)
        used = o.prefix_levels - before
        assert used.sum() == 2 * len(pairs) * (d // 512)
        if r == 0:
            assert used.tolist() == [used.sum(), 0, 0]
        else:
            assert used[0] == 0 and used[1] == used.sum()     # 12.8 or 25.6 cells: beyond 4 bits, inside 8
        for i, j in pairs:                                    # each node averaged its point with the partner's old one
            age = min(r, S)
            old = published[r - age]
            for me, other in ((i, j), (j, i)):
                assert np.abs(o.X[me] - 0.5 * (X[me] + old[other])).max() <= 1.5 * eps
    assert o.prefix_unconfirmed == 0 and o.decode_failures == 0


def test_global_scale_adds_the_pending_local_steps_on_top_of_the_average():
    """Deferred apply under the per-round scale: X_i' = average + (W_i - X_i), as under the fixed one."""
    n, d, eps = 4, 64, 2.0 ** -5
    gen = np.random.Generator(np.random.PCG64(31))
    X = (gen.standard_normal((n, d)) * 0.1).astype(np.float32)
    plain, stepped = global_oracle(n, d, 8, eps, X=X), global_oracle(n, d, 8, eps, X=X)
    step = (gen.standard_normal(d) * 0.01).astype(np.float32)
    stepped.W[0] = X[0] + step
    stepped.pending[0] = True
    for o in (plain, stepped):
        o.gossip_round([(0, 1), (2, 3)])
    assert np.allclose(stepped.X[0], plain.X[0].astype(np.float64) + (stepped.W[0].astype(np.float64) - X[0]), atol=1e-7)
    assert np.array_equal(stepped.X[1:], plain.X[1:]) and stepped.eps_cur == plain.eps_cur


def test_prefix_codec_counts_tiles_that_no_level_confirms():
    n, d, eps = 2, 1024, 2.0 ** -6
    gen = np.random.Generator(np.random.PCG64(32))
    o = prefix_oracle(n, d, eps)
    o.X[:] = (gen.standard_normal((1, d)) + gen.uniform(-0.01, 0.01, (n, d))).astype(np.float32)
    o.X[1, 600] += 40000 * eps                               # beyond the 16-bit radius, second tile only
    o.gossip_round([(0, 1)])
    assert o.prefix_unconfirmed == 2 and o.prefix_levels.tolist() == [2, 0, 2] and o.decode_failures == 2


def test_algorithm1_with_prefix_registers():
    """One step of Algorithm 1 where the initiator reads the responder's multi-resolution register:
    same update as with 8-bit registers where 8 bits decode; the tile that is 24 cells away costs
    8 bits per coordinate to read and as many to write the average back, the others 4."""
    n, d, eps = 3, 1024, 2.0 ** -4
    gen = np.random.Generator(np.random.PCG64(41))
    X = (gen.standard_normal((1, d)) + gen.uniform(-0.1, 0.1, (n, d))).astype(np.float32)
    X[1, 512:] += 1.5
    p = SwarmOracle(n, d, wl.complete_graph(n), 16, eps, 0, 0.0, 0, 4, state_dtype=np.float32, codec="prefix")
    f = SwarmOracle(n, d, wl.complete_graph(n), 8, eps, 0, 0.0, 0, 4, state_dtype=np.float32)
    for o in (p, f):
        o.X[:] = X
        o.Xhat[:] = X
        o.W[0] = X[0] + 0.01
        o.pending[0] = True
        o.interact(0, 1)
    assert np.array_equal(p.X, f.X) and np.array_equal(p.Xhat, f.Xhat) and p.decode_failures == 0 == f.decode_failures
    assert np.array_equal(p.X[0] - np.float32(0.01), p.X[1]) or np.allclose(p.X[0] - 0.01, p.X[1], atol=1e-6)
    assert p.prefix_levels.tolist() == [1, 1, 0]
    assert p.bits_communicated == 2 * (512 * 4 + 512 * 8 + 2 * 64) and f.bits_communicated == 2 * d * 8

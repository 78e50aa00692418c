"""Objective data of the synthetic workloads, float32, seeded (numpy PCG64)."""
import numpy as np

# The five workload configurations (shapes follow the paper's experiments:
# 8..256 nodes, ResNet-50- and Transformer-sized flat models, H = 2..5, 8-bit codes).
CONFIGS = {
    1: dict(n=8, d=4096, graph="complete", objective="lsq", m_rows=256, batch=32, H=2, lr=0.05,
            bits=8, stale_max=0, mode="sequential", steps=200, shift_sigma=0.1),
    2: dict(n=64, d=1 << 20, graph="torus8x8", objective="diag", a_law="uniform", a_lo=0.5, a_hi=2.0,
            shift_sigma=1.0, sigma=0.1, H=3, lr=0.1, bits=8, stale_max=0, mode="rounds", steps=500),
    3: dict(n=256, d=1024 * 4096 + 4096 + 4096 * 1024 + 1024, graph="regular8", objective="mlp",
            n_in=1024, n_hid=4096, n_out=1024, data_sigma=0.5, alpha=0.5, batch=128, H=2, lr=0.02,
            bits=8, stale_max=0, mode="rounds"),
    4: dict(n=64, d=25_600_000, graph="regular4", objective="diag", a_law="uniform", a_lo=0.5, a_hi=2.0,
            shift_sigma=1.0, sigma=0.05, H=3, lr=0.1, bits=4, stale_max=1, stale="fixed1", mode="rounds"),
    5: dict(n=32, d=110_000_000, graph="complete", objective="diag", a_law="loguniform", a_lo=0.1,
            a_hi=10.0, shift_sigma=2.0, sigma=0.1, H=5, lr=0.1, bits=8, stale_max=2, stale="uniform",
            mode="rounds", steps=100),
}


def diag_quadratic_data(n, d, seed, a_law="uniform", a_lo=0.5, a_hi=2.0, shift_sigma=1.0):
    """a_ik ~ U[a_lo, a_hi] (or log-uniform), c_ik ~ N(mu_i, 1), mu_i ~ N(0, shift_sigma^2)."""
    gen = np.random.Generator(np.random.PCG64(seed))
    u = gen.random((n, d), dtype=np.float32)
    if a_law == "uniform":
        a = a_lo + (a_hi - a_lo) * u
    else:
        a = np.exp(np.log(a_lo) + (np.log(a_hi) - np.log(a_lo)) * u)
    mu = shift_sigma * gen.standard_normal(n).astype(np.float32)
    c = mu[:, None] + gen.standard_normal((n, d), dtype=np.float32)
    return a.astype(np.float32), c.astype(np.float32)


def least_squares_data(n, d, m_rows, seed, shift_sigma=0.1):
    """A_i ~ N(0, 1/d), b_i = A_i (x* + delta_i), x* ~ N(0, I), delta_i ~ N(0, shift_sigma^2 I)."""
    gen = np.random.Generator(np.random.PCG64(seed))
    A = (gen.standard_normal((n, m_rows, d), dtype=np.float32) / np.float32(np.sqrt(d)))
    xstar = gen.standard_normal(d, dtype=np.float32)
    delta = np.float32(shift_sigma) * gen.standard_normal((n, d), dtype=np.float32)
    b = np.einsum("nmd,nd->nm", A.astype(np.float64), (xstar[None, :] + delta).astype(np.float64))
    return A.astype(np.float32), b.astype(np.float32), xstar


def mixture_data(n, n_in, n_out, seed, alpha=0.5):
    """Class means ~ N(0, I); per-node label law ~ Dirichlet(alpha), returned as a float32 CDF."""
    gen = np.random.Generator(np.random.PCG64(seed))
    means = gen.standard_normal((n_out, n_in), dtype=np.float32)
    law = gen.dirichlet(np.full(n_out, alpha), size=n)
    cdf = np.cumsum(law, axis=1)
    cdf[:, -1] = 1.0
    return means, cdf.astype(np.float32)

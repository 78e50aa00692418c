"""Shared helpers of the GPU parity tests: build the oracle and the HIP swarm from one
configuration and force the oracle's state into the device ("teacher forcing")."""
import numpy as np

from oracle.swarm import SwarmOracle

TOL_ELEMENTWISE = 1e-6     # averaging and elementwise updates (float32 path vs float64 oracle)
# Where float32 local steps feed the averaging there are two float32 stages between the uploaded state and
# the compared model: the H steps (each update w <- w - eta g rounds once, relative 6e-8 each, and the
# gradient's own roundings enter scaled by eta <= 0.1) and then delta = w - x and average + delta (two more
# roundings).  Each stage stays within the 1e-6 bound on its own; their sum is compared at twice that.
TOL_TWO_STAGE = 2 * TOL_ELEMENTWISE
TOL_GEMM = 1e-4            # GEMM-based gradients


def close(gpu, cpu, tol):
    """|gpu - cpu| <= tol * max(1, |cpu|) elementwise (relative error is ill-defined near 0)."""
    gpu = np.asarray(gpu, dtype=np.float64)
    cpu = np.asarray(cpu, dtype=np.float64)
    return np.abs(gpu - cpu) <= tol * np.maximum(1.0, np.abs(cpu))


def assert_close(gpu, cpu, tol, what=""):
    ok = close(gpu, cpu, tol)
    if not ok.all():
        bad = np.argwhere(~ok)
        idx = tuple(bad[0])
        raise AssertionError(f"{what}: {(~ok).sum()} of {ok.size} entries differ, first at {idx}: "
                             f"gpu={np.asarray(gpu)[idx]!r} cpu={np.asarray(cpu)[idx]!r}")


def make_both(swarm_mod, n, d, edges, bits, eps, H, lr, stale_max=0, seed=0, inplace=False, geometric=False, pair_scale=False,
              global_scale=False, prefix=False):
    gpu = swarm_mod.Swarm(n, d, edges, bits, eps, H, lr, stale_max, seed,
                          apply_mode=swarm_mod.INPLACE if inplace else swarm_mod.DEFERRED,
                          steps_law=swarm_mod.GEOMETRIC if geometric else swarm_mod.CONSTANT,
                          scale_policy=(swarm_mod.SCALE_PAIR_LINF if pair_scale else
                                        swarm_mod.SCALE_GLOBAL_LINF if global_scale else swarm_mod.SCALE_FIXED),
                          codec=swarm_mod.CODEC_PREFIX if prefix else swarm_mod.CODEC_FIXED)
    cpu = SwarmOracle(n, d, edges, bits, eps, H, lr, stale_max, seed,
                      apply_mode="inplace" if inplace else "deferred",
                      steps_law="geometric" if geometric else "constant",
                      scale_policy="pair_linf" if pair_scale else "global_linf" if global_scale else "fixed",
                      codec="prefix" if prefix else "fixed")
    return gpu, cpu


def force_state(swarm_mod, gpu, cpu):
    """Upload the oracle's X, and W of the nodes with pending local steps."""
    gpu.write_models(swarm_mod.COMM, cpu.X)
    for i in np.flatnonzero(cpu.pending):
        gpu.write_models(swarm_mod.LIVE, cpu.W[i:i + 1], node0=int(i))


def ring_row(cpu, node, age=0):
    depth = cpu.S + 1
    last = (cpu.round - 1) % depth if cpu.round else 0
    return cpu.ring[(last - age) % depth][node]


def disjoint_prefix(c, limit):
    """How many of the oracle's next interactions touch pairwise disjoint nodes (without stepping it)."""
    t0, used, k = c.interactions, set(), 0
    try:
        while k < limit:
            c.interactions = t0 + k
            i, j = c.sample_pair()
            if i in used or j in used:
                break
            used |= {i, j}
            k += 1
    finally:
        c.interactions = t0
    return k

"""Writes tests/golden/oracle_small_case.json: what the oracle computes for one small, fully seeded
case (random words, rounding thresholds, noise, a matching, two rounds with local steps, stale
reads and 4-bit codes, one round with multi-resolution registers).  It calls nothing but oracle/
and workloads/; tests compare the oracle (exactly for integers, 1e-12 for floats) and the GPU
library (to its tolerances) with the stored values, so an unintended change of the oracle's
arithmetic shows up as a diff of this file.

    python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import workloads as wl                                   # noqa: E402
from oracle import quantizer as qz                       # noqa: E402
from oracle import rng                                   # noqa: E402
from oracle.objectives import DiagQuadratic              # noqa: E402
from oracle.swarm import SwarmOracle                     # noqa: E402

CASE = dict(n=6, d=24, bits=4, eps=0.25, H=2, lr=0.1, S=1, seed=20240, sigma=0.05)


def run_case(codec="fixed"):
    c = CASE
    edges = wl.torus_graph(2, 3)
    a, cc = wl.diag_quadratic_data(c["n"], c["d"], 5)
    o = SwarmOracle(c["n"], c["d"], edges, 16 if codec == "prefix" else c["bits"], c["eps"], c["H"], c["lr"], c["S"],
                    c["seed"], codec=codec)
    o.objective = DiagQuadratic(a, cc, c["sigma"])
    gen = np.random.Generator(np.random.PCG64(c["seed"]))
    o.X[:] = (gen.standard_normal((c["n"], c["d"])) * 0.5).astype(np.float32)
    rounds = []
    for r in range(2):
        pairs = o.sample_matching()
        stale = o.sample_stale()
        o.local_steps()
        o.gossip_round(pairs, stale)
        slot = r % (c["S"] + 1)
        rounds.append(dict(pairs=pairs.tolist(), stale=stale.tolist(),
                           registers=[bytes(o.ring[slot][i]).hex() for i in range(c["n"])],
                           X=[[float(v) for v in row] for row in o.X]))
    return o, rounds


def build():
    c = CASE
    words = rng.stream(c["seed"], rng.TAG_SR, 0, 3, 7, np.arange(2))
    o, rounds = run_case()
    p, prefix_rounds = run_case("prefix")
    return dict(case=c,
                philox_words=[[int(w[k]) for w in words] for k in range(2)],
                rounding_halves=[int(v) for v in rng.sr_halves(c["seed"], 3, 7, 0, 16)],
                noise=[float(v) for v in rng.noise_normals(c["seed"], 3, 7, 1, 0, 8)],
                rounds=rounds, decode_failures=int(o.decode_failures), bits_communicated=int(o.bits_communicated),
                potential=float(o.potential()),
                prefix_rounds=prefix_rounds, prefix_levels=[int(v) for v in p.prefix_levels],
                prefix_bits_communicated=int(p.bits_communicated))


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_small_case.json")
    with open(path, "w") as f:                     # one top-level key per line
        items = [f' {json.dumps(k)}: {json.dumps(v, separators=(",", ":"))}' for k, v in build().items()]
        f.write("{\n" + ",\n".join(items) + "\n}\n")
    print("wrote", path)

"""The stored small case (tests/golden/oracle_small_case.json, written by tests/golden/make_golden.py
from the oracle alone): the oracle still computes it, and the GPU library reproduces it."""
import importlib.util
import json
import os

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def load():
    with open(os.path.join(HERE, "golden", "oracle_small_case.json")) as f:
        stored = json.load(f)
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return stored, mod


def same(a, b, path=""):
    if isinstance(a, dict):
        assert a.keys() == b.keys(), path
        for k in a:
            same(a[k], b[k], f"{path}/{k}")
    elif isinstance(a, list):
        assert len(a) == len(b), path
        for i, (x, y) in enumerate(zip(a, b)):
            same(x, y, f"{path}[{i}]")
    elif isinstance(a, float):
        assert a == pytest.approx(b, rel=0, abs=1e-12), path
    else:
        assert a == b, path


def test_oracle_reproduces_the_stored_case():
    stored, mod = load()
    same(mod.build(), stored)


@pytest.mark.gpu
@pytest.mark.parametrize("codec", ["fixed", "prefix"])
def test_gpu_reproduces_the_stored_case(gpu, codec):
    import torch
    import workloads as wl
    from helpers import TOL_ELEMENTWISE, assert_close
    stored, mod = load()
    c = stored["case"]
    edges = wl.torus_graph(2, 3)
    a, cc = wl.diag_quadratic_data(c["n"], c["d"], 5)
    g = gpu.Swarm(c["n"], c["d"], edges, 16 if codec == "prefix" else c["bits"], c["eps"], c["H"], c["lr"], c["S"], c["seed"],
                  codec=gpu.CODEC_PREFIX if codec == "prefix" else gpu.CODEC_FIXED)
    g.set_objective_diag(torch.from_numpy(a).cuda(), torch.from_numpy(cc).cuda(), c["sigma"])
    gen = np.random.Generator(np.random.PCG64(c["seed"]))
    X = (gen.standard_normal((c["n"], c["d"])) * 0.5).astype(np.float32)
    rounds = stored["prefix_rounds" if codec == "prefix" else "rounds"]
    for r, want in enumerate(rounds):
        g.write_models(gpu.COMM, X)                          # the stored state goes in: nothing drifts
        assert g.sample_matching().tolist() == want["pairs"] and g.sample_stale().tolist() == want["stale"]
        g.local_steps()
        g.gossip_round(None, np.array(want["stale"], dtype=np.uint8))
        for i in range(c["n"]):
            assert g.read_codes(i).tobytes().hex() == want["registers"][i], f"register of node {i}, round {r}"
        X = np.array(want["X"], dtype=np.float64)
        assert_close(g.read_models(gpu.COMM), X, 2 * TOL_ELEMENTWISE, f"X after round {r}")
        X = X.astype(np.float32)
    cnt = g.counters()
    if codec == "prefix":
        assert g.prefix_stats()[0] == stored["prefix_levels"] and cnt["bits_communicated"] == stored["prefix_bits_communicated"]
    else:
        assert cnt["decode_failures"] == stored["decode_failures"] and cnt["bits_communicated"] == stored["bits_communicated"]
        assert g.potential() == pytest.approx(stored["potential"], rel=1e-5)

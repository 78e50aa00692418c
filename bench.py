#!/usr/bin/env python3
"""Benchmark of one swarm interaction round on one MI355X.

A step is one pass of the whole hot path over the synthetic swarm of the headline
workload (n = 64 nodes on a random 4-regular graph, d = 25.6 M float32 parameters,
diagonal-quadratic objectives with gradient noise 0.05, H = 3 local steps, 4-bit codes,
every read one round stale): H local steps on every node, the round's random maximal
matching, the fused quantized gossip pass over the matched pairs, and the unmatched
nodes' own updates.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
# HBM bytes per pair-coordinate of the fused gossip pass from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs,
# scaled by the stream-copy calibration (17.00 B fetched + 8.99 B written at 4-bit codes, stale reads).
MEASURED_TRAFFIC_PER_PAIR_COORDINATE = {(4, True): 25.99}


def algorithmic_bytes_per_pair_coordinate(bits, stale, delta=True):
    """Fused gossip pass: read X_i, X_j (+ W_i, W_j when local steps are pending), write
    X_i', X_j', write two b-bit codes, read two b-bit stale codes when the reads are stale."""
    return 8 + (8 if delta else 0) + 8 + 2 * bits / 8 + (2 * bits / 8 if stale else 0)


def build_workload(cfg_id, scale_d=None):
    import numpy as np
    import torch
    import workloads as wl
    cfg = dict(wl.CONFIGS[cfg_id])
    if scale_d:
        cfg["d"] = scale_d
    n, d = cfg["n"], cfg["d"]
    if cfg["graph"] == "regular4":
        edges = wl.random_regular_graph(n, 4, 0)
    elif cfg["graph"] == "regular8":
        edges = wl.random_regular_graph(n, 8, 0)
    elif cfg["graph"] == "torus8x8":
        edges = wl.torus_graph(8, 8)
    elif cfg["graph"] == "complete":
        edges = wl.complete_graph(n)
    else:
        raise SystemExit(f"bench: graph {cfg['graph']} not supported here")
    if cfg["objective"] == "mlp":
        means, cdf = wl.mixture_data(n, cfg["n_in"], cfg["n_out"], 0, cfg["alpha"])
        return cfg, edges, torch.from_numpy(means).cuda(), torch.from_numpy(cdf).cuda()
    gen = torch.Generator(device="cuda")
    gen.manual_seed(0)
    # a ~ U[lo, hi] (or log-uniform), c ~ N(mu_i, 1), mu_i ~ N(0, shift^2): generated on the device, row by row
    a = torch.empty((n, d), dtype=torch.float32, device="cuda")
    c = torch.empty((n, d), dtype=torch.float32, device="cuda")
    mu = torch.randn(n, generator=gen, device="cuda") * cfg["shift_sigma"]
    lo, hi = cfg["a_lo"], cfg["a_hi"]
    for i in range(n):
        a[i].uniform_(0.0, 1.0, generator=gen)
        if cfg["a_law"] == "uniform":
            a[i].mul_(hi - lo).add_(lo)
        else:
            a[i].mul_(float(np.log(hi) - np.log(lo))).add_(float(np.log(lo))).exp_()
        c[i].normal_(0.0, 1.0, generator=gen).add_(mu[i])
    torch.cuda.synchronize()
    return cfg, edges, a, c


def eps_for(cfg):
    # power of two so that the decoding radius (2^(b-1) - 5/2) eps covers the usual disagreement
    if cfg["objective"] == "mlp":
        return 2.0 ** -10          # weights of order 0.02: radius 125 eps = 0.12
    if cfg["shift_sigma"] >= 2.0:
        return 0.25                # strongly heterogeneous nodes sit several units apart
    return 0.5 if cfg["bits"] == 4 else 2.0 ** -4


def stale_plan(cfg, swarm_obj):
    import numpy as np
    if cfg["stale_max"] == 0:
        return None
    if cfg.get("stale") == "fixed1":
        return np.ones(cfg["n"], dtype=np.uint8)
    return swarm_obj.sample_stale()


def cpu_baseline(cfg, edges, a, c, eps, seconds_target=15.0):
    """The oracle as it stands, timed on the host: one round on a column window of the same
    workload, scaled to the full dimension."""
    import numpy as np
    from oracle.objectives import DiagQuadratic
    from oracle.swarm import SwarmOracle
    n, d = cfg["n"], cfg["d"]
    if cfg["objective"] == "mlp":
        return cpu_baseline_mlp(cfg, edges, a, c, eps)
    width = 1 << 14
    result = None
    while True:
        k1 = min(width, d - d % 8)
        o = SwarmOracle(n, d, edges, cfg["bits"], eps, cfg["H"], cfg["lr"], cfg["stale_max"], 0, k0=0, k1=k1)
        o.objective = DiagQuadratic(a[:, :k1].cpu().numpy(), c[:, :k1].cpu().numpy(), cfg["sigma"], k0=0)
        o.local_steps()
        o.gossip_round(o.sample_matching())           # round 0 fills the ring so that round 1 can read stale codes
        t0 = time.perf_counter()
        o.local_steps()
        pairs = o.sample_matching()
        stale = np.minimum(1, o.round) * np.ones(n, dtype=np.int64) if cfg["stale_max"] else None
        o.gossip_round(pairs, stale)
        dt = time.perf_counter() - t0
        result = dict(value=len(pairs) / (dt * d / k1), unit="interactions/s", cores=1, kind="oracle",
                      sample=f"1 full round (local steps + matching + gossip) on columns [0,{k1}) of d={d}, "
                             f"all {n} nodes, {dt:.2f} s, scaled by d/{k1}")
        if dt >= seconds_target / 4 or k1 >= d - d % 8 or width >= 1 << 22:
            return result
        width *= 4


def cpu_baseline_mlp(cfg, edges, means, cdf, eps):
    """The MLP objective needs whole models: time the oracle's local steps on two nodes and one
    pairwise gossip of full rows, and scale to the whole swarm (n nodes, n/2 pairs)."""
    import numpy as np
    from oracle.objectives import MixtureMLP
    from oracle.swarm import SwarmOracle
    n, d = cfg["n"], cfg["d"]
    sub = 2
    o = SwarmOracle(sub, d, [(0, 1)], cfg["bits"], eps, cfg["H"], cfg["lr"], 0, 0)
    o.objective = MixtureMLP(cfg["n_in"], cfg["n_hid"], cfg["n_out"], means.cpu().numpy(), cdf.cpu().numpy()[:sub],
                             cfg["data_sigma"], cfg["batch"])
    o.X[:] = 0.02 * np.random.Generator(np.random.PCG64(0)).standard_normal(d).astype(np.float32)
    t0 = time.perf_counter()
    o.local_steps()
    o.gossip_round([(0, 1)])
    dt = time.perf_counter() - t0
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return dict(value=1.0 / dt, unit="interactions/s", cores=threads, kind="oracle",
                sample=f"2 of {n} nodes: H local MLP steps each (numpy float64 GEMMs, BLAS threads) + 1 pairwise "
                       f"gossip of full rows, {dt:.2f} s; a round of the whole swarm is {n // 2} such units")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=4, help="workload configuration (2, 3, 4 or 5)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--d", type=int, default=None, help="override the model dimension (debugging only)")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py: this build simulates the whole swarm on ONE GPU; --gpus must be 1 "
                         "(no collectives or sharding across GPUs are part of it)")
    import numpy as np
    import torch
    import paper_1910_12308_amd as swarm

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    cfg, edges, a, c = build_workload(args.config, args.d)
    n, d, bits = cfg["n"], cfg["d"], cfg["bits"]
    eps = eps_for(cfg)
    s = swarm.Swarm(n, d, edges, bits, eps, cfg["H"], cfg["lr"], cfg["stale_max"], seed=0)
    if cfg["objective"] == "mlp":
        x0 = 0.02 * torch.randn(d, device="cuda", generator=torch.Generator(device="cuda").manual_seed(1))
        s.close()
        s = swarm.Swarm(n, d, edges, bits, eps, cfg["H"], cfg["lr"], cfg["stale_max"], seed=0, x0=x0)
        s.set_objective_mlp(cfg["n_in"], cfg["n_hid"], cfg["n_out"], a, c, cfg["data_sigma"], cfg["batch"])
    else:
        s.set_objective_diag(a, c, cfg["sigma"])

    def step():
        s.local_steps()
        s.gossip_round(None, stale_plan(cfg, s))

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    before = s.counters(raise_on_range=False)
    s.timing_reset()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    after = s.counters(raise_on_range=False)
    times = s.kernel_times()
    interactions = after["interactions"] - before["interactions"]

    # Roofline of the dominant kernel (the fused gossip pass): algorithmic bytes / measured kernel time.
    stale = cfg["stale_max"] > 0 and cfg.get("stale") == "fixed1"
    per_pc = algorithmic_bytes_per_pair_coordinate(bits, stale)
    if cfg.get("stale") == "uniform":                 # each read is stale with probability S/(S+1) after warm-up
        per_pc = algorithmic_bytes_per_pair_coordinate(bits, False) + (2 * bits / 8) * cfg["stale_max"] / (cfg["stale_max"] + 1)
    gossip_bytes = per_pc * d * interactions
    gossip_s = times["gossip_ms"] * 1e-3
    achieved = gossip_bytes / gossip_s / 1e9 if gossip_s > 0 else 0.0
    local_bytes = 16.0 * d * n * times["local_calls"]
    local_gbs = local_bytes / (times["local_ms"] * 1e-3) / 1e9 if times["local_ms"] > 0 else 0.0
    mlp = None
    if cfg["objective"] == "mlp":
        # 5 GEMMs of 2*batch*in*hid (= 2*batch*hid*out here) flops per node and local step
        flops = 5 * 2.0 * cfg["batch"] * cfg["n_in"] * cfg["n_hid"] * n * cfg["H"] * times["local_calls"]
        mlp = flops / (times["local_ms"] * 1e-3) / 1e12

    out = {
        "metric": "node-interactions/sec + gossip-avg HBM GB/s (% of peak), n=64 d=25.6M",
        "value": interactions / dt,
        "unit": "interactions/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"config {args.config}: n={n} d={d} graph={cfg['graph']} {cfg['objective']} "
                               f"sigma={cfg.get('sigma', cfg.get('data_sigma'))} H={cfg['H']} lr={cfg['lr']} bits={bits} "
                               f"stale_max={cfg['stale_max']} ({cfg.get('stale', 'fresh')}) eps={eps}",
                   "pairs_per_round": interactions / args.steps,
                   "decode_failures": after["decode_failures"] - before["decode_failures"],
                   "gossip_ms_per_round": times["gossip_ms"] / max(1, times["gossip_calls"]),
                   "local_steps_ms_per_round": times["local_ms"] / max(1, times["local_calls"]),
                   "local_steps_GBps": None if mlp is not None else local_gbs,
                   "local_steps_mfma_f32_TFLOPs": mlp,
                   "local_steps_mfma_frac_of_157.3": None if mlp is None else mlp / 157.3},
        "roofline": {"kernel": "gossip_pairs_kernel (fused quantize/exchange/decode/average)",
                     "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": (MEASURED_TRAFFIC_PER_PAIR_COORDINATE[(bits, stale)] * d * interactions
                                 / max(1, times["gossip_calls"])
                                 if (bits, stale) in MEASURED_TRAFFIC_PER_PAIR_COORDINATE else None),
                     "traffic_unit": "bytes per launch (counters, calibrated on the stream copy)",
                     "achieved_bytes_per_launch": gossip_bytes / max(1, times["gossip_calls"]),
                     "bytes_per_pair_coordinate": per_pc},
    }
    # Measured ceiling: a plain streaming copy kernel over one model matrix worth of bytes.
    src, dst = s.models_view(swarm.COMM), s.models_view(swarm.LIVE)   # W is rebuilt by every step
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    swarm.stream_copy(dst, src)
    ev0.record()
    for _ in range(5):
        swarm.stream_copy(dst, src)
    ev1.record()
    torch.cuda.synchronize()
    copy_gbs = 2.0 * src.numel() * 4 * 5 / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
    out["roofline"]["copy_kernel_GBps"] = copy_gbs
    out["roofline"]["frac_of_copy"] = achieved / copy_gbs
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, edges, a, c, eps)
    print(json.dumps(out))


if __name__ == "__main__":
    main()

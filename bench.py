#!/usr/bin/env python3
"""Benchmark of one swarm interaction round on one MI355X.

A step is one pass of the whole hot path over the synthetic swarm of the headline
workload (n = 64 nodes on a random 4-regular graph, d = 25.6 M float32 parameters,
diagonal-quadratic objectives with gradient noise 0.05, H = 3 local steps, 4-bit codes,
every read one round stale): H local steps on every node, the round's random maximal
matching, the quantized gossip pass over the matched pairs, and the unmatched nodes' own
updates.  For per-coordinate objectives the library runs all of it in one kernel pass
(swarm_round_fused, bit-identical to swarm_local_steps + swarm_gossip_round); that is the
timed step, and the two-call variant is measured after it and reported in the same line.
After the headline's timed region the other workload configurations (2, 5, 3, 1 and
Algorithm 1 at the headline's shape) run a few steps each and are reported in a compact
"configs" block of the same line.  Prints ONE JSON line.
"""
import argparse
import json
import os
import subprocess
import sys
import tempfile
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_F32_PEAK_TFLOPS = 157.3   # MI355X published dense fp32 matrix rate
MFMA_BF16_PEAK_TFLOPS = 2500.0 # MI355X published dense bf16 matrix rate
# HBM bytes per pair-coordinate from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs scaled by the stream-copy
# calibration (see profiles/), at 4-bit codes with stale reads: key = (kernel, bits, stale).
MEASURED_TRAFFIC_PER_PAIR_COORDINATE = {("gossip", 4, True): 25.99, ("round", 4, True): 33.99}
BOX_CPU_SHARE = 16             # host cores a one-GPU machine grants, whatever os.cpu_count() shows
# Vector-ALU side of the one-pass round at 8-bit codes with gradient noise: vector instructions a wave issues per
# 512-coordinate tile of one node, from the rocprofv3 SQ_INSTS_VALU / SQ_WAVES runs at H = 3 and H = 5 under
# profiles/ (fused_nodes_kernel 647 / 889, fused_pairs_kernel 1276 / 1760 per pair): 121 per local step and, taking
# the smaller of the two kernels' figures, 275 that do not depend on H.
VALU_PER_NODE_TILE_8BIT = (275.0, 121.0)
# 256 compute units x 4 SIMDs x 16 lanes x 2.4 GHz: lane-operations per second the vector ALUs can issue
VALU_PEAK_TLANEOPS = 256 * 4 * 16 * 2.4e9 / 1e12


def algorithmic_bytes_per_pair_coordinate(kernel, bits, stale_fraction, inplace=False, prefix=False):
    """Gossip pass: read X_i, X_j, W_i, W_j (16 B), write X_i', X_j' (8 B), write two b-bit codes, read
    two b-bit partner codes when the reads are stale.  One-pass round (local steps inside the gossip
    pass): read X, a, c of both nodes (24 B) instead of X and W; W never moves.  Multi-resolution
    registers: 16 bits and 8/512 B of checksum written per coordinate, 4 bits and the checksum read by a
    stale reader (tiles that escalate to 8 or 16 bits are added by the caller from the library's counts)."""
    reads = (8 if inplace else 16) if kernel == "gossip" else 24    # in-place apply: no second matrix to read
    if prefix:
        return reads + 8 + 2 * (2 + 8 / 512) + stale_fraction * 2 * (0.5 + 8 / 512)
    return reads + 8 + 2 * bits / 8 + stale_fraction * 2 * bits / 8


def unmatched_bytes_per_node_coordinate(kernel, bits, inplace=False):
    """An unmatched node of the one-pass round reads X, a, c and writes X (16 B) and its b-bit code; in the
    gossip pass it reads X and W and writes X (12 B; 4 B read for the code alone without pending steps)."""
    return (16 if kernel == "round" else (4 if inplace else 12)) + bits / 8


def build_workload(cfg_id, scale_d=None, steps_H=None):
    import numpy as np
    import torch
    import workloads as wl
    cfg = dict(wl.CONFIGS[cfg_id])
    if scale_d:
        cfg["d"] = scale_d
    if steps_H:
        cfg["H"] = steps_H
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
    if cfg["objective"] == "lsq":
        A, b, _ = wl.least_squares_data(n, d, cfg["m_rows"], 0, cfg["shift_sigma"])
        return cfg, edges, torch.from_numpy(A).cuda(), torch.from_numpy(b).cuda()
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
    if cfg["objective"] == "lsq":
        return 2.0 ** -6
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


# ---------------------------------------------------------------------------- the oracle beside it
def oracle_round_on_window(cfg, edges, a_win, c_win, eps, k0, k1):
    """Seconds the oracle takes for one full round (local steps + matching + gossip) on columns [k0, k1)."""
    import numpy as np
    from oracle.objectives import DiagQuadratic
    from oracle.swarm import SwarmOracle
    n, d = cfg["n"], cfg["d"]
    o = SwarmOracle(n, d, edges, cfg["bits"], eps, cfg["H"], cfg["lr"], cfg["stale_max"], 0, k0=k0, k1=k1,
                    codec=cfg.get("codec", "fixed"))
    o.objective = DiagQuadratic(a_win, c_win, cfg["sigma"], k0=k0)
    o.local_steps()
    o.gossip_round(o.sample_matching())           # round 0 fills the ring so that round 1 can read stale codes
    t0 = time.perf_counter()
    o.local_steps()
    pairs = o.sample_matching()
    stale = np.minimum(1, o.round) * np.ones(n, dtype=np.int64) if cfg["stale_max"] else None
    o.gossip_round(pairs, stale)
    return time.perf_counter() - t0, len(pairs)


def cpu_worker(path):
    """Child process of the all-cores leg: the oracle's round on this worker's column window."""
    import numpy as np
    job = np.load(path, allow_pickle=False)
    cfg = json.loads(str(job["cfg"]))
    dt, pairs = oracle_round_on_window(cfg, job["edges"], job["a"], job["c"], float(job["eps"]), int(job["k0"]), int(job["k1"]))
    print(json.dumps({"seconds": dt, "pairs": pairs}))


def cpu_baseline(cfg, edges, a, c, eps, seconds_target=15.0):
    """The oracle as it stands, timed on the host: one round on a column window of the same
    workload, scaled to the full dimension -- on one core, then with one process per host core, each
    on a window of its own (the oracle itself stays single-threaded)."""
    import numpy as np
    n, d = cfg["n"], cfg["d"]
    host_cores = os.cpu_count() or 1
    if cfg["objective"] == "mlp":
        return cpu_baseline_mlp(cfg, edges, a, c, eps)
    if cfg["objective"] == "lsq":
        return cpu_baseline_sequential(cfg, edges, a, c, eps)
    width = 1 << 14
    while True:
        k1 = min(width, d - d % 8)
        dt, pairs = oracle_round_on_window(cfg, edges, a[:, :k1].cpu().numpy(), c[:, :k1].cpu().numpy(), eps, 0, k1)
        if dt >= seconds_target / 4 or k1 >= d - d % 8 or width >= 1 << 22:
            break
        width *= 4
    result = dict(value=pairs / (dt * d / k1), unit="interactions/s", cores=1, kind="oracle", host_cores=host_cores,
                  sample=f"1 full round (local steps + matching + gossip) on columns [0,{k1}) of d={d}, "
                         f"all {n} nodes, {dt:.2f} s, scaled by d/{k1}")
    # all cores: one child process per core, each running the same oracle round on the next window of k1 columns
    workers = max(1, min(host_cores, BOX_CPU_SHARE, (d - d % 8) // k1))
    if workers > 1:
        with tempfile.TemporaryDirectory() as tmp:
            procs = []
            for w in range(workers):
                k0w = w * k1
                path = os.path.join(tmp, f"job{w}.npz")
                np.savez(path, cfg=json.dumps(cfg), edges=np.asarray(edges), eps=eps, k0=k0w, k1=k0w + k1,
                         a=a[:, k0w:k0w + k1].cpu().numpy(), c=c[:, k0w:k0w + k1].cpu().numpy())
                procs.append(path)
            t0 = time.perf_counter()
            running = [subprocess.Popen([sys.executable, os.path.abspath(__file__), "--cpu-worker", path],
                                        stdout=subprocess.PIPE, text=True,
                                        env=dict(os.environ, OMP_NUM_THREADS="1", OPENBLAS_NUM_THREADS="1"))
                       for path in procs]
            outs = [p.communicate()[0] for p in running]
            wall = time.perf_counter() - t0
        rounds = [json.loads(o.strip().splitlines()[-1]) for o in outs if o.strip()]
        if len(rounds) == workers:
            slowest = max(r["seconds"] for r in rounds)
            result["all_cores"] = dict(value=pairs / (slowest * d / (workers * k1)), unit="interactions/s", cores=workers,
                                       sample=f"{workers} processes, each the same round on its own window of {k1} "
                                              f"columns; slowest {slowest:.2f} s ({wall:.1f} s with start-up), "
                                              f"scaled by d/{workers * k1}")
    return result


def cpu_baseline_sequential(cfg, edges, A, b, eps):
    """Algorithm 1 on the small least-squares workload: the oracle runs the same interactions in full."""
    from oracle.objectives import LeastSquares
    from oracle.swarm import SwarmOracle
    o = SwarmOracle(cfg["n"], cfg["d"], edges, cfg["bits"], eps, cfg["H"], cfg["lr"], 0, 0)
    o.objective = LeastSquares(A.cpu().numpy(), b.cpu().numpy(), cfg["batch"])
    t0 = time.perf_counter()
    for _ in range(cfg["steps"]):
        o.step_sequential()
    dt = time.perf_counter() - t0
    return dict(value=cfg["steps"] / dt, unit="interactions/s", cores=1, kind="oracle", host_cores=os.cpu_count() or 1,
                sample=f"{cfg['steps']} sequential interactions of Algorithm 1 at full size, {dt:.2f} s")


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
    return dict(value=1.0 / dt, unit="interactions/s", cores=threads, kind="oracle", host_cores=os.cpu_count() or 1,
                sample=f"2 of {n} nodes: H local MLP steps each (numpy float64 GEMMs, BLAS threads) + 1 pairwise "
                       f"gossip of full rows, {dt:.2f} s; a round of the whole swarm is {n // 2} such units")


# ---------------------------------------------------------------------------- timing
def measure(torch, s, step, steps, warmup):
    """W untimed steps, then exactly `steps` timed ones between two device synchronisations."""
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    before = s.counters(raise_on_range=False)
    tiles_before = s.prefix_stats()[0]
    s.timing_reset()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    after = s.counters(raise_on_range=False)
    return dict(dt=dt, steps=steps, times=s.kernel_times(), interactions=after["interactions"] - before["interactions"],
                decode_failures=after["decode_failures"] - before["decode_failures"],
                prefix_tiles=[x - y for x, y in zip(s.prefix_stats()[0], tiles_before)])


def roofline(kernel, name, cfg, m, d, inplace=False):
    """Algorithmic bytes of the timed launches / their summed HIP-event duration, against 8 TB/s."""
    bits, S = cfg["bits"], cfg["stale_max"]
    prefix = cfg.get("codec") == "prefix"
    stale_fraction = {"fixed1": 1.0, "uniform": S / (S + 1.0)}.get(cfg.get("stale"), 0.0)
    per_pc = algorithmic_bytes_per_pair_coordinate(kernel, bits, stale_fraction, inplace, prefix)
    launches = max(1, m["times"]["gossip_calls"])
    total = per_pc * d * m["interactions"]
    if prefix:                                   # planes 1 and 2 of the tiles that escalated
        total += 512 * (0.5 * (m["prefix_tiles"][1] + m["prefix_tiles"][2]) + 1.0 * m["prefix_tiles"][2])
    seconds = m["times"]["gossip_ms"] * 1e-3
    achieved = total / seconds / 1e9 if seconds > 0 else 0.0
    measured = None if inplace or prefix else MEASURED_TRAFFIC_PER_PAIR_COORDINATE.get((kernel, bits, stale_fraction == 1.0))
    return {"kernel": name, "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": None if measured is None else measured * d * m["interactions"] / launches,
            "traffic_unit": "bytes per launch = the per-pair-coordinate constant stored from the rocprofv3 FETCH_SIZE + "
                            "WRITE_SIZE runs under profiles/ (calibrated on the stream copy) x d x pairs; not counted in this run",
            "achieved_bytes_per_launch": total / launches, "bytes_per_pair_coordinate": per_pc,
            "ms_per_launch": m["times"]["gossip_ms"] / launches}


def alu_roofline(cfg, m, d):
    """The instruction-issue side of the one-pass round (8-bit codes, gradient noise): from H = 4 on these kernels are
    bound by the vector ALUs, not by HBM.  None for workloads whose instruction count was not measured."""
    if cfg["bits"] != 8 or not cfg.get("sigma") or cfg.get("codec") == "prefix":
        return None
    per_tile = VALU_PER_NODE_TILE_8BIT[0] + VALU_PER_NODE_TILE_8BIT[1] * cfg["H"]
    lane_ops = 64.0 * per_tile * 2 * m["interactions"] * ((d + 511) // 512)
    rate = lane_ops / (m["times"]["gossip_ms"] * 1e-3) / 1e12
    return {"bound": "alu", "valu_instructions_per_node_tile": per_tile, "achieved": rate, "peak": VALU_PEAK_TLANEOPS,
            "unit": "T lane-ops/s", "frac": rate / VALU_PEAK_TLANEOPS,
            "note": "instruction count per tile = the stored SQ_INSTS_VALU / SQ_WAVES figure from "
                    "profiles/fused_pairs_kernel_config5.md, not counted in this run; a wave64 instruction holds its "
                    "SIMD's issue port 4 cycles"}


def step_roofline(kernel, cfg, m, d, n, inplace=False):
    """Every compulsory byte of the step (pairs and unmatched nodes) over the wall time of the step."""
    bits, S = cfg["bits"], cfg["stale_max"]
    stale_fraction = {"fixed1": 1.0, "uniform": S / (S + 1.0)}.get(cfg.get("stale"), 0.0)
    pair_bytes = algorithmic_bytes_per_pair_coordinate(kernel, bits, stale_fraction, inplace, cfg.get("codec") == "prefix")
    unmatched = n * m["steps"] - 2 * m["interactions"]
    total = d * (pair_bytes * m["interactions"] + unmatched_bytes_per_node_coordinate(kernel, bits, inplace) * unmatched)
    if kernel == "gossip":
        total += 16.0 * d * n * m["steps"]       # the stand-alone local steps: read X, a, c, write W
    achieved = total / m["dt"] / 1e9
    return {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
            "what": "all compulsory bytes of the step (pairs + unmatched nodes) / ms_per_step"}


def make_swarm(swarm, torch, cfg, edges, a, c, eps, args=None, stale_max=None):
    n, d, bits = cfg["n"], cfg["d"], cfg["bits"]
    S = cfg["stale_max"] if stale_max is None else stale_max
    if cfg["objective"] == "mlp":
        x0 = 0.02 * torch.randn(d, device="cuda", generator=torch.Generator(device="cuda").manual_seed(1))
        s = swarm.Swarm(n, d, edges, bits, eps, cfg["H"], cfg["lr"], S, seed=0, x0=x0)
        s.set_objective_mlp(cfg["n_in"], cfg["n_hid"], cfg["n_out"], a, c, cfg["data_sigma"], cfg["batch"])
        if args is not None and args.mlp_bf16x3:
            s.set_mlp_arithmetic(swarm.MLP_BF16X3)
    elif cfg["objective"] == "lsq":
        s = swarm.Swarm(n, d, edges, bits, eps, cfg["H"], cfg["lr"], 0, seed=0)
        s.set_objective_lsq(a, c, cfg["m_rows"], cfg["batch"])
    else:
        s = swarm.Swarm(n, d, edges, bits, eps, cfg["H"], cfg["lr"], S, seed=0,
                        apply_mode=swarm.INPLACE if args is not None and args.inplace else swarm.DEFERRED,
                        codec=swarm.CODEC_PREFIX if args is not None and args.prefix else swarm.CODEC_FIXED,
                        scale_policy=(swarm.SCALE_GLOBAL_LINF if args is not None and args.global_scale else
                                      swarm.SCALE_PAIR_LINF if args is not None and args.pair_scale else swarm.SCALE_FIXED))
        s.set_objective_diag(a, c, cfg["sigma"])
    return s


def sequential_report(torch, swarm, s, cfg, batch, steps, warmup, compare_single=True):
    """Algorithm 1: `batch` interactions per swarm_run_sequential call (a step), and, beside it, the same
    number of interactions as one swarm_sample_pair + swarm_interact per interaction."""
    n, d, bits = cfg["n"], cfg["d"], cfg["bits"]
    launches = []

    def step():
        launches.append(s.run_sequential(batch)[1])

    m = measure(torch, s, step, steps, warmup)
    per_launch = m["interactions"] / max(1, sum(launches[-steps:]))
    rep = {"step": f"swarm_run_sequential({batch}): Algorithm 1, interactions on disjoint nodes share a launch",
           "steps": steps, "ms_per_step": m["dt"] / steps * 1e3, "interactions_per_s": m["interactions"] / m["dt"],
           "interactions_per_launch": per_launch}
    if cfg["objective"] == "diag":
        # per interaction-coordinate: read X_i, X_j, Xhat_i, a_i, c_i (20 B), write X_i', X_j', Xhat_i' (12 B), two codes
        per_ic = 32.0 + 2 * bits / 8
        seconds = m["times"]["gossip_ms"] * 1e-3
        achieved = per_ic * d * m["interactions"] / seconds / 1e9
        rep["roofline"] = {"kernel": "interact_kernel<local steps inside> (Algorithm 1, many interactions per launch)",
                           "bound": "hbm", "bytes_per_interaction_coordinate": per_ic, "achieved": achieved,
                           "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                           "ms_per_interaction": m["times"]["gossip_ms"] / max(1, m["interactions"])}
    else:
        # least squares: 2 * H * batch rows of A per interaction dominate (read twice per step), plus the rows of the pair
        per_i = cfg["H"] * 2 * cfg["batch"] * d * 4 + 28.0 * d + 16.0 * d
        achieved = per_i * m["interactions"] / m["dt"] / 1e9
        rep["roofline"] = {"kernel": "lsq_split_kernel (an initiator's local steps and its interaction in one launch; latency-bound: "
                                     "a few dozen workgroups per launch, one exchange between them per local step)",
                           "bound": "hbm", "bytes_per_interaction": per_i, "achieved": achieved, "peak": HBM_PEAK_GBS,
                           "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS}
    if compare_single:
        def single():
            for _ in range(batch):
                s.interact(*s.sample_pair())
        m1 = measure(torch, s, single, max(1, steps // 2), 1)
        rep["one_call_per_interaction"] = {"interactions_per_s": m1["interactions"] / m1["dt"],
                                           "speedup_of_the_batched_run": (m["interactions"] / m["dt"]) / (m1["interactions"] / m1["dt"])}
    return rep


def compact_config(torch, swarm, cfg_id, steps, warmup):
    """A few timed steps of another workload configuration, as a compact record."""
    cfg, edges, a, c = build_workload(cfg_id)
    eps = eps_for(cfg)
    n, d, bits = cfg["n"], cfg["d"], cfg["bits"]
    s = make_swarm(swarm, torch, cfg, edges, a, c, eps)
    rec = {"workload": f"config {cfg_id}: n={n} d={d} graph={cfg['graph']} {cfg['objective']} H={cfg['H']} bits={bits} "
                       f"stale_max={cfg['stale_max']} ({cfg.get('stale', 'fresh')}) eps={eps}"}
    if cfg["mode"] == "sequential":
        rec.update(sequential_report(torch, swarm, s, cfg, cfg["steps"], steps, warmup))
    elif cfg["objective"] == "diag":
        m = measure(torch, s, lambda: s.round_fused(None, stale_plan(cfg, s)), steps, warmup)
        form = "nodes" if cfg.get("stale") == "fixed1" else "pairs" + ("/nodes by staleness class" if cfg["stale_max"] else "")
        roof = roofline("round", f"fused_{form}_kernel (one-pass round)", cfg, m, d)
        rec.update({"step": "one-pass round (swarm_round_fused)", "steps": steps, "ms_per_step": m["dt"] / steps * 1e3,
                    "interactions_per_s": m["interactions"] / m["dt"],
                    "roofline": {k: roof[k] for k in ("kernel", "bound", "bytes_per_pair_coordinate", "achieved", "peak", "unit",
                                                      "frac", "ms_per_launch")},
                    "step_roofline_frac": step_roofline("round", cfg, m, d, n)["frac"]})
        alu = alu_roofline(cfg, m, d)
        if alu:
            rec["alu_roofline"] = alu
    else:   # MLP: the local steps are GEMMs on the matrix cores, the gossip pass is the HBM-bound one
        def step():
            s.local_steps()
            s.gossip_round(None, None)
        flops_node_step = 5 * 2.0 * cfg["batch"] * cfg["n_in"] * cfg["n_hid"]
        # weights read by the three forward/backward GEMMs and read + written by the two updating ones, per node and step
        weight_bytes_node_step = 4.0 * (2 + 3 + 2) * cfg["n_in"] * cfg["n_hid"]

        def local_steps_record(m, peak, what):
            t = m["times"]
            calls = max(1, t["local_calls"])
            tflops = flops_node_step * n * cfg["H"] * calls / (t["local_ms"] * 1e-3) / 1e12
            return {"kernel": what, "bound": "mfma", "flops_per_node_step": flops_node_step, "achieved": tflops, "peak": peak,
                    "unit": "TFLOP/s", "frac": tflops / peak, "ms_per_round": t["local_ms"] / calls,
                    "weight_traffic_GBps": weight_bytes_node_step * n * cfg["H"] * calls / (t["local_ms"] * 1e-3) / 1e9}

        m = measure(torch, s, step, steps, warmup)
        goss = roofline("gossip", "gossip_pairs_kernel", cfg, m, d)
        rec.update({"step": "swarm_local_steps (grouped fp32 MFMA GEMMs) + swarm_gossip_round", "steps": steps,
                    "ms_per_step": m["dt"] / steps * 1e3, "interactions_per_s": m["interactions"] / m["dt"],
                    "roofline": local_steps_record(m, MFMA_F32_PEAK_TFLOPS,
                                                   "mlp_gemm_kernel (5 grouped float32 GEMMs per node and local step, all "
                                                   "local-step kernels timed)"),
                    "gossip_pass": {k: goss[k] for k in ("kernel", "bound", "bytes_per_pair_coordinate", "achieved", "peak", "unit",
                                                         "frac", "ms_per_launch")}})
        # the same steps with every product taken as three bf16 products (float32 accumulation): against a third of
        # the dense bf16 rate, and against HBM for the weights it has to move
        s.set_mlp_arithmetic(swarm.MLP_BF16X3)
        m3 = measure(torch, s, step, steps, warmup)
        r3 = local_steps_record(m3, MFMA_BF16_PEAK_TFLOPS / 3.0,
                                "mlp_gemm3_kernel (the same GEMMs as hi*hi + hi*lo + lo*hi on the bf16 matrix cores)")
        r3["hbm_frac_of_weight_traffic"] = r3["weight_traffic_GBps"] / HBM_PEAK_GBS
        rec["bf16x3"] = {"ms_per_step": m3["dt"] / steps * 1e3, "interactions_per_s": m3["interactions"] / m3["dt"],
                         "roofline": r3}
    s.close()
    del s, a, c
    torch.cuda.empty_cache()
    return rec


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20,
                    help="untimed steps first: the first ~10 launches run up to 15 %% slower (clock ramp)")
    ap.add_argument("--config", type=int, default=4, help="workload configuration (1 to 5)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the compact runs of the other configurations after the headline's timed region")
    ap.add_argument("--config-steps", type=int, default=12, help="timed steps of each of the other configurations")
    ap.add_argument("--two-call", action="store_true",
                    help="time swarm_local_steps + swarm_gossip_round as the step instead of the one-pass round")
    ap.add_argument("--sequential", action="store_true",
                    help="Algorithm 1 (swarm_run_sequential) at the configuration's shape with fresh reads, instead of rounds")
    ap.add_argument("--inplace", action="store_true",
                    help="in-place apply mode (local steps update the exchanged model; one matrix) instead of the "
                         "paper's deferred apply")
    ap.add_argument("--prefix", action="store_true",
                    help="multi-resolution registers: 16-bit codes in planes, readers fetch the shortest confirmed "
                         "prefix (instead of the configuration's fixed b bits)")
    ap.add_argument("--global-scale", action="store_true",
                    help="one lattice scale per round, set from the disagreement the previous round reported "
                         "(needs a configuration with at least 8-bit codes)")
    ap.add_argument("--pair-scale", action="store_true",
                    help="every matched pair uses its own lattice scale from a pre-pass over its two models "
                         "(SWARM_SCALE_PAIR_LINF; fresh reads, two-call round only)")
    ap.add_argument("--mlp-bf16x3", action="store_true",
                    help="MLP objective: GEMMs as three bf16 products per term instead of float32 matrix instructions")
    ap.add_argument("--d", type=int, default=None, help="override the model dimension (debugging only)")
    ap.add_argument("--H", type=int, default=None,
                    help="override the number of local steps (to find where a kernel turns ALU-bound)")
    ap.add_argument("--cpu-worker", default=None, help=argparse.SUPPRESS)
    args = ap.parse_args()
    if args.cpu_worker:
        return cpu_worker(args.cpu_worker)
    if args.gpus != 1:
        raise SystemExit("bench.py: this build simulates the whole swarm on ONE GPU; --gpus must be 1 "
                         "(no collectives or sharding across GPUs are part of it)")
    import torch
    import paper_1910_12308_amd as swarm

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    cfg, edges, a, c = build_workload(args.config, args.d, args.H)
    if args.prefix:
        if cfg["objective"] != "diag" or cfg["bits"] == 0:
            raise SystemExit("bench.py: --prefix needs a configuration with the diagonal objective and quantized codes")
    eps = eps_for(cfg)         # the configuration's scale: the first plane decodes what its b-bit code would
    if args.prefix:
        cfg["codec"], cfg["bits"] = "prefix", 16
    n, d, bits = cfg["n"], cfg["d"], cfg["bits"]
    sequential = args.sequential or cfg["mode"] == "sequential"
    s = make_swarm(swarm, torch, cfg, edges, a, c, eps, args, stale_max=0 if sequential else None)

    # clock ramp: a few plain copies before the warm-up steps (not steps of the path, never timed)
    ramp_src = s.models_view(swarm.COMM)
    ramp_dst = torch.empty_like(ramp_src[: max(1, n // 4)])
    for _ in range(20):
        swarm.stream_copy(ramp_dst, ramp_src[: max(1, n // 4)])
    torch.cuda.synchronize()
    del ramp_dst

    workload = (f"config {args.config}: n={n} d={d} graph={cfg['graph']} {cfg['objective']} "
                f"sigma={cfg.get('sigma', cfg.get('data_sigma'))} H={cfg['H']} lr={cfg['lr']} bits={bits} "
                f"stale_max={cfg['stale_max']} ({cfg.get('stale', 'fresh')}) eps={eps}")
    if sequential:
        batch = cfg.get("steps", 256) if cfg["mode"] == "sequential" else 256
        rep = sequential_report(torch, swarm, s, cfg, batch, args.steps, args.warmup)
        out = {"metric": "node-interactions/sec + gossip-avg HBM GB/s (% of peak), n=64 d=25.6M",
               "value": rep["interactions_per_s"], "unit": "interactions/s", "n_gpus": 1, "steps": args.steps,
               "warmup": args.warmup, "ms_per_step": rep["ms_per_step"], "higher_is_better": True, "scaling": "weak",
               "vs_baseline": None, "dtype": "f32", "data": "synthetic",
               "config": {"workload": workload + " -- Algorithm 1, fresh reads", "step": rep["step"],
                          "interactions_per_launch": rep["interactions_per_launch"],
                          **({"one_call_per_interaction": rep["one_call_per_interaction"]}
                             if "one_call_per_interaction" in rep else {})},
               "roofline": rep["roofline"]}
        if not args.no_cpu_baseline and cfg["objective"] == "lsq":
            out["cpu_baseline"] = cpu_baseline(cfg, edges, a, c, eps)
        print(json.dumps(out))
        return

    def step_two_calls():
        s.local_steps()
        s.gossip_round(None, stale_plan(cfg, s))

    def step_one_pass():
        s.round_fused(None, stale_plan(cfg, s))

    # The step is one pass of the whole hot path.  For per-coordinate objectives the library offers it as
    # one kernel pass (local steps inside the gossip pass, bit-identical to the two calls); that is the
    # timed step unless --two-call is given.  The other variant is measured after the timed region and
    # reported beside it.
    one_pass_ok = cfg["objective"] == "diag"
    one_pass_ok = one_pass_ok and not args.pair_scale       # the per-pair scale needs the pre-pass of the two-call round
    use_one_pass = one_pass_ok and not args.two_call
    main_m = measure(torch, s, step_one_pass if use_one_pass else step_two_calls, args.steps, args.warmup)
    other_m = None
    if one_pass_ok:
        other_m = measure(torch, s, step_two_calls if use_one_pass else step_one_pass, args.steps, 3)
    one_m, two_m = (main_m, other_m) if use_one_pass else (other_m, main_m)

    # Pairs whose reads are both stale are processed node by node (two grid rows per pair); every
    # other class goes through the pair kernels.
    all_stale = cfg.get("stale") == "fixed1"
    form = "nodes" if all_stale else "pairs"
    k_round = (f"prefix_{form}_kernel<local steps>" if args.prefix else f"fused_{form}_kernel") + \
        " (H local steps + quantize/exchange/decode/average, one pass)"
    k_gossip = (f"prefix_{form}_kernel" if args.prefix else f"gossip_{form}_kernel") + " (quantize/exchange/decode/average)"

    def two_call_report(m):
        t = m["times"]
        rep = {"interactions_per_s": m["interactions"] / m["dt"], "ms_per_step": m["dt"] / args.steps * 1e3,
               "gossip_pass": roofline("gossip", k_gossip, cfg, m, d,
                                       args.inplace),
               "local_steps_ms_per_round": t["local_ms"] / max(1, t["local_calls"])}
        if cfg["objective"] == "mlp":
            # 5 GEMMs of 2*batch*in*hid (= 2*batch*hid*out here) flops per node and local step
            flops = 5 * 2.0 * cfg["batch"] * cfg["n_in"] * cfg["n_hid"] * n * cfg["H"] * t["local_calls"]
            rep["local_steps_mfma_f32_TFLOPs"] = flops / (t["local_ms"] * 1e-3) / 1e12
            rep["local_steps_mfma_frac_of_157.3"] = rep["local_steps_mfma_f32_TFLOPs"] / 157.3
            rep["local_steps_arithmetic"] = "three bf16 products per term" if args.mlp_bf16x3 else "float32 matrix instructions"
        elif t["local_ms"] > 0:
            rep["local_steps_GBps"] = 16.0 * d * n * t["local_calls"] / (t["local_ms"] * 1e-3) / 1e9
            rep["local_steps_frac_of_hbm_peak"] = rep["local_steps_GBps"] / HBM_PEAK_GBS
        return rep

    if use_one_pass:
        roof = roofline("round", k_round, cfg, main_m, d)
    else:
        roof = roofline("gossip", k_gossip, cfg, main_m, d)
    out = {
        "metric": "node-interactions/sec + gossip-avg HBM GB/s (% of peak), n=64 d=25.6M",
        "value": main_m["interactions"] / main_m["dt"],
        "unit": "interactions/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": main_m["dt"] / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": workload,
                   "apply_mode": "inplace" if args.inplace else "deferred",
                   **({"scale": "per round (SWARM_SCALE_GLOBAL_LINF)", "eps_after_the_run": s.scale()[0]}
                      if args.global_scale else {}),
                   **({"scale": "per pair (SWARM_SCALE_PAIR_LINF): pair_linf_kernel pre-pass, 8 B per pair-coordinate, "
                                "inside the timed gossip bracket"} if args.pair_scale else {}),
                   "step": ("one-pass round (swarm_round_fused)" if use_one_pass
                            else "swarm_local_steps + swarm_gossip_round"),
                   "pairs_per_round": main_m["interactions"] / args.steps,
                   "node_updates_per_s": 2.0 * main_m["interactions"] / main_m["dt"],
                   # the device counts a decode failure where a FRESH read decodes to another lattice point than the
                   # sender's; with every read stale there is nothing to compare with on the device
                   "decode_failures": None if all_stale else main_m["decode_failures"],
                   **({"decode_failures_note": "not counted: every read is stale"} if all_stale else {}),
                   "gradient_noise": "16-bit uniforms, one Philox call per 8 normals (the build's choice; with one call "
                                     "per 4 normals on 24-bit uniforms the same kernel measured about 5 points lower)",
                   **({"registers": "multi-resolution (16-bit planes, prefix reads)",
                       "tile_reads_at_4_8_16_bits": main_m["prefix_tiles"]} if args.prefix else {})},
        "roofline": roof,
    }
    if cfg["objective"] == "diag":
        out["step_roofline"] = step_roofline("round" if use_one_pass else "gossip", cfg, main_m, d, n, args.inplace)
        alu = alu_roofline(cfg, main_m, d) if use_one_pass and not args.prefix and not args.inplace else None
        if alu:
            out["alu_roofline"] = alu
    if two_m is not None:
        out["two_call_round"] = two_call_report(two_m)
    if one_m is not None and not use_one_pass:
        out["one_pass_round"] = {"interactions_per_s": one_m["interactions"] / one_m["dt"],
                                 "ms_per_step": one_m["dt"] / args.steps * 1e3,
                                 "roofline": roofline("round", k_round, cfg, one_m, d)}
    # Measured ceiling: a plain streaming copy kernel over one model matrix worth of bytes.
    src = s.models_view(swarm.COMM)
    dst = torch.empty_like(src)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    swarm.stream_copy(dst, src)
    ev0.record()
    for _ in range(5):
        swarm.stream_copy(dst, src)
    ev1.record()
    torch.cuda.synchronize()
    copy_gbs = 2.0 * src.numel() * 4 * 5 / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
    out["roofline"]["copy_kernel_GBps"] = copy_gbs
    out["roofline"]["frac_of_copy"] = out["roofline"]["achieved"] / copy_gbs
    # The same copy with the float streams one node of the timed kernel touches: 3 reads (X, a, c) and one
    # write for the one-pass round, 2 reads (X, W) and one write for the gossip pass.
    n_read = 3 if use_one_pass else 2
    stream_bytes = (n // n_read) * d * 4                         # each stream is a block of rows of the model matrix
    swarm.stream_mix(dst, src, stream_bytes, n_read, 1)
    ev0.record()
    for _ in range(5):
        swarm.stream_mix(dst, src, stream_bytes, n_read, 1)
    ev1.record()
    torch.cuda.synchronize()
    mix_gbs = (n_read + 1) * stream_bytes * 5 / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
    out["roofline"]["same_streams_copy_GBps"] = mix_gbs
    out["roofline"]["frac_of_same_streams_copy"] = out["roofline"]["achieved"] / mix_gbs
    del dst, src
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, edges, a, c, eps)
    # The other configurations, after the headline's timed region: compact records in the same line.
    if args.config == 4 and not args.no_configs and not (args.inplace or args.prefix or args.global_scale or args.pair_scale
                                                         or args.d or args.H):
        configs = {}
        # Algorithm 1 at the headline's shape (fresh reads; the sequential model has no stale partner copies)
        seq = make_swarm(swarm, torch, cfg, edges, a, c, eps, stale_max=0)
        rec = sequential_report(torch, swarm, seq, cfg, 256, max(2, args.config_steps // 4), 1)
        rec["workload"] = workload + " -- Algorithm 1, fresh reads"
        configs["4-sequential"] = rec
        seq.close()
        s.close()
        del seq, s, a, c
        torch.cuda.empty_cache()
        for other in (2, 5, 3, 1):
            configs[str(other)] = compact_config(torch, swarm, other, args.config_steps, 3)
        out["configs"] = configs
    print(json.dumps(out))


if __name__ == "__main__":
    main()

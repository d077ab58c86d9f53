#!/usr/bin/env python3
"""Solve time of the dispatcher's integer program per scheduling tick, at the cluster sizes
of the paper's dispatcher-scalability table (128 to 4096 GPUs).

    python -m paper_2510_02838_amd.dispatch_bench [--grid-json FILE ...] [--node-limit N] [--ticks 5]

Request runtimes t[r][i][k] come from the Diffuse-stage profiler table when --grid-json names
outputs of `stage_profile grid` (seconds per step at k = 1 on one MI355X, times the steps of
a sample); otherwise from a log-uniform stand-in of the same range.  Degrees above 1 are a
MODEL, not a measurement (this build runs on one GPU): t_k = t_1 / k + the two all-to-all
exchanges per attention of head/sequence re-sharding over k-1 xGMI links of 153 GB/s.  The
efficiency filter E[r][k] keeps degrees with t_1 / (k t_k) >= 0.8, as in the paper; the
placement filter F[r][i][k] keeps options whose weights plus workspace share fit the HBM left
on a replica of type i.  Deadlines are tau + slack * t_1, slack uniform in [0.6, 3].
Prints one JSON line per cluster size.
"""
import argparse
import json
import time

import numpy as np

from . import dispatch as T

DEGREES = (1, 2, 4, 8)
HBM = 288e9
LINK = 153e9


def load_grid(paths):
    rows = []
    for p in paths:
        for line in open(p):
            line = line.strip()
            if line.startswith("{"):
                d = json.loads(line)
                if d.get("table") == "grid":
                    rows.append(d)
    return rows


def make_tick(rng, gpus, grid):
    R = gpus // 4
    if grid:
        pick = rng.integers(0, len(grid), R)
        steps = np.array([50 if grid[j]["workload"] == "wan" else 28 for j in pick])
        t1 = np.array([grid[j]["s_per_step"] for j in pick]) * steps
        tokens = np.array([grid[j]["tokens"] for j in pick], float)
        mem = np.array([grid[j]["weight_bytes"] + grid[j]["workspace_bytes"] for j in pick], float)
        width = np.array([5120.0 if grid[j]["workload"] == "wan" else 3072.0 if grid[j]["workload"] == "flux" else 1536.0 for j in pick])
        blocks = np.array([40.0 if grid[j]["workload"] == "wan" else 57.0 if grid[j]["workload"] == "flux" else 24.0 for j in pick])
    else:
        t1 = np.exp(rng.uniform(np.log(0.1), np.log(300.0), R))
        tokens = np.exp(rng.uniform(np.log(200.0), np.log(8e4), R))
        mem = rng.uniform(5e9, 60e9, R)
        steps, width, blocks = np.full(R, 28), np.full(R, 3072.0), np.full(R, 57.0)
    t = np.empty((R, 4, 4))
    feas = np.zeros((R, 4, 4), np.uint8)
    resident = np.array([30e9, 12e9, 20e9, 0.0])          # encoder/decoder weights sharing the replica
    for ki, k in enumerate(DEGREES):
        vol = 4.0 * (tokens / k) * width * 2.0 * (k - 1) / k          # bytes sent per GPU per attention
        comm = steps * blocks * (vol / (LINK * max(k - 1, 1)))
        tk = t1 / k + (comm if k > 1 else 0.0)
        eff_ok = t1 / (k * tk) >= 0.8
        for i in range(4):
            t[:, i, ki] = tk * (1.0 + 0.02 * i)
            fits = mem / k + resident[i] <= HBM
            feas[:, i, ki] = eff_ok & fits
    feas[:, 1:3] = 0                                       # a cluster usually has 1-2 Primary types
    deadline = rng.uniform(0.6, 3.0, R) * t1
    length = tokens * steps
    B = [gpus // 8, 0, 0, gpus // 8]
    return t, feas, deadline, length, B


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--grid-json", nargs="*", default=[])
    ap.add_argument("--node-limit", type=int, default=200000)
    ap.add_argument("--ticks", type=int, default=5)
    args = ap.parse_args()
    grid = load_grid(args.grid_json)
    for gpus in (128, 256, 512, 1024, 4096):
        rng = np.random.default_rng(gpus)
        ms, gaps, proven, objs = [], [], 0, []
        for _ in range(args.ticks):
            t, feas, deadline, length, B = make_tick(rng, gpus, grid)
            t0 = time.perf_counter()
            W = T.reward_weights(t, feas, deadline, 0.0)
            Q = T.comm_penalty(length)
            got = T.solve(W, Q, feas, B, t, deadline, 0.0, node_limit=args.node_limit)
            ms.append((time.perf_counter() - t0) * 1e3)
            gaps.append(got["upper_bound"] - got["objective"])
            objs.append(got["objective"])
            proven += got["status"] == T.TDS_OK
        print(json.dumps({"gpus": gpus, "requests_per_tick": gpus // 4, "idle_replicas": gpus // 4,
                          "ms_per_tick_mean": float(np.mean(ms)), "ms_per_tick_max": float(np.max(ms)),
                          "proven_optimal": f"{proven}/{args.ticks}", "max_gap": float(np.max(gaps)),
                          "mean_objective": float(np.mean(objs)), "node_limit": args.node_limit,
                          "runtimes": "profiler grid" if grid else "stand-in",
                          "paper_context_ms": {128: 25, 256: 26, 512: 36, 1024: 45, 4096: 98}[gpus]}), flush=True)


if __name__ == "__main__":
    main()

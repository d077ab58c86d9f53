#!/usr/bin/env python3
"""Benchmark of the Diffuse-stage hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload sd3|flux|hetero8|wan|tiny]

A step is one denoising step (model evaluation + latent update) for the whole request
batch of the workload; the timed region is one dit_sample call of exactly K steps with all
inputs already resident in HBM.  Prints ONE JSON line: steps/s, the roofline of the dominant
kernel (the MFMA GEMM) from HIP-event timings taken inside the library, the per-class
breakdown, and the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0
# Fabric-side bytes per GEMM launch (rocprofv3 FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, the scale
# factors from the streaming calibration kernel), averaged over the GEMM launches of a step;
# measured once per workload, see profiles/<workload>_hbm_traffic.txt.  None = not measured.
MEASURED_GEMM_TRAFFIC_BYTES = {"sd3": 219.3e6}


def cpu_baseline(name, arch, reqs):
    """The oracle as it stands, on the host cores: one denoising step of the first request
    of the workload at reduced depth, scaled to full depth by block count."""
    import numpy as np
    import synth
    from oracle import dit_oracle as O
    depth = dict(n_blocks=min(arch["n_blocks"], 1), n_single=min(arch["n_single"], 1))
    small = dict(arch, **depth)
    f, h, w, nc = reqs[0]
    if name == "wan":      # 32760 tokens is hours on a CPU: one frame-slab of the video
        f = arch["patch"][0]
    lat, cond, sig = synth.make_inputs([(f, h, w, nc)], arch["latent_ch"], arch["cond_dim"], 1)
    params = synth.make_params(O.param_shapes(small), 1, 0.02)
    m = O.DiTOracle(small, params)
    t0 = time.perf_counter()
    m.step(lat[0], cond[0], sig[0][0], sig[0][1])
    dt = time.perf_counter() - t0
    blocks_full = arch["n_blocks"] + arch["n_single"]
    blocks_small = small["n_blocks"] + small["n_single"]
    scale = blocks_full / blocks_small
    tokens_full = sum((rf // arch["patch"][0]) * (rh // arch["patch"][1]) * (rw // arch["patch"][2]) + rc
                      for rf, rh, rw, rc in reqs)
    tokens_small = (f // arch["patch"][0]) * (h // arch["patch"][1]) * (w // arch["patch"][2]) + nc
    est = dt * scale * (tokens_full / tokens_small)
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count()
    cores = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))
    return {"value": 1.0 / est, "unit": "steps/s", "cores": cores, "kind": "oracle",
            "sample": f"float64 NumPy oracle, one step of request 0 ({tokens_small} tokens) at "
                      f"{blocks_small} of {blocks_full} blocks: {dt:.2f} s measured, scaled linearly by "
                      f"block count and token count to the full workload ({tokens_full} tokens)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="sd3")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run the streaming update kernel on 2^26 floats (reads 512 MiB, writes "
                         "256 MiB): a kernel of known traffic to scale rocprofv3 FETCH_SIZE/WRITE_SIZE by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus above 1 is not supported "
              "(requests are independent and would shard with no exchange)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import synth
    from paper_2510_02838_amd import binding as B

    name = args.workload
    cfg = synth.CONFIGS[name]
    arch, reqs = cfg["arch"], synth.make_requests(name)
    K = args.steps if args.steps is not None else (4 if name == "wan" else 28)
    W = max(args.warmup, 0)

    torch.cuda.set_device(0)
    m = B.DiT(arch)
    m.ensure_workspace(reqs, max(K, W, 1))
    m.init_weights(1, 0.02)
    lat, cond, _ = synth.make_inputs(reqs, arch["latent_ch"], arch["cond_dim"], 1, None)
    pack = lambda arrs: np.concatenate([np.asarray(a, np.float32).ravel() for a in arrs])
    d_cond = torch.from_numpy(pack(cond)).cuda().to(torch.bfloat16)   # values are bf16-exact
    x0 = torch.from_numpy(pack(lat)).cuda()
    shifts = cfg["shifts"]

    def sig(T):
        return np.stack([synth.default_sigmas(T, s) for s in shifts])

    if args.calibrate_copy:
        n = 1 << 26
        ca, cb = torch.zeros(n, device="cuda"), torch.ones(n, device="cuda")
        for _ in range(3):
            assert B.dit_op_latent_update(None, ca.data_ptr(), cb.data_ptr(), n, 1.0, 0.5) == 0
        torch.cuda.synchronize()
        del ca, cb
    x = x0.clone()
    if W > 0:
        m.sample(reqs, x, d_cond, sig(W))
    torch.cuda.synchronize()
    x.copy_(x0)
    sg = sig(K)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    m.sample(reqs, x, d_cond, sg)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    finite = bool(torch.isfinite(x).all().item())

    # second pass of the same K steps with per-class HIP events inside the library
    x.copy_(x0)
    m.profile_enable(True)
    m.sample(reqs, x, d_cond, sg)
    prof = m.profile_read()
    m.profile_enable(False)

    g, a = prof["gemm"], prof["attention"]
    gemm_tf = g["flop"] / g["ms"] / 1e9 if g["ms"] > 0 else 0.0
    attn_tf = a["flop"] / a["ms"] / 1e9 if a["ms"] > 0 else 0.0
    both_tf = (g["flop"] + a["flop"]) / (g["ms"] + a["ms"]) / 1e9
    ew = {}
    for k in ("ln_modulate", "qknorm_rope_vt", "update"):
        p = prof[k]
        ew[k] = {"ms_per_step": p["ms"] / K, "GBps": p["bytes"] / p["ms"] / 1e6 if p["ms"] > 0 else 0.0,
                 "frac_hbm": (p["bytes"] / p["ms"] / 1e6) / PEAK_HBM_GBS if p["ms"] > 0 else 0.0}
    out = {
        "metric": "denoising_steps_per_sec", "value": K / dt, "unit": "steps/s", "n_gpus": 1,
        "steps": K, "warmup": W, "ms_per_step": dt / K * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{name}: {len(reqs)} request(s), "
                               f"{sum((f//arch['patch'][0])*(h//arch['patch'][1])*(w//arch['patch'][2]) + c for f,h,w,c in reqs)} tokens, "
                               f"hidden {arch['hidden']}, {arch['n_blocks']}+{arch['n_single']} blocks, "
                               f"{arch['n_heads']}x{arch['head_dim']} heads",
                   "steps_per_sample": K, "finite": finite},
        "roofline": {"bound": "mfma", "kernel": "gemm_kernel (bf16 MFMA GEMM, all launches of the step)",
                     "achieved": gemm_tf, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": gemm_tf / PEAK_BF16_TFLOPS, "traffic": MEASURED_GEMM_TRAFFIC_BYTES.get(name),
                     "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE/WRITE_SIZE, scaled)",
                     "algorithmic_bytes_per_launch": g["bytes"] / max(g["launches"], 1),
                     "avg_launch_us": g["ms"] / max(g["launches"], 1) * 1e3,
                     "flop_per_launch": g["flop"] / max(g["launches"], 1)},
        "mfma": {"gemm_tflops": gemm_tf, "gemm_frac_peak": gemm_tf / PEAK_BF16_TFLOPS,
                 "attention_tflops": attn_tf, "attention_frac_peak": attn_tf / PEAK_BF16_TFLOPS,
                 "attention_plus_gemm_tflops": both_tf, "attention_plus_gemm_frac_peak": both_tf / PEAK_BF16_TFLOPS,
                 "gemm_ms_per_step": g["ms"] / K, "attention_ms_per_step": a["ms"] / K,
                 "other_ms_per_step": prof["other"]["ms"] / K},
        "elementwise": ew,
        "paper_context": "the paper reports no absolute Diffuse-stage number; its runs were on NVIDIA L20 48 GB",
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(name, arch, reqs)
    print(json.dumps(out))


if __name__ == "__main__":
    main()

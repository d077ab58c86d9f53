#!/usr/bin/env python3
"""Benchmark of the Diffuse-stage hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload sd3|flux|hetero8|wan|tiny]
                    [--also hetero8,flux,wan | --also none]

A step is one denoising step (model evaluation + latent update) for the whole request
batch of the workload; the timed region is one dit_sample call of exactly K steps with all
inputs already resident in HBM.  Prints ONE JSON line: steps/s of the headline workload
(benchmark config 2, the 4096-token request), the roofline of the dominant kernel (the MFMA
GEMM) from HIP-event timings taken inside the library, the per-class breakdown, the same
figures for the other benchmark configurations under "workloads" (each timed the same way, on
its own short run), and the CPU oracle timed on a bounded sample of the headline workload.

Other legs (no JSON contract, used for the committed profiles):
    --calibrate-copy           a streaming kernel of known traffic before the run
    --gemm-shapes MxNxK,...    the GEMM alone beside torch.matmul on the same operands
    --gemm-profile-run         with --gemm-shapes: three launches each, no timing (counter runs)
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
DEFAULT_STEPS = {"sd3": 28, "hetero8": 10, "flux": 10, "wan": 4, "tiny": 28}


def n_tokens(arch, reqs):
    pt, ph, pw = arch["patch"]
    return sum((f // pt) * (h // ph) * (w // pw) + c for f, h, w, c in reqs)


def _host_cores():
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count()
    return min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))


def _oracle_step_seconds(arch, reqs, blocks):
    import synth
    from oracle import dit_oracle as O
    small = dict(arch, n_blocks=min(arch["n_blocks"], blocks), n_single=0)
    lat, cond, sig = synth.make_inputs(reqs[:1], arch["latent_ch"], arch["cond_dim"], 1)
    params = synth.make_params(O.param_shapes(small), 1, 0.02)
    m = O.DiTOracle(small, params)
    t0 = time.perf_counter()
    m.step(lat[0], cond[0], sig[0][0], sig[0][1])
    return time.perf_counter() - t0


def cpu_baseline(name, arch, reqs):
    """The oracle as it stands on the host cores: one denoising step of the headline request at
    1 and at 3 blocks; every block costs the same (same shapes), so a step at full depth is
    fixed + depth x per-block.  A second leg repeats the 1-block step on one core."""
    cores = _host_cores()
    t1 = _oracle_step_seconds(arch, reqs, 1)
    t3 = _oracle_step_seconds(arch, reqs, 3)
    per_block = (t3 - t1) / 2.0
    depth = arch["n_blocks"] + arch["n_single"]
    est = (t1 - per_block) + depth * per_block
    out = {"value": 1.0 / est, "unit": "steps/s", "cores": cores, "kind": "oracle",
           "sample": f"float64 NumPy oracle, one step of request 0 ({n_tokens(arch, reqs[:1])} tokens) at 1 and at 3 "
                     f"of {depth} blocks: {t1:.2f} s and {t3:.2f} s measured, i.e. {per_block:.2f} s per block; "
                     f"full depth = fixed part + {depth} x per-block = {est:.1f} s per step"}
    try:
        from threadpoolctl import threadpool_limits
        with threadpool_limits(limits=1):
            s1 = _oracle_step_seconds(arch, reqs, 1)
        out["one_core"] = {"value": 1.0 / (est * s1 / t1), "unit": "steps/s", "cores": 1,
                           "sample": f"the 1-block step on one core: {s1:.2f} s against {t1:.2f} s on {cores}; "
                                     f"the full-depth estimate is scaled by that ratio"}
    except Exception as e:          # threadpoolctl missing: the all-cores leg stands alone
        out["one_core"] = {"value": None, "cores": 1, "sample": f"not timed ({e})"}
    return out


def run_workload(name, K, W, calibrate=False):
    """One dit_sample of K steps (timed) after W warm-up steps, then the same K steps again with
    per-class HIP events inside the library.  Returns the figures of that workload."""
    import numpy as np
    import torch
    import synth
    from paper_2510_02838_amd import binding as B

    cfg = synth.CONFIGS[name]
    arch, reqs = cfg["arch"], synth.make_requests(name)
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

    if calibrate:
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
    m.close()
    del m, x, x0, d_cond
    torch.cuda.empty_cache()

    g, a = prof["gemm"], prof["attention"]
    gemm_tf = g["flop"] / g["ms"] / 1e9 if g["ms"] > 0 else 0.0
    attn_tf = a["flop"] / a["ms"] / 1e9 if a["ms"] > 0 else 0.0
    both_tf = (g["flop"] + a["flop"]) / (g["ms"] + a["ms"]) / 1e9
    ew = {}
    for k in ("ln_modulate", "qknorm_rope_vt", "update"):
        p = prof[k]
        if p["ms"] <= 0:          # class without a launch in this step (q/k norm, rotary code and V^T run in the QKV epilogue)
            continue
        ew[k] = {"ms_per_step": p["ms"] / K, "GBps": p["bytes"] / p["ms"] / 1e6 if p["ms"] > 0 else 0.0,
                 "frac_hbm": (p["bytes"] / p["ms"] / 1e6) / PEAK_HBM_GBS if p["ms"] > 0 else 0.0}
    return {
        "workload": f"{name}: {len(reqs)} request(s), {n_tokens(arch, reqs)} tokens, hidden {arch['hidden']}, "
                    f"{arch['n_blocks']}+{arch['n_single']} blocks, {arch['n_heads']}x{arch['head_dim']} heads",
        "steps": K, "warmup": W, "steps_per_s": K / dt, "ms_per_step": dt / K * 1e3, "finite": finite,
        "mfma": {"gemm_tflops": gemm_tf, "gemm_frac_peak": gemm_tf / PEAK_BF16_TFLOPS,
                 "attention_tflops": attn_tf, "attention_frac_peak": attn_tf / PEAK_BF16_TFLOPS,
                 "attention_plus_gemm_tflops": both_tf, "attention_plus_gemm_frac_peak": both_tf / PEAK_BF16_TFLOPS,
                 "gemm_ms_per_step": g["ms"] / K, "attention_ms_per_step": a["ms"] / K,
                 "other_ms_per_step": prof["other"]["ms"] / K},
        "elementwise": ew,
        "gemm_launch": {"algorithmic_bytes_per_launch": g["bytes"] / max(g["launches"], 1),
                        "avg_launch_us": g["ms"] / max(g["launches"], 1) * 1e3,
                        "flop_per_launch": g["flop"] / max(g["launches"], 1), "launches": g["launches"]},
    }


def gemm_leg(shapes, profile_run, rounds=4, iters=10):
    """The library's GEMM (its own tile choice) beside torch.matmul on the same operands: timing
    with the candidates' order rotated from round to round (the shader clock sags during a run,
    so a fixed order favours whoever goes first), or three untimed launches each for counters."""
    import torch
    from paper_2510_02838_amd import binding as B
    for M, N, K in shapes:
        torch.manual_seed(0)
        A = torch.randn(M, K, device="cuda").to(torch.bfloat16)
        Wm = torch.zeros((N + 255) // 256 * 256, K, dtype=torch.bfloat16, device="cuda")
        Wm[:N] = (torch.randn(N, K, device="cuda") * 0.05).to(torch.bfloat16)
        ldc = (N + 7) // 8 * 8
        out = torch.empty(M, ldc, dtype=torch.bfloat16, device="cuda")
        Wt = Wm[:N].t()

        def ours():
            st = B.dit_op_gemm(None, A.data_ptr(), K, Wm.data_ptr(), K, None, M, N, K, 0, out.data_ptr(), ldc, None, 0, None)
            assert st == 0, st

        def lib():
            torch.matmul(A, Wt)

        if profile_run:
            for fn in (ours, lib):
                for _ in range(3):
                    fn()
                torch.cuda.synchronize()
            continue
        ref = torch.matmul(A, Wt).float()
        ours()
        torch.cuda.synchronize()
        err = ((out[:, :N].float() - ref).abs().max() / ref.abs().max()).item()
        assert err < 2e-2, err
        acc = {"dit_op_gemm": [], "torch.matmul": []}
        for r in range(rounds):
            for nm, fn in ((("dit_op_gemm", ours), ("torch.matmul", lib)) if r % 2 == 0 else (("torch.matmul", lib), ("dit_op_gemm", ours))):
                for _ in range(2):
                    fn()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(iters):
                    fn()
                e1.record()
                torch.cuda.synchronize()
                acc[nm].append(e0.elapsed_time(e1) / iters * 1e-3)
        flop = 2.0 * M * N * K
        print(json.dumps({"M": M, "N": N, "K": K,
                          "candidates": {c: {"best_us": min(t) * 1e6, "mean_us": sum(t) / len(t) * 1e6,
                                             "best_tflops": flop / min(t) / 1e12} for c, t in acc.items()}}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="sd3")
    ap.add_argument("--also", default="hetero8,flux,wan",
                    help="other benchmark configurations reported under \"workloads\" (comma list, or none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run the streaming update kernel on 2^26 floats (reads 512 MiB, writes "
                         "256 MiB): a kernel of known traffic to scale rocprofv3 FETCH_SIZE/WRITE_SIZE by")
    ap.add_argument("--gemm-shapes", default=None)
    ap.add_argument("--gemm-profile-run", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus above 1 is not supported "
              "(requests are independent and would shard with no exchange)", file=sys.stderr)
        sys.exit(2)

    import torch
    torch.cuda.set_device(0)
    if args.gemm_shapes:
        gemm_leg([tuple(int(v) for v in s.split("x")) for s in args.gemm_shapes.split(",")], args.gemm_profile_run)
        return

    import synth
    name = args.workload
    K = args.steps if args.steps is not None else DEFAULT_STEPS.get(name, 28)
    W = max(args.warmup, 0)
    head = run_workload(name, K, W, args.calibrate_copy)
    gl, mf = head["gemm_launch"], head["mfma"]
    out = {
        "metric": "denoising_steps_per_sec", "value": head["steps_per_s"], "unit": "steps/s", "n_gpus": 1,
        "steps": K, "warmup": W, "ms_per_step": head["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": head["workload"], "steps_per_sample": K, "finite": head["finite"]},
        # traffic: fabric-side bytes per launch need a rocprofv3 counter run (FETCH_SIZE / WRITE_SIZE); this
        # process cannot read them, so the figure lives in profiles/ with the command that produced it
        "roofline": {"bound": "mfma", "kernel": "gemm_kernel (bf16 MFMA GEMM, all launches of the step)",
                     "achieved": mf["gemm_tflops"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": mf["gemm_frac_peak"], "traffic": None,
                     "algorithmic_bytes_per_launch": gl["algorithmic_bytes_per_launch"],
                     "avg_launch_us": gl["avg_launch_us"], "flop_per_launch": gl["flop_per_launch"]},
        "mfma": mf,
        "elementwise": head["elementwise"],
        "paper_context": "the paper reports no absolute Diffuse-stage number; its runs were on NVIDIA L20 48 GB",
    }
    others = [w for w in args.also.split(",") if w and w != "none" and w != name]
    if others:
        out["workloads"] = {}
        for w in others:
            if w not in synth.CONFIGS:
                raise SystemExit(f"unknown workload {w}")
            r = run_workload(w, DEFAULT_STEPS.get(w, 10), 1)
            r.pop("gemm_launch")
            out["workloads"][w] = r
    if not args.no_cpu_baseline:
        cfg = synth.CONFIGS[name]
        out["cpu_baseline"] = cpu_baseline(name, cfg["arch"], synth.make_requests(name))
    print(json.dumps(out))


if __name__ == "__main__":
    main()

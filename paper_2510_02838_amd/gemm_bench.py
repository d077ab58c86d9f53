#!/usr/bin/env python3
"""The library's bf16 GEMM (`dit_op_gemm` / `dit_op_gemm_variant`) beside torch.matmul
(hipBLASLt) on the same operands: timing, or a short fixed launch sequence for a counter run.

    python -m paper_2510_02838_amd.gemm_bench [--shapes 8192x8192x8192,4250x6144x1536] [--variants 0,1256256,128128]
    python -m paper_2510_02838_amd.gemm_bench --profile-run [--shapes ...]     # 3 + 3 launches per shape, no timing

Shapes are M x N x K (A [M][K], W [N][K], bf16 output).  Variant 0 is the launcher's own tile
choice; other codes force a tile (see launch_gemm).  Timing rotates the order of the candidates
from round to round and reports the best and the mean per candidate: the shader clock sags
during a run, so a fixed order favours whoever goes first.  One JSON line per shape.
"""
import argparse
import json

import torch

from . import binding as B


def _time(fn, iters=10, warm=2):
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters * 1e-3


def _operands(M, N, K):
    torch.manual_seed(0)
    A = torch.randn(M, K, device="cuda").to(torch.bfloat16)
    W = torch.zeros((N + 255) // 256 * 256, K, dtype=torch.bfloat16, device="cuda")    # rows padded to the widest tile
    W[:N] = (torch.randn(N, K, device="cuda") * 0.05).to(torch.bfloat16)
    ldc = (N + 7) // 8 * 8
    out = torch.empty(M, ldc, dtype=torch.bfloat16, device="cuda")
    return A, W, out, ldc


def _ours(A, W, out, ldc, M, N, K, variant):
    if variant == 0:
        st = B.dit_op_gemm(None, A.data_ptr(), K, W.data_ptr(), K, None, M, N, K, 0, out.data_ptr(), ldc, None, 0, None)
    else:
        st = B.dit_op_gemm_variant(None, A.data_ptr(), K, W.data_ptr(), K, None, M, N, K, 0, out.data_ptr(), ldc, variant)
    if st != 0:
        raise RuntimeError(f"gemm variant {variant} returned status {st}")


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--shapes", default="8192x8192x8192,18384x1536x6144,4250x6144x1536,4250x4608x1536,4250x1536x6144,4250x1536x1536")
    ap.add_argument("--variants", default="0")
    ap.add_argument("--rounds", type=int, default=4)
    ap.add_argument("--profile-run", action="store_true", help="three launches of variant 1256256 and three of torch.matmul per shape")
    args = ap.parse_args()
    shapes = [tuple(int(v) for v in s.split("x")) for s in args.shapes.split(",")]
    variants = [int(v) for v in args.variants.split(",")]
    for M, N, K in shapes:
        A, W, out, ldc = _operands(M, N, K)
        Wt = W[:N].t()
        if args.profile_run:
            for _ in range(3):
                _ours(A, W, out, ldc, M, N, K, 1256256)
            torch.cuda.synchronize()
            for _ in range(3):
                torch.matmul(A, Wt)
            torch.cuda.synchronize()
            continue
        ref = torch.matmul(A, Wt).float()
        cands = [str(v) for v in variants] + ["torch"]
        for v in variants:                      # every candidate is checked before it is timed
            out.zero_()
            _ours(A, W, out, ldc, M, N, K, v)
            torch.cuda.synchronize()
            err = ((out[:, :N].float() - ref).abs().max() / ref.abs().max()).item()
            if not err < 2e-2:
                raise RuntimeError(f"variant {v} differs from torch.matmul by {err:.3g} of the largest value")
        acc = {c: [] for c in cands}
        for r in range(args.rounds):
            order = cands[r % len(cands):] + cands[:r % len(cands)]
            if r % 2:
                order = order[::-1]
            for c in order:
                fn = (lambda: torch.matmul(A, Wt)) if c == "torch" else (lambda c=c: _ours(A, W, out, ldc, M, N, K, int(c)))
                acc[c].append(_time(fn))
        flop = 2.0 * M * N * K
        print(json.dumps({"M": M, "N": N, "K": K,
                          "candidates": {c: {"best_us": min(t) * 1e6, "mean_us": sum(t) / len(t) * 1e6, "best_tflops": flop / min(t) / 1e12}
                                         for c, t in acc.items()}}), flush=True)


if __name__ == "__main__":
    main()

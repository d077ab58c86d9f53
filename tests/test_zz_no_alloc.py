"""The allocation-free split-K entry point (scratch in the library's own device image) against
the entry point that takes the caller's scratch buffer: same kernels, so the outputs must agree
bit for bit, on two calls in a row, the second with a smaller input (the shared array then
still holds the first call's partial tiles)."""
import numpy as np
import pytest

import synth
from helpers import to_dev_bf16

pytestmark = pytest.mark.gpu


def rnd(seed, name, shape, std=1.0):
    return synth.gaussian_bf16(seed, name, int(np.prod(shape)), std).reshape(shape)


def test_static_scratch_split_k_matches_caller_scratch_on_two_calls():
    import torch
    from paper_2510_02838_amd import binding as B
    assert torch.cuda.is_available()
    n_req = 3
    # first a product that fills most of the array (240 of 256 partial tiles), then a smaller one
    for call, (M, N, K, splits) in enumerate([(300, 2500, 1536, 4), (154, 1000, 768, 5)]):
        A, W = rnd(1 + call, "A", (M, K)), rnd(3 + call, "W", (N, K), 0.05)
        bias = rnd(5 + call, "b", (N,), 0.5)
        gate = synth.gaussian(7 + call, "g", n_req * N).reshape(n_req, N)
        x0 = synth.gaussian(9 + call, "x", M * N).reshape(M, N)
        row_req = (np.arange(M) * n_req // M).astype(np.int32)
        npad = (N + 255) // 256 * 256
        Wp = np.zeros((npad, K), np.float32); Wp[:N] = W
        dA, dW = to_dev_bf16(torch, A), to_dev_bf16(torch, Wp)
        dg, db, dr = torch.from_numpy(gate).cuda(), torch.from_numpy(bias).cuda(), torch.from_numpy(row_req).cuda()
        tiles = ((M + 127) // 128) * ((N + 127) // 128)
        wb = tiles * splits * 65536
        assert wb <= 16 << 20
        work = torch.empty(wb, dtype=torch.uint8, device="cuda")
        ldc = (N + 7) // 8 * 8
        prod = A.astype(np.float64) @ W.astype(np.float64).T + bias
        for kind in (0, 1, 2, 3):
            def fresh():
                if kind == 3:
                    o = torch.zeros((M, ldc), dtype=torch.float32, device="cuda")
                    o[:, :N] = torch.from_numpy(x0).cuda()
                    return o
                return torch.full((M, ldc), float("nan"), dtype=torch.float32 if kind == 1 else torch.bfloat16, device="cuda")
            ref, got = fresh(), fresh()
            work.fill_(0xFF)
            g = dg.data_ptr() if kind == 3 else None
            r = dr.data_ptr() if kind == 3 else None
            assert B.dit_op_gemm_splitk(None, dA.data_ptr(), K, dW.data_ptr(), K, db.data_ptr(), M, N, K, kind,
                                        ref.data_ptr(), ldc, g, N, r, splits, work.data_ptr(), wb) == 0
            assert B.dit_op_gemm_splitk_static(None, dA.data_ptr(), K, dW.data_ptr(), K, db.data_ptr(), M, N, K, kind,
                                               got.data_ptr(), ldc, g, N, r, splits) == 0
            torch.cuda.synchronize()
            a, b = ref[:, :N].to(torch.float32).cpu().numpy(), got[:, :N].to(torch.float32).cpu().numpy()
            assert np.isfinite(b).all(), (call, kind)
            assert np.array_equal(a, b), (call, kind, float(np.abs(a - b).max()))
            # and both are the product (float64 reference, the GEMM tests' tolerance)
            if kind in (0, 1):
                err = np.abs(b - prod) / (np.abs(prod) + 1.0)
                assert err.max() <= (1e-4 if kind == 1 else 2.0 ** -8), (call, kind, err.max())
    # beyond the array: rejected before anything is launched
    big = torch.zeros((256, 4096), dtype=torch.bfloat16, device="cuda")
    dA, dW = to_dev_bf16(torch, rnd(1, "A", (256, 1024))), to_dev_bf16(torch, rnd(2, "W", (4096, 1024)))
    assert B.dit_op_gemm_splitk_static(None, dA.data_ptr(), 1024, dW.data_ptr(), 1024, None, 256, 4096, 1024, 0,
                                       big.data_ptr(), 4096, None, 0, None, 16) == 3      # 64 tiles x 16 shares x 64 KiB = 64 MiB
    torch.cuda.synchronize()
    assert not big.any()

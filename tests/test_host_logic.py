"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, and its
host logic (tensor table, size queries, argument validation) behaves.  No kernel runs."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import synth
from oracle import dit_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2510_02838_amd import binding
    return binding


def test_library_exports_every_declared_symbol(B):
    hdr = open(os.path.join(ROOT, "include", "dit.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(dit_[a-z_0-9]+)\s*\(", hdr))
    assert len(declared) >= 20
    for name in declared:
        assert hasattr(B.lib, name), f"{name} declared in dit.h but not exported"
    assert declared == set(B.EXPORTS)


@pytest.mark.parametrize("name", list(synth.CONFIGS))
def test_tensor_table_matches_oracle_parameter_list(B, name):
    arch = synth.CONFIGS[name]["arch"]
    m = B.DiT(arch, bind=False)
    shapes = O.param_shapes(arch)
    table = m.tensors()
    assert [t[0] for t in table] == list(shapes.keys())
    kinds = {"matrix": 0, "bias": 1, "gain": 2, "table": 3}
    for tname, r, c, k in table:
        shape, kind = shapes[tname]
        assert k == kinds[kind]
        assert (r, c) == (tuple(shape) if len(shape) == 2 else (1, shape[0]))
    # arena holds every matrix in bf16 (padded) and every vector in fp32
    n_params = sum(int(np.prod(s)) for s, _ in shapes.values())
    assert 2 * n_params <= m.weight_bytes() <= 2.2 * n_params + (1 << 22)
    m.close()


def test_workspace_size_grows_with_batch_and_steps(B):
    arch = synth.CONFIGS["tiny"]["arch"]
    m = B.DiT(arch, bind=False)
    a = m.workspace_bytes([(1, 16, 16, 16)], 4)
    b = m.workspace_bytes([(1, 16, 16, 16), (1, 32, 32, 16)], 4)
    c = m.workspace_bytes([(1, 16, 16, 16)], 28)
    assert 0 < a < b and a < c
    assert m.workspace_bytes([(1, 15, 16, 16)], 4) == 0      # not divisible by the patch
    assert m.workspace_bytes([(2, 16, 16, 16)], 4) == 0      # family J is single-frame
    assert m.workspace_bytes([(1, 16, 16, 0)], 4) == 0       # empty condition
    assert m.workspace_bytes([], 4) == 0
    assert m.workspace_bytes([(1, 16, 16, 16)], 0) == 0
    # tokens x widest activation row must stay below 2^31 elements (32-bit offsets in the kernels):
    # tiny has hidden 256, mlp 1024 -> 1280 columns -> at most 1 677 721 tokens, but also <= 2^20
    assert m.workspace_bytes([(1, 2048, 2044, 16)], 1) > 0       # 1 044 484 + 16 tokens
    assert m.workspace_bytes([(1, 2048, 2048, 16)], 1) == 0      # 2^20 + 16 tokens
    m.close()
    wan = B.DiT(synth.CONFIGS["wan"]["arch"], bind=False)       # 18944 columns -> at most 113 359 tokens
    assert wan.workspace_bytes([(21, 120, 176, 512)], 1) > 0     # 110 880 + 512 tokens
    assert wan.workspace_bytes([(21, 120, 180, 512)], 1) == 0    # 113 400 + 512 tokens
    wan.close()


def test_attention_plan_splits_the_last_round_of_same_shape_blocks(B):
    """Host arithmetic of the self-attention launch.  An XCD (32 CUs; 3 workgroups of 128 queries per CU at head
    size 64, 2 at head size 128, 1 of 256 queries) holds 96 / 64 / 32 workgroups at a time and owns n_heads/8
    heads; blocks that would make a partly filled last round are cut into key-split shares when that saves at
    least a quarter of a round."""
    sd3 = B.DiT(synth.CONFIGS["sd3"]["arch"], bind=False)
    # 4250 tokens: 34 blocks x 3 heads = 102 per XCD = 96 + 6: the last 2 blocks of every head in 4 shares
    assert sd3.attention_plan(synth.make_requests("sd3")) == (128, 34, 2, 4)
    assert sd3.attention_plan([(1, 96, 192, 154)]) == (128, 38, 6, 4)      # 114 per XCD: 18 over a round
    assert sd3.attention_plan([(1, 128, 128, 154)] * 2) == (128, 68, 4, 4) # same-shape batch: 204 = 2 x 96 + 12
    # 4 x 1146 tokens: 36 blocks per head, 108 per XCD; 18 key tiles per block allow two shares only (8 tiles each at least)
    assert sd3.attention_plan([(1, 62, 64, 154)] * 4) == (128, 36, 4, 2)
    assert sd3.attention_plan([(1, 32, 32, 154)])[2:] == (0, 1)            # 4 blocks: one round, nothing to split
    assert sd3.attention_plan([(1, 104, 104, 112)])[2:] == (0, 1)          # 66 per XCD: one round
    assert sd3.attention_plan(synth.make_requests("hetero8"))[2:] == (0, 1)   # mixed shapes: longest-first order instead
    sd3.close()
    flux = B.DiT(synth.CONFIGS["flux"]["arch"], bind=False)
    assert flux.attention_plan(synth.make_requests("flux")) == (128, 36, 0, 1)    # 108 per XCD: 4 shares would cost 0.79 rounds
    flux.close()
    wan = B.DiT(synth.CONFIGS["wan"]["arch"], bind=False)
    assert wan.attention_plan(synth.make_requests("wan")) == (256, 128, 0, 1)     # 640 per XCD = 20 full rounds of 32
    wan.close()
    tiny = B.DiT(synth.CONFIGS["tiny"]["arch"], bind=False)
    assert tiny.attention_plan([(1, 256, 256, 16)])[2:] == (0, 1)          # head count not a multiple of 8
    tiny.close()


def test_create_rejects_bad_configurations(B):
    base = synth.CONFIGS["tiny"]["arch"]
    def status(**kw):
        arch = dict(base); arch.update(kw)
        cfg = B.make_config(arch)
        ctx = C.c_void_p()
        st = B.dit_create(C.byref(cfg), 0, None, C.byref(ctx))
        if st == 0:
            B.dit_destroy(ctx)
        else:
            assert not ctx.value
        return st
    assert status() == 0
    assert status(hidden=250) == 2
    assert status(n_heads=3) == 2
    assert status(head_dim=32, n_heads=8) == 2
    assert status(mlp_hidden=1000) == 2
    assert status(cond_dim=100) == 2
    assert status(rope_axes=(10, 10, 10)) == 2
    assert status(n_single=3) == 2
    assert status(rope_axes=(16, 24, 24)) == 5       # rotary code with family J
    assert B.dit_create(None, 0, None, None) == 1


def test_calls_fail_cleanly_without_buffers(B):
    m = B.DiT(synth.CONFIGS["tiny"]["arch"], bind=False)
    assert B.dit_init_weights(m.ctx, 1, 0.02) == 1
    assert b"dit_bind" in B.dit_last_error(m.ctx)
    a = np.zeros(4, np.float32)
    assert B.dit_set_tensor(m.ctx, b"nope", a.ctypes.data_as(C.POINTER(C.c_float)), 4) == 1
    assert B.dit_bind(m.ctx, None, 0, None, 0) == 1
    assert B.dit_bind(m.ctx, 256, 16, 512, 16) == 3          # arena too small (never dereferenced)
    assert B.dit_bind(m.ctx, 257, 1 << 30, 512, 16) == 1     # misaligned
    reqs = B.make_reqs([(1, 16, 16, 16)])
    s = np.zeros(1, np.float32).ctypes.data_as(C.POINTER(C.c_float))
    assert B.dit_denoise_step(m.ctx, 1, reqs, 256, 256, s, s, 0, None) == 1   # nothing bound
    assert B.dit_denoise_step(None, 1, reqs, 256, 256, s, s, 0, None) == 1
    assert B.dit_op_gemm(None, None, 0, None, 0, None, 1, 1, 64, 0, None, 1, None, 0, None) == 1
    assert B.dit_op_gemm(None, 256, 64, 256, 64, None, 4, 4, 65, 0, 256, 4, None, 0, None) == 2
    assert B.dit_op_attention_work_bytes(0, None) == 0
    m.close()


def test_profiler_tool_host_logic():
    """The offline profiler's CPU-side pieces: the paper's 20 % batching rule (Appendix "Impact of
    Batch Size"), request-spec parsing, token counts and the decoder's product flop count."""
    from paper_2510_02838_amd import stage_profile as SP
    # largest B whose latency stays below 1.2 x latency(B = 1); B = 1 when even B = 2 exceeds it
    assert SP.optimal_batch({1: 1.0, 2: 1.05, 3: 1.19, 4: 1.21, 8: 2.0}) == 3
    assert SP.optimal_batch({1: 1.0, 2: 1.3, 4: 1.1}) == 4          # the rule looks at every B, not the first failure
    assert SP.optimal_batch({1: 2.0, 2: 2.5}) == 1
    cfg = synth.CONFIGS["sd3"]
    assert SP._latent_dims(cfg, "1024") == (1, 128, 128)
    assert SP._latent_dims(cfg, "480x832") == (1, 60, 104)
    assert SP._latent_dims(cfg, "81x480x832") == (21, 60, 104)
    assert SP._tokens(cfg["arch"], (1, 128, 128, 154)) == 4096 + 154
    # decoder flops by hand for a one-level decoder at a 4 x 4 latent: conv_in, two mid residual
    # blocks, the attention's four 1x1 products and two pixel products, one level block, conv_out
    arch = dict(latent_ch=4, out_ch=3, channels=(128,), n_res=1)
    px, c = 16, 128
    conv = lambda cin, cout, k: 2.0 * px * k * k * cin * cout
    want = conv(4, c, 3) + 3 * 2 * conv(c, c, 3) + 4 * conv(c, c, 1) + 4.0 * px * px * c + conv(c, 3, 3)
    assert SP.decoder_flops(arch, 4, 4) == want
    # a level change adds the shortcut and quadruples the pixels after the upsampling convolution
    arch2 = dict(latent_ch=4, out_ch=3, channels=(128, 64), n_res=1)
    up = 2.0 * (4 * px) * 9 * c * c
    lvl1 = 2.0 * (4 * px) * 9 * (c * 64 + 64 * 64) + 2.0 * (4 * px) * c * 64
    want2 = want - conv(c, 3, 3) + up + lvl1 + 2.0 * (4 * px) * 9 * 64 * 3
    assert SP.decoder_flops(arch2, 4, 4) == want2
    # video decoder: 27 taps, frames as pixels; with one frame-rate doubling 3 frames become 5 before
    # the upsampling convolution; the per-frame attention does not grow with the frame count squared
    v1 = dict(arch, t_up=0)
    want_v = 3 * (3 * (conv(4, c, 3) + 3 * 2 * conv(c, c, 3) + conv(c, 3, 3)) + 4 * conv(c, c, 1) + 4.0 * px * px * c)
    assert SP.video_decoder_flops(v1, 3, 4, 4) == want_v
    v2 = dict(arch2, t_up=1)
    lvl0 = 3 * (3 * (conv(4, c, 3) + 3 * 2 * conv(c, c, 3)) + 4 * conv(c, c, 1) + 4.0 * px * px * c)
    px1 = 5 * 4 * px
    want_v2 = lvl0 + 2.0 * px1 * 27 * c * c + 2.0 * px1 * 27 * (c * 64 + 64 * 64) + 2.0 * px1 * c * 64 + 2.0 * px1 * 27 * 64 * 3
    assert SP.video_decoder_flops(v2, 3, 4, 4) == want_v2

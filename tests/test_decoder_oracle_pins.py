"""Pins of the Decode-stage oracle (AutoencoderKL-style decoder) against brute force, closed
forms and invariants."""
import numpy as np
import pytest

import synth
from oracle import decoder_oracle as D

ARCH = synth.DECODERS["ae_tiny"]


def _params(arch=ARCH, seed=1, std=0.05, bias_std=0.1, gain_std=0.1):
    return synth.make_params(D.param_shapes(arch), seed, std, bias_std, gain_std)


def _rnd(seed, name, shape, std=1.0):
    return synth.gaussian(seed, name, int(np.prod(shape))).reshape(shape).astype(np.float64) * std


def test_conv_matches_six_nested_loops():
    x, w, b = _rnd(1, "x", (5, 4, 3)), _rnd(2, "w", (27, 2)), _rnd(3, "b", (2,))
    y = D.conv2d(x, w, b, 3)
    ref = np.zeros((5, 4, 2))
    for i in range(5):
        for j in range(4):
            for o in range(2):
                acc = b[o]
                for ky in range(3):
                    for kx in range(3):
                        ii, jj = i + ky - 1, j + kx - 1
                        if 0 <= ii < 5 and 0 <= jj < 4:
                            for c in range(3):
                                acc += x[ii, jj, c] * w[(ky * 3 + kx) * 3 + c, o]
                ref[i, j, o] = acc
    assert np.allclose(y, ref, atol=1e-12)


def test_conv_single_tap_shifts_and_centre_tap_is_identity():
    x = _rnd(1, "x", (6, 7, 4))
    w = np.zeros((36, 4)); w[4 * 4:5 * 4] = np.eye(4)                  # centre tap (ky, kx) = (1, 1)
    assert np.allclose(D.conv2d(x, w, np.zeros(4), 3), x)
    w = np.zeros((36, 4)); w[(0 * 3 + 2) * 4:(0 * 3 + 2) * 4 + 4] = np.eye(4)   # tap (0, 2): reads x[i-1][j+1]
    y = D.conv2d(x, w, np.zeros(4), 3)
    assert np.allclose(y[1:, :-1], x[:-1, 1:]) and np.all(y[0] == 0) and np.all(y[:, -1] == 0)
    w1 = _rnd(5, "w1", (4, 3))
    assert np.allclose(D.conv2d(x, w1, np.ones(3), 1), x @ w1 + 1.0)   # 1x1 convolution is a matmul


def test_group_norm_moments_membership_and_invariance():
    x = _rnd(1, "x", (4, 5, 64), 3.0) + 1.5
    y = D.group_norm(x, np.ones(64), np.zeros(64))
    g = y.reshape(20, 32, 2)
    assert np.allclose(g.mean(axis=(0, 2)), 0, atol=1e-12) and np.allclose(g.var(axis=(0, 2)), 1, atol=1e-5)
    x2 = x.copy(); x2[..., 10:12] = _rnd(2, "o", (4, 5, 2))           # group 5 only
    y2 = D.group_norm(x2, np.ones(64), np.zeros(64))
    keep = np.r_[0:10, 12:64]
    assert np.array_equal(y2[..., keep], y[..., keep]) and not np.allclose(y2[..., 10:12], y[..., 10:12])
    assert np.allclose(D.group_norm(2 * x + 7, np.ones(64), np.zeros(64)), y, atol=1e-6)    # affine invariance
    gain, beta = _rnd(3, "g", (64,)), _rnd(4, "b", (64,))
    assert np.allclose(D.group_norm(x, gain, beta), y * gain + beta)
    # one group of two channels over two pixels, by hand: values 1, 3, 5, 7 -> mean 4, var 5
    x = np.zeros((1, 2, 64)); x[0, 0, :2] = (1, 3); x[0, 1, :2] = (5, 7)
    y = D.group_norm(x, np.ones(64), np.zeros(64))
    assert np.allclose(y[0, :, :2].ravel(), (np.array([1, 3, 5, 7]) - 4) / np.sqrt(5 + 1e-6))


def test_upsample_and_silu():
    x = _rnd(1, "x", (3, 2, 5))
    y = D.upsample2(x)
    assert y.shape == (6, 4, 5)
    for i in range(6):
        for j in range(4):
            assert np.array_equal(y[i, j], x[i // 2, j // 2])
    v = np.array([-3.0, 0.0, 2.0])
    assert np.allclose(D.silu(v), v / (1 + np.exp(-v))) and D.silu(0.0) == 0.0
    assert np.allclose(D.silu(v) - D.silu(-v), v)                      # silu(x) - silu(-x) = x


def test_attention_limits():
    p = _params()
    m = D.DecoderOracle(ARCH, p)
    C = ARCH["channels"][0]
    x = _rnd(1, "x", (1, 1, C))                                         # one pixel: softmax is 1
    h = m.gn("mid.attn.gn", x)
    v = m.conv("mid.attn.v", h, 1)
    assert np.allclose(m.attn(x), x + m.conv("mid.attn.proj", v, 1), atol=1e-12)
    p2 = dict(p); p2["mid.attn.k.w"] = np.zeros_like(p["mid.attn.k.w"])  # equal keys: mean of the values
    m2 = D.DecoderOracle(ARCH, p2)
    x = _rnd(2, "x", (3, 4, C))
    v = m2.conv("mid.attn.v", m2.gn("mid.attn.gn", x), 1)
    mean_v = np.broadcast_to(v.reshape(12, C).mean(0), (3, 4, C))
    assert np.allclose(m2.attn(x), x + m2.conv("mid.attn.proj", mean_v, 1), atol=1e-10)


def test_residual_block_closed_forms():
    p = _params()
    for k in list(p):
        if k.startswith("mid.res0.conv2.w"):
            p[k] = np.zeros_like(p[k])
    m = D.DecoderOracle(ARCH, p)
    x = _rnd(1, "x", (4, 4, ARCH["channels"][0]))
    assert np.allclose(m.res("mid.res0", x), x + p["mid.res0.conv2.b"], atol=1e-12)     # identity shortcut
    name = "up2.res0"                                                   # 128 -> 64 channels: 1x1 shortcut
    assert (name + ".short.w") in p
    p[name + ".conv2.w"] = np.zeros_like(p[name + ".conv2.w"])
    x = _rnd(2, "x", (3, 3, 128))
    want = x @ p[name + ".short.w"].astype(np.float64) + p[name + ".short.b"] + p[name + ".conv2.b"]
    assert np.allclose(D.DecoderOracle(ARCH, p).res(name, x), want, atol=1e-12)


def test_forward_shape_and_zero_weight_closed_form():
    p = _params()
    z = _rnd(1, "z", (4, 6, ARCH["latent_ch"]))
    y = D.DecoderOracle(ARCH, p).forward(z)
    assert y.shape == (32, 48, 3) and np.isfinite(y).all()              # three 2x upsamplings
    pz = {k: (np.zeros_like(v) if k.endswith(".w") else v) for k, v in p.items()}
    y = D.DecoderOracle(ARCH, pz).forward(z)
    assert np.allclose(y, np.broadcast_to(p["conv_out.b"], y.shape), atol=1e-12)
    # input independence once conv_in is cut: only biases and norms of a zero field remain
    pc = dict(p); pc["conv_in.w"] = np.zeros_like(p["conv_in.w"])
    m = D.DecoderOracle(ARCH, pc)
    assert np.allclose(m.forward(z), m.forward(_rnd(9, "z2", z.shape)), atol=1e-12)


def test_parameter_count_of_the_autoencoder_decoder():
    shapes = D.param_shapes(synth.DECODERS["ae_kl"])
    n = sum(int(np.prod(s)) for s, _ in shapes.values())
    assert 48e6 < n < 51e6        # the published decoder has ~49.5 M parameters (the paper's table: 0.1 B for the whole autoencoder)

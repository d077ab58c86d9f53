"""Pins of the video decoder oracle: the causal 3x3x3 convolution against nested loops and a
library correlation, time shifts and causality, and the whole network against the (pinned) image
decoder oracle in the case where only the current-frame taps are non-zero."""
import numpy as np
from scipy import signal

import synth
from oracle import decoder_oracle as D
from oracle import video_decoder_oracle as V

ARCH = synth.VIDEO_DECODERS["vae3d_tiny"]


def _rnd(seed, name, shape, std=1.0):
    return synth.gaussian(seed, name, int(np.prod(shape))).reshape(shape).astype(np.float64) * std


def _params(arch=ARCH, seed=1):
    return synth.make_params(V.param_shapes(arch), seed, 0.05, 0.1, 0.1)


def test_causal_conv_matches_nested_loops():
    F, H, W, Ci, Co = 4, 3, 5, 2, 3
    x, w, b = _rnd(1, "x", (F, H, W, Ci)), _rnd(2, "w", (27 * Ci, Co)), _rnd(3, "b", (Co,))
    y = V.conv3d_causal(x, w, b)
    ref = np.zeros((F, H, W, Co))
    for f in range(F):
        for i in range(H):
            for j in range(W):
                for o in range(Co):
                    acc = b[o]
                    for kf in range(3):
                        for ky in range(3):
                            for kx in range(3):
                                ff, ii, jj = f + kf - 2, i + ky - 1, j + kx - 1
                                if ff >= 0 and 0 <= ii < H and 0 <= jj < W:
                                    for c in range(Ci):
                                        acc += x[ff, ii, jj, c] * w[((kf * 3 + ky) * 3 + kx) * Ci + c, o]
                    ref[f, i, j, o] = acc
    assert np.allclose(y, ref, atol=1e-12)


def test_causal_conv_matches_library_correlation():
    F, H, W, Ci, Co = 5, 6, 4, 3, 2
    x, w = _rnd(4, "x", (F, H, W, Ci)), _rnd(5, "w", (27 * Ci, Co))
    y = V.conv3d_causal(x, w, np.zeros(Co))
    xp = np.zeros((F + 2, H + 2, W + 2, Ci)); xp[2:, 1:-1, 1:-1] = x       # two frames in front, one pixel around
    k = w.reshape(3, 3, 3, Ci, Co)
    for o in range(Co):
        ref = sum(signal.correlate(xp[..., c], k[..., c, o], mode="valid") for c in range(Ci))
        assert np.allclose(y[..., o], ref, atol=1e-12)


def test_single_taps_delay_frames_and_the_last_tap_is_the_present():
    x = _rnd(1, "x", (5, 4, 4, 2))
    for kf in range(3):
        w = np.zeros((54, 2)); t = ((kf * 3 + 1) * 3 + 1) * 2; w[t:t + 2] = np.eye(2)     # centre pixel of frame tap kf
        y = V.conv3d_causal(x, w, np.zeros(2))
        d = 2 - kf
        assert np.array_equal(y[d:], x[:5 - d]) and np.all(y[:d] == 0)
    # no tap reaches a later frame: changing frame 3 leaves frames 0..2 as they were
    w = _rnd(2, "w", (54, 3))
    x2 = x.copy(); x2[3] += 1.0
    y, y2 = V.conv3d_causal(x, w, np.zeros(3)), V.conv3d_causal(x2, w, np.zeros(3))
    assert np.array_equal(y[:3], y2[:3]) and not np.allclose(y[3], y2[3]) and not np.allclose(y[4], y2[4])


def test_frame_rate_doubling_keeps_the_first_frame_once():
    x = np.arange(4.0).reshape(4, 1, 1, 1)
    assert V.upsample_frames(x).ravel().tolist() == [0, 1, 1, 2, 2, 3, 3]
    assert V.out_frames(dict(t_up=2), 13) == 49 and V.out_frames(dict(t_up=0), 5) == 5


def test_parameter_list_is_the_image_decoders_with_27_taps():
    a, b = D.param_shapes(ARCH), V.param_shapes(ARCH)
    assert list(a) == list(b)
    for n in a:
        (sa, ka), (sb, kb) = a[n], b[n]
        three = n.endswith(".w") and len(sa) == 2 and (".conv" in n or n.startswith("conv_") or ".upconv" in n)
        assert ka == kb and sb == ((3 * sa[0], sa[1]) if three else sa), n


def test_present_taps_only_reduce_to_the_image_decoder_per_frame():
    """With the taps of the two earlier frames zero the network sees each frame by itself, so
    every output frame is the image decoder's result for the latent frame it shows."""
    p3 = _params()
    p2 = {}
    for n, v in p3.items():
        if v.ndim == 2 and v.shape[0] == D.param_shapes(ARCH)[n][0][0] * 3:
            v = v.copy(); v[:2 * v.shape[0] // 3] = 0.0
            p3[n] = v
            p2[n] = v[2 * v.shape[0] // 3:]
        else:
            p2[n] = v
    z = _rnd(7, "z", (3, 4, 4, ARCH["latent_ch"]))
    got = V.VideoDecoderOracle(ARCH, p3).forward(z)
    img = D.DecoderOracle(ARCH, p2)
    src = [0, 1, 1, 2, 2]                                    # t_up = 1: 3 frames -> 5
    assert got.shape[0] == len(src)
    for g, f in enumerate(src):
        assert np.allclose(got[g], img.forward(z[f]), atol=1e-9), g


def test_network_is_causal_through_the_frame_rate_doubling():
    p = _params(seed=2)
    z = _rnd(8, "z", (3, 4, 4, ARCH["latent_ch"]))
    z2 = z.copy(); z2[2] += 0.5                              # the last latent frame: shown from output frame 3 on
    a, b = V.VideoDecoderOracle(ARCH, p).forward(z), V.VideoDecoderOracle(ARCH, p).forward(z2)
    assert np.array_equal(a[:3], b[:3]) and not np.allclose(a[3], b[3]) and not np.allclose(a[4], b[4])
    # the first latent frame reaches every output frame (each convolution looks two frames back)
    z3 = z.copy(); z3[0] += 0.5
    c = V.VideoDecoderOracle(ARCH, p).forward(z3)
    assert all(not np.allclose(a[g], c[g]) for g in range(5))

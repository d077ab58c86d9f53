"""Reference for the Decode stage of the video family (TEST INFRASTRUCTURE): the causal
three-dimensional form of the convolutional decoder in decoder_oracle.py, float64 NumPy.

The paper's pipeline table lists video models whose latents are decoded by causal 3-D
autoencoder decoders; it does not describe their inside.  The reading taken here keeps the
image decoder's structure and changes only what makes it a video decoder:

  * every 3x3 convolution becomes a causal 3x3x3 convolution: output frame f reads input
    frames f-2, f-1, f (frames before the first are zero), spatial zero padding as before;
  * 1x1 convolutions (shortcuts, attention projections), GroupNorm and the mid-block attention
    act on each frame by itself;
  * at the first t_up level transitions the frame rate doubles before the spatial upsampling:
    the first frame is kept once and every later frame twice (F frames -> 2F - 1), which is
    the inverse of a causal temporal compression that leaves the first frame alone.

Tensors are [F][H][W][C].  Only tests and a benchmark's CPU-baseline leg may import this module.
"""
import numpy as np

from . import decoder_oracle as D

F64 = np.float64


def param_shapes(arch):
    """As the image decoder's list, the 3x3 convolutions with 27 taps: input index
    ((kf*3 + ky)*3 + kx)*C_in + c, kf = 2 being the output's own frame."""
    return D.param_shapes(arch, kt=3)


def conv3d_causal(x, w, b):
    """x: [F][H][W][Cin]; w: [27*Cin][Cout].
    y[f][i][j][o] = b[o] + sum_{kf,ky,kx,c} x[f+kf-2][i+ky-1][j+kx-1][c] w[((kf*3+ky)*3+kx)*Cin+c][o],
    terms outside the video being zero."""
    F, H, W, Cin = x.shape
    xp = np.zeros((F + 2, H + 2, W + 2, Cin), F64)
    xp[2:, 1:H + 1, 1:W + 1] = x
    y = np.zeros((F, H, W, w.shape[1]), F64) + b
    for kf in range(3):
        for ky in range(3):
            for kx in range(3):
                t = ((kf * 3 + ky) * 3 + kx) * Cin
                y += xp[kf:kf + F, ky:ky + H, kx:kx + W].reshape(F * H * W, Cin).dot(w[t:t + Cin]).reshape(F, H, W, -1)
    return y


def upsample_frames(x):
    """F frames -> 2F - 1: output frame g shows input frame (g + 1) // 2."""
    F = x.shape[0]
    return x[(np.arange(2 * F - 1) + 1) // 2]


def out_frames(arch, F):
    for _ in range(arch["t_up"]):
        F = 2 * F - 1
    return F


class VideoDecoderOracle:
    def __init__(self, arch, params):
        self.arch = arch
        self.p = {k: np.asarray(v, F64) for k, v in params.items()}

    def conv3(self, name, x):
        return conv3d_causal(x, self.p[name + ".w"], self.p[name + ".b"])

    def conv1(self, name, x):
        return x @ self.p[name + ".w"] + self.p[name + ".b"]

    def gn(self, name, x):
        return np.stack([D.group_norm(f, self.p[name + ".g"], self.p[name + ".b"]) for f in x])

    def res(self, name, x):
        h = self.conv3(name + ".conv1", D.silu(self.gn(name + ".gn1", x)))
        h = self.conv3(name + ".conv2", D.silu(self.gn(name + ".gn2", h)))
        sc = self.conv1(name + ".short", x) if (name + ".short.w") in self.p else x
        return sc + h

    def attn(self, x):
        F, H, W, C = x.shape
        h = self.gn("mid.attn.gn", x)
        out = []
        for f in range(F):
            q, k, v = (self.conv1("mid.attn." + n, h[f]).reshape(H * W, C) for n in ("q", "k", "v"))
            out.append((D.softmax_rows(q @ k.T / np.sqrt(C)) @ v).reshape(H, W, C))
        return x + self.conv1("mid.attn.proj", np.stack(out))

    def forward(self, z, taps=None):
        """z: [F][h][w][latent_ch] -> video [F'][h * 2^(levels-1)][w * 2^(levels-1)][out_ch],
        F' = out_frames(arch, F)."""
        a = self.arch
        h = self.conv3("conv_in", np.asarray(z, F64))
        h = self.res("mid.res0", h)
        if taps is not None:
            taps["mid.res0"] = h
        h = self.attn(h)
        if taps is not None:
            taps["mid.attn"] = h
        h = self.res("mid.res1", h)
        for l in range(len(a["channels"])):
            for r in range(a["n_res"]):
                h = self.res(f"up{l}.res{r}", h)
            if taps is not None:
                taps[f"up{l}"] = h
            if l != len(a["channels"]) - 1:
                if l < a["t_up"]:
                    h = upsample_frames(h)
                h = self.conv3(f"up{l}.upconv", np.stack([D.upsample2(f) for f in h]))
        return self.conv3("conv_out", D.silu(self.gn("out.gn", h)))

"""Reference for the Decode stage (TEST INFRASTRUCTURE): an AutoencoderKL-style convolutional
decoder in float64 NumPy, every step written out plainly.

The paper's Decode stage maps the latent result to pixel space with a memory-bound decoder
(Section 2.1; its batch-size figure names AutoEncoderKL); it does not describe the decoder's
inside, so the published AutoencoderKL decoder structure is the reading taken here:

  h = conv3x3(z)                                              latent channels -> ch[0]
  mid:   h = Res(h); h = h + proj(attention(GN(h)));  h = Res(h)      (one head over all pixels)
  for each level l:  n_res x  h = Res(h)  (channels ch[l-1] -> ch[l] in the first one)
                     if not last: h = conv3x3(upsample_nearest_2x(h))
  y = conv3x3(SiLU(GN(h)))                                    ch[-1] -> out channels (3)
  Res(x) = shortcut(x) + conv3x3(SiLU(GN(conv3x3(SiLU(GN(x))))))   shortcut = 1x1 conv if the
           channel count changes, identity otherwise
  GN: GroupNorm with 32 groups, eps 1e-6, affine; all convolutions have a bias and zero padding;
  attention: q, k, v, proj are 1x1 convolutions, softmax(q k^T / sqrt(C)) v over the H*W pixels.

Tensors are channels-last: [H][W][C].  Only tests and a benchmark's CPU-baseline leg may import
this module.
"""
import numpy as np

F64 = np.float64
GN_GROUPS = 32
GN_EPS = 1e-6


def param_shapes(arch, kt=1):
    """{name: (shape, kind)}; conv weights are matrices [taps*C_in, C_out] with the input index
    (ky*3 + kx)*C_in + c (1x1: just c).  kt = 3: the 3x3 convolutions also span three frames
    (the video decoder's), input index ((kf*3 + ky)*3 + kx)*C_in + c."""
    ch, zc, oc = arch["channels"], arch["latent_ch"], arch["out_ch"]
    out = {}

    def conv(name, cin, cout, k):
        out[name + ".w"] = (((kt if k == 3 else 1) * k * k * cin, cout), "matrix")
        out[name + ".b"] = ((cout,), "bias")

    def gn(name, c):
        out[name + ".g"] = ((c,), "gain")
        out[name + ".b"] = ((c,), "bias")

    def res(name, cin, cout):
        gn(name + ".gn1", cin); conv(name + ".conv1", cin, cout, 3)
        gn(name + ".gn2", cout); conv(name + ".conv2", cout, cout, 3)
        if cin != cout:
            conv(name + ".short", cin, cout, 1)

    conv("conv_in", zc, ch[0], 3)
    res("mid.res0", ch[0], ch[0])
    gn("mid.attn.gn", ch[0])
    for n in ("q", "k", "v", "proj"):
        conv("mid.attn." + n, ch[0], ch[0], 1)
    res("mid.res1", ch[0], ch[0])
    prev = ch[0]
    for l, c in enumerate(ch):
        for r in range(arch["n_res"]):
            res(f"up{l}.res{r}", prev if r == 0 else c, c)
        prev = c
        if l != len(ch) - 1:
            conv(f"up{l}.upconv", c, c, 3)
    gn("out.gn", ch[-1])
    conv("conv_out", ch[-1], oc, 3)
    return out


def silu(x):
    return x / (1.0 + np.exp(-x))


def group_norm(x, gain, beta, groups=GN_GROUPS):
    """x: [H][W][C]; statistics over (H, W, C/groups) per group, biased variance."""
    H, W, C = x.shape
    g = x.reshape(H * W, groups, C // groups)
    mean = g.mean(axis=(0, 2), keepdims=True)
    var = ((g - mean) ** 2).mean(axis=(0, 2), keepdims=True)
    y = ((g - mean) / np.sqrt(var + GN_EPS)).reshape(H, W, C)
    return y * gain + beta


def conv2d(x, w, b, k):
    """x: [H][W][Cin]; w: [k*k*Cin][Cout] with input index (ky*k + kx)*Cin + c; zero padding
    (k-1)/2, stride 1: y[i][j][o] = b[o] + sum_{ky,kx,c} x[i+ky-p][j+kx-p][c] w[(ky*k+kx)*Cin+c][o]."""
    H, W, Cin = x.shape
    p = (k - 1) // 2
    xp = np.zeros((H + 2 * p, W + 2 * p, Cin), F64)
    xp[p:p + H, p:p + W] = x
    y = np.zeros((H, W, w.shape[1]), F64) + b
    for ky in range(k):
        for kx in range(k):
            t = (ky * k + kx) * Cin
            y += xp[ky:ky + H, kx:kx + W].reshape(H * W, Cin).dot(w[t:t + Cin]).reshape(H, W, -1)
    return y


def upsample2(x):
    """Nearest-neighbour 2x: y[i][j] = x[i//2][j//2]."""
    return np.repeat(np.repeat(x, 2, axis=0), 2, axis=1)


def softmax_rows(s):
    m = s.max(axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / e.sum(axis=-1, keepdims=True)


class DecoderOracle:
    def __init__(self, arch, params):
        self.arch = arch
        self.p = {k: np.asarray(v, F64) for k, v in params.items()}

    def conv(self, name, x, k):
        return conv2d(x, self.p[name + ".w"], self.p[name + ".b"], k)

    def gn(self, name, x):
        return group_norm(x, self.p[name + ".g"], self.p[name + ".b"])

    def res(self, name, x):
        h = self.conv(name + ".conv1", silu(self.gn(name + ".gn1", x)), 3)
        h = self.conv(name + ".conv2", silu(self.gn(name + ".gn2", h)), 3)
        sc = self.conv(name + ".short", x, 1) if (name + ".short.w") in self.p else x
        return sc + h

    def attn(self, x):
        H, W, C = x.shape
        h = self.gn("mid.attn.gn", x)
        q, k, v = (self.conv("mid.attn." + n, h, 1).reshape(H * W, C) for n in ("q", "k", "v"))
        o = softmax_rows(q @ k.T / np.sqrt(C)) @ v
        return x + self.conv("mid.attn.proj", o.reshape(H, W, C), 1)

    def forward(self, z, taps=None):
        """z: [h][w][latent_ch] -> image [h * 2^(levels-1)][w * 2^(levels-1)][out_ch]."""
        a = self.arch
        h = self.conv("conv_in", np.asarray(z, F64), 3)
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
                h = self.conv(f"up{l}.upconv", upsample2(h), 3)
        return self.conv("conv_out", silu(self.gn("out.gn", h)), 3)

"""Reference (oracle) implementation of the Diffuse stage: T-step denoising of a latent
through a diffusion transformer.

THIS IS TEST INFRASTRUCTURE.  It is a plain, slow float64 NumPy program, one request at a
time, that only tests, the smoke check and the benchmark's CPU-baseline leg may call.  It
shares no code with the GPU library and must never be used as a product code path.

What it computes (paper section 2.1, the equation defining the Diffuse stage):

    eps_t   = eps_theta(x_t, t, c)          -- `DiTOracle.velocity`
    x_{t-1} = Phi(x_t, t, eps_t)            -- `update_coefficients` / `DiTOracle.step`

starting from Gaussian x_T, for T steps (`DiTOracle.sample`); section 1 states that the
latent is concatenated with the condition c, which here is the joint [text; image] token
sequence every attention runs over.  The paper does not describe the inside of eps_theta;
the three block families below follow the benchmark configurations (J: joint two-stream
blocks; F: double-stream then single-stream blocks with rotary positions; W: self-attention,
cross-attention and MLP blocks with 3-axis rotary positions).  Each function's docstring
states the reading it takes where the paper leaves a detail open.

All arithmetic is float64.  No blocking, fusion or reordering: softmax is the two-pass
definition, attention materialises the score matrix, linear layers are one matmul.

Pins (tests that tie each function to something other than itself) live in
tests/test_oracle_pins.py.  Full-depth full-shape runs of the two largest configurations
are not affordable on the CPU: for them parity is unpinned except by composition of
reduced-depth and row-sampled runs.
"""
import math

import numpy as np

F64 = np.float64
LN_EPS = 1e-6
RMS_EPS = 1e-6
T_FREQ_DIM = 256  # width of the sinusoidal timestep feature


# ----------------------------------------------------------------------------------------
# parameter table
# ----------------------------------------------------------------------------------------
def param_shapes(arch):
    """{name: (logical shape, kind)}; matrices are [in, out] (y = x @ W + b)."""
    d, dh, dff = arch["hidden"], arch["head_dim"], arch["mlp_hidden"]
    pt, ph, pw = arch["patch"]
    pdim = arch["latent_ch"] * pt * ph * pw
    fam = arch["family"]
    t = {}

    def lin(name, i, o):
        t[name + ".w"] = ((i, o), "matrix")
        t[name + ".b"] = ((o,), "bias")

    def stream_block(p):
        lin(p + ".mod", d, 6 * d)
        lin(p + ".qkv", d, 3 * d)
        t[p + ".qnorm.g"] = ((dh,), "gain")
        t[p + ".knorm.g"] = ((dh,), "gain")
        lin(p + ".proj", d, d)
        lin(p + ".mlp1", d, dff)
        lin(p + ".mlp2", dff, d)

    lin("t_embed.1", T_FREQ_DIM, d)
    lin("t_embed.2", d, d)
    lin("x_embed", pdim, d)
    lin("c_embed", arch["cond_dim"], d)
    if fam == "J":
        for l in range(arch["n_blocks"]):
            for s in ("txt", "img"):
                stream_block(f"blk{l}.{s}")
    elif fam == "F":
        for l in range(arch["n_blocks"]):
            for s in ("txt", "img"):
                stream_block(f"dbl{l}.{s}")
        for l in range(arch["n_single"]):
            p = f"sgl{l}"
            lin(p + ".mod", d, 3 * d)
            lin(p + ".lin1", d, 3 * d + dff)
            t[p + ".qnorm.g"] = ((dh,), "gain")
            t[p + ".knorm.g"] = ((dh,), "gain")
            lin(p + ".lin2", d + dff, d)
    elif fam == "W":
        lin("t_proj", d, 6 * d)
        for l in range(arch["n_blocks"]):
            p = f"blk{l}"
            t[p + ".mod_table"] = ((6, d), "table")
            lin(p + ".qkv", d, 3 * d)
            t[p + ".qnorm.g"] = ((dh,), "gain")
            t[p + ".knorm.g"] = ((dh,), "gain")
            lin(p + ".proj", d, d)
            t[p + ".xnorm.g"] = ((d,), "gain")
            t[p + ".xnorm.b"] = ((d,), "bias")
            lin(p + ".xq", d, d)
            lin(p + ".xkv", d, 2 * d)
            t[p + ".xqnorm.g"] = ((dh,), "gain")
            t[p + ".xknorm.g"] = ((dh,), "gain")
            lin(p + ".xproj", d, d)
            lin(p + ".mlp1", d, dff)
            lin(p + ".mlp2", dff, d)
    else:
        raise ValueError(fam)
    lin("final.mod", d, 2 * d)
    lin("final", d, pdim)
    return t


# ----------------------------------------------------------------------------------------
# elementary functions
# ----------------------------------------------------------------------------------------
def silu(x):
    return x / (1.0 + np.exp(-x))


def gelu_tanh(x):
    return 0.5 * x * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (x + 0.044715 * x ** 3)))


def layer_norm(x, eps=LN_EPS):
    """Row-wise (x - mean) / sqrt(var + eps), biased variance, no affine."""
    mu = x.mean(axis=-1, keepdims=True)
    xc = x - mu
    var = (xc * xc).mean(axis=-1, keepdims=True)
    return xc / np.sqrt(var + eps)


def rms_norm(x, gain, eps=RMS_EPS):
    """Row-wise x / sqrt(mean(x^2) + eps) * gain over the last axis."""
    ms = (x * x).mean(axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def modulate(x, shift, scale):
    return layer_norm(x) * (1.0 + scale) + shift


def softmax_rows(s):
    """Two-pass softmax over the last axis: subtract the row max, exponentiate, normalise."""
    m = s.max(axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / e.sum(axis=-1, keepdims=True)


def attention(q, k, v):
    """softmax(q k^T / sqrt(d_h)) v for one head.  q: [nq, dh], k: [nk, dh], v: [nk, dh]."""
    s = (q @ k.T) / math.sqrt(q.shape[-1])
    return softmax_rows(s) @ v


def multi_head_attention(q, k, v, n_heads):
    """q: [nq, H*dh], k, v: [nk, H*dh] with head-major columns -> [nq, H*dh]."""
    nq, d = q.shape
    dh = d // n_heads
    out = np.empty((nq, d), dtype=F64)
    for h in range(n_heads):
        sl = slice(h * dh, (h + 1) * dh)
        out[:, sl] = attention(q[:, sl], k[:, sl], v[:, sl])
    return out


def timestep_features(sigma):
    """[cos(tau f_k), sin(tau f_k)], tau = 1000 sigma, f_k = exp(-ln(1e4) k / 128), k < 128."""
    half = T_FREQ_DIM // 2
    f = np.exp(-math.log(10000.0) * np.arange(half, dtype=F64) / half)
    a = 1000.0 * float(sigma) * f
    return np.concatenate([np.cos(a), np.sin(a)])


def sincos_pe(gh, gw, d):
    """Absolute 2-D position code for a gh x gw token grid (row-major tokens):
    [sin(i w), cos(i w), sin(j w), cos(j w)], each d/4 wide, w_k = 1e4^(-k/(d/4))."""
    q = d // 4
    w = 10000.0 ** (-np.arange(q, dtype=F64) / q)
    i = np.repeat(np.arange(gh, dtype=F64), gw)[:, None] * w[None, :]
    j = np.tile(np.arange(gw, dtype=F64), gh)[:, None] * w[None, :]
    return np.concatenate([np.sin(i), np.cos(i), np.sin(j), np.cos(j)], axis=1)


def patchify(x, patch):
    """[C, F, H, W] -> [n_tokens, C*pt*ph*pw]; token (f, i, j) row-major, feature
    ((c*pt + dt)*ph + dh)*pw + dw."""
    c, f, h, w = x.shape
    pt, ph, pw = patch
    gf, gh, gw = f // pt, h // ph, w // pw
    y = x.reshape(c, gf, pt, gh, ph, gw, pw)
    y = y.transpose(1, 3, 5, 0, 2, 4, 6)  # gf, gh, gw, c, pt, ph, pw
    return y.reshape(gf * gh * gw, c * pt * ph * pw)


def unpatchify(y, shape, patch):
    """Inverse of `patchify` for a latent of the given [C, F, H, W] shape."""
    c, f, h, w = shape
    pt, ph, pw = patch
    gf, gh, gw = f // pt, h // ph, w // pw
    x = y.reshape(gf, gh, gw, c, pt, ph, pw).transpose(3, 0, 4, 1, 5, 2, 6)
    return x.reshape(c, f, h, w)


def token_positions(gf, gh, gw):
    """Integer (frame, row, col) of every image token, row-major."""
    f, i, j = np.meshgrid(np.arange(gf), np.arange(gh), np.arange(gw), indexing="ij")
    return np.stack([f.ravel(), i.ravel(), j.ravel()], axis=1).astype(F64)


def rope(x, pos, axes, theta):
    """Rotary position code on x: [n, H, dh].  The head dimension is cut into per-axis chunks
    of widths `axes`; inside a chunk of width D pair (2j, 2j+1) is rotated by the angle
    pos_axis * theta^(-2j/D).  pos: [n, 3]."""
    out = x.copy()
    off = 0
    for a, width in enumerate(axes):
        if width == 0:
            continue
        jj = np.arange(width // 2, dtype=F64)
        ang = pos[:, a][:, None] * theta ** (-2.0 * jj / width)[None, :]  # [n, width/2]
        c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
        x0 = x[:, :, off:off + width:2]
        x1 = x[:, :, off + 1:off + width:2]
        out[:, :, off:off + width:2] = x0 * c - x1 * s
        out[:, :, off + 1:off + width:2] = x0 * s + x1 * c
        off += width
    return out


def update_coefficients(kind, sigma_cur, sigma_next):
    """(a, b) of the affine latent update x <- a x + b v.

    kind 0, Euler step of the flow-matching ODE: a = 1, b = sigma_next - sigma_cur.
    kind 1, deterministic DDIM with alpha_bar = 1 - sigma^2:
        a = sqrt(abar_next / abar_cur),
        b = sqrt(1 - abar_next) - sqrt(abar_next (1 - abar_cur) / abar_cur).
    """
    sc, sn = float(sigma_cur), float(sigma_next)
    if kind == 0:
        return 1.0, sn - sc
    if kind == 1:
        ac, an = 1.0 - sc * sc, 1.0 - sn * sn
        if ac <= 0.0:
            raise ValueError("DDIM needs sigma_cur < 1")
        return math.sqrt(an / ac), math.sqrt(1.0 - an) - math.sqrt(an * (1.0 - ac) / ac)
    raise ValueError(kind)


# ----------------------------------------------------------------------------------------
# the model
# ----------------------------------------------------------------------------------------
class DiTOracle:
    """eps_theta and the sampling loop for one request at a time.

    arch: dict with the keys of `synth.CONFIGS[...]['arch']`.
    params: {name: array} with the shapes of `param_shapes(arch)`.
    """

    def __init__(self, arch, params):
        self.arch = dict(arch)
        self.p = params
        assert arch["hidden"] == arch["n_heads"] * arch["head_dim"]

    # -- helpers ------------------------------------------------------------------------
    def _w(self, name):
        return np.asarray(self.p[name], dtype=F64)

    def _lin(self, x, name):
        return x @ self._w(name + ".w") + self._w(name + ".b")

    def _heads(self, x):
        return x.reshape(x.shape[0], self.arch["n_heads"], self.arch["head_dim"])

    def _qk_norm_rope(self, q, k, prefix, pos):
        """Per-head RMS norm of q and k, then the rotary code where `pos` is given."""
        a = self.arch
        qh = rms_norm(self._heads(q), self._w(prefix + "qnorm.g"))
        kh = rms_norm(self._heads(k), self._w(prefix + "knorm.g"))
        if pos is not None and sum(a["rope_axes"]) > 0:
            qh = rope(qh, pos, a["rope_axes"], a["rope_theta"])
            kh = rope(kh, pos, a["rope_axes"], a["rope_theta"])
        n = q.shape[0]
        return qh.reshape(n, -1), kh.reshape(n, -1)

    def conditioning(self, sigma):
        """vec = W2 SiLU(W1 s + b1) + b2 from the sinusoidal feature s; returns SiLU(vec)."""
        s = timestep_features(sigma)
        vec = self._lin(silu(self._lin(s, "t_embed.1")), "t_embed.2")
        return silu(vec)

    # -- blocks -------------------------------------------------------------------------
    def _joint_block(self, p, xt, xi, m, pos_t, pos_i, tap):
        """Two-stream block: each stream has its own weights, attention is joint."""
        d = self.arch["hidden"]
        H = self.arch["n_heads"]
        nt = xt.shape[0]
        mods, qs, ks, vs = {}, [], [], []
        for s, x, pos in (("txt", xt, pos_t), ("img", xi, pos_i)):
            mod = self._lin(m, f"{p}.{s}.mod")
            mods[s] = [mod[i * d:(i + 1) * d] for i in range(6)]
            sh1, sc1 = mods[s][0], mods[s][1]
            h = modulate(x, sh1, sc1)
            tap(f"{p}.{s}.ln1", h)
            qkv = self._lin(h, f"{p}.{s}.qkv")
            tap(f"{p}.{s}.qkv", qkv)
            q, k, v = qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:]
            q, k = self._qk_norm_rope(q, k, f"{p}.{s}.", pos)
            qs.append(q), ks.append(k), vs.append(v)
        q, k, v = np.concatenate(qs), np.concatenate(ks), np.concatenate(vs)
        tap(f"{p}.q", q), tap(f"{p}.k", k), tap(f"{p}.v", v)
        o = multi_head_attention(q, k, v, H)
        tap(f"{p}.attn", o)
        outs = []
        for s, x, oo in (("txt", xt, o[:nt]), ("img", xi, o[nt:])):
            _, _, g1, sh2, sc2, g2 = mods[s]
            x = x + g1 * self._lin(oo, f"{p}.{s}.proj")
            tap(f"{p}.{s}.x_attn", x)
            h = modulate(x, sh2, sc2)
            u = gelu_tanh(self._lin(h, f"{p}.{s}.mlp1"))
            tap(f"{p}.{s}.mlp_act", u)
            x = x + g2 * self._lin(u, f"{p}.{s}.mlp2")
            tap(f"{p}.{s}.x_out", x)
            outs.append(x)
        return outs[0], outs[1]

    def _single_block(self, p, x, m, pos, tap):
        """Single-stream block on the concatenated [text; image] sequence."""
        d = self.arch["hidden"]
        mod = self._lin(m, p + ".mod")
        sh, sc, g = mod[:d], mod[d:2 * d], mod[2 * d:]
        h = modulate(x, sh, sc)
        y = self._lin(h, p + ".lin1")
        tap(p + ".lin1", y)
        q, k, v, u = y[:, :d], y[:, d:2 * d], y[:, 2 * d:3 * d], y[:, 3 * d:]
        q, k = self._qk_norm_rope(q, k, p + ".", pos)
        o = multi_head_attention(q, k, v, self.arch["n_heads"])
        tap(p + ".attn", o)
        x = x + g * self._lin(np.concatenate([o, gelu_tanh(u)], axis=1), p + ".lin2")
        tap(p + ".x_out", x)
        return x

    def _w_block(self, p, x, cproj, e_base, pos, tap, rows=None):
        """Self-attention, cross-attention to the projected condition, MLP.

        rows: optional index array.  Keys and values are still formed from every token, but the
        query side and everything after it are evaluated for these tokens only and only their
        rows are returned (the same formulas on fewer rows; used on the last block of a model
        whose full score matrix is too large for the CPU)."""
        d = self.arch["hidden"]
        H = self.arch["n_heads"]
        e = self._w(p + ".mod_table") + e_base.reshape(6, d)
        sh1, sc1, g1, sh2, sc2, g2 = (e[i] for i in range(6))
        h = modulate(x, sh1, sc1)
        qkv = self._lin(h, p + ".qkv")
        q, k, v = qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:]
        q, k = self._qk_norm_rope(q, k, p + ".", pos)
        if rows is not None:
            q, x = q[rows], x[rows]
        o = multi_head_attention(q, k, v, H)
        tap(p + ".attn", o)
        x = x + g1 * self._lin(o, p + ".proj")
        tap(p + ".x_attn", x)
        # cross-attention: pre-norm is LayerNorm with affine, no modulation, no gate
        hx = layer_norm(x) * self._w(p + ".xnorm.g") + self._w(p + ".xnorm.b")
        q = self._lin(hx, p + ".xq")
        kv = self._lin(cproj, p + ".xkv")
        k, v = kv[:, :d], kv[:, d:]
        qh = rms_norm(self._heads(q), self._w(p + ".xqnorm.g")).reshape(q.shape[0], -1)
        kh = rms_norm(self._heads(k), self._w(p + ".xknorm.g")).reshape(k.shape[0], -1)
        ox = multi_head_attention(qh, kh, v, H)
        tap(p + ".xattn", ox)
        x = x + self._lin(ox, p + ".xproj")
        tap(p + ".x_cross", x)
        h = modulate(x, sh2, sc2)
        u = gelu_tanh(self._lin(h, p + ".mlp1"))
        x = x + g2 * self._lin(u, p + ".mlp2")
        tap(p + ".x_out", x)
        return x

    # -- eps_theta ----------------------------------------------------------------------
    def velocity(self, latent, cond, sigma, taps=None):
        """eps_theta(x_t, t, c): latent [C, F, H, W], cond [n_cond, d_c] -> [C, F, H, W]."""
        a = self.arch
        d = a["hidden"]
        pt, ph, pw = a["patch"]
        latent = np.asarray(latent, dtype=F64)
        cond = np.asarray(cond, dtype=F64)
        _, f, h, w = latent.shape
        gf, gh, gw = f // pt, h // ph, w // pw

        def tap(name, val):
            if taps is not None:
                taps[name] = np.array(val, dtype=F64, copy=True)

        m = self.conditioning(sigma)
        tap("m", m)
        xi = self._lin(patchify(latent, a["patch"]), "x_embed")
        if a["family"] == "J":
            if gf != 1:
                raise ValueError("family J takes single-frame latents")
            xi = xi + sincos_pe(gh, gw, d)
        xt = self._lin(cond, "c_embed")
        tap("x_img0", xi), tap("x_txt0", xt)
        pos_i = token_positions(gf, gh, gw)
        pos_t = np.zeros((xt.shape[0], 3), dtype=F64)
        nt = xt.shape[0]

        if a["family"] == "J":
            for l in range(a["n_blocks"]):
                xt, xi = self._joint_block(f"blk{l}", xt, xi, m, None, None, tap)
        elif a["family"] == "F":
            for l in range(a["n_blocks"]):
                xt, xi = self._joint_block(f"dbl{l}", xt, xi, m, pos_t, pos_i, tap)
            x = np.concatenate([xt, xi])
            pos = np.concatenate([pos_t, pos_i])
            for l in range(a["n_single"]):
                x = self._single_block(f"sgl{l}", x, m, pos, tap)
            xi = x[nt:]
        else:
            e_base = self._lin(m, "t_proj")
            for l in range(a["n_blocks"]):
                xi = self._w_block(f"blk{l}", xi, xt, e_base, pos_i, tap)

        mod = self._lin(m, "final.mod")
        y = self._lin(modulate(xi, mod[:d], mod[d:]), "final")
        tap("final", y)
        return unpatchify(y, latent.shape, a["patch"])

    def final_rows_w(self, latent, cond, sigma, rows, taps=None):
        """Family W only: the final layer's output rows (before unpatchify) for the image tokens
        `rows`, with the LAST block evaluated for those query rows only (see `_w_block`).  For a
        one-block model this is exact at any token count."""
        a = self.arch
        assert a["family"] == "W"
        d = a["hidden"]
        pt, ph, pw = a["patch"]
        latent = np.asarray(latent, dtype=F64)
        cond = np.asarray(cond, dtype=F64)
        _, f, h, w = latent.shape
        m = self.conditioning(sigma)
        xi = self._lin(patchify(latent, a["patch"]), "x_embed")
        xt = self._lin(cond, "c_embed")
        pos_i = token_positions(f // pt, h // ph, w // pw)
        e_base = self._lin(m, "t_proj")
        nb = a["n_blocks"]
        for l in range(nb):
            def tap(name, val, last=(l == nb - 1)):
                if taps is not None and last:
                    taps[name] = np.array(val, dtype=F64, copy=True)
            xi = self._w_block(f"blk{l}", xi, xt, e_base, pos_i, tap,
                               rows=rows if l == nb - 1 else None)
        mod = self._lin(m, "final.mod")
        return self._lin(modulate(xi, mod[:d], mod[d:]), "final")

    # -- Phi and the loop ---------------------------------------------------------------
    def step(self, latent, cond, sigma_cur, sigma_next, kind=0, taps=None):
        """One denoising step; returns (x_next, v)."""
        v = self.velocity(latent, cond, sigma_cur, taps)
        ca, cb = update_coefficients(kind, sigma_cur, sigma_next)
        return ca * np.asarray(latent, dtype=F64) + cb * v, v

    def sample(self, latent, cond, sigmas, kind=0):
        """T steps along sigmas[0..T]; returns the final latent."""
        x = np.asarray(latent, dtype=F64)
        for j in range(len(sigmas) - 1):
            x, _ = self.step(x, cond, sigmas[j], sigmas[j + 1], kind)
        return x

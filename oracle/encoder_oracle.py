"""Reference for the Encode stage (TEST INFRASTRUCTURE): a T5-v1.1-style text encoder in
float64 NumPy, one sequence at a time, every step written out plainly.

The paper's Encode stage embeds the prompt into the condition c with a Transformer encoder
(Section 2.1; its Table of pipelines names T5-XXL, 4.8 B parameters, 30-500 tokens); it does
not describe the encoder's inside, so the published T5-v1.1 encoder architecture is the
reading taken here:

  x = E[token]
  per layer:  h = RMSNorm(x) * g1            (no mean subtraction, eps 1e-6, no bias anywhere)
              q, k, v = h Wq, h Wk, h Wv;  scores = q k^T + bias[head][bucket(j - i)]   (NO 1/sqrt(d))
              x = x + softmax(scores) v Wo
              h = RMSNorm(x) * g2;  x = x + (gelu_tanh(h Wi0) * (h Wi1)) Wo2
  y = RMSNorm(x) * g_final
  bucket: 32 relative-position buckets, 16 per direction; 8 exact (distance 0..7), 8 spaced
  logarithmically up to distance 128, larger distances share the last one; the bias table
  [32][heads] is shared by all layers.

Only tests and a benchmark's CPU-baseline leg may import this module.
"""
import numpy as np

F64 = np.float64
RMS_EPS = 1e-6
NUM_BUCKETS = 32
MAX_DISTANCE = 128


def param_shapes(arch):
    """{name: (shape, kind)} in a fixed order; matrices are [in, out]."""
    d, inner, dff = arch["d_model"], arch["n_heads"] * arch["head_dim"], arch["d_ff"]
    out = {"embed": ((arch["vocab"], d), "table"), "rel_bias": ((NUM_BUCKETS, arch["n_heads"]), "table")}
    for l in range(arch["n_layers"]):
        p = f"l{l}"
        out[p + ".ln1.g"] = ((d,), "gain")
        out[p + ".q.w"] = ((d, inner), "matrix")
        out[p + ".k.w"] = ((d, inner), "matrix")
        out[p + ".v.w"] = ((d, inner), "matrix")
        out[p + ".o.w"] = ((inner, d), "matrix")
        out[p + ".ln2.g"] = ((d,), "gain")
        out[p + ".wi0.w"] = ((d, dff), "matrix")
        out[p + ".wi1.w"] = ((d, dff), "matrix")
        out[p + ".wo.w"] = ((dff, d), "matrix")
    out["final.g"] = ((d,), "gain")
    return out


def relative_position_bucket(rel):
    """Bucket of rel = key position - query position (bidirectional form).

    Half of the 32 buckets serve keys after the query (offset 16), half keys at or before it.
    Inside a half: distances 0..7 have a bucket each; 8 <= n < 128 fall into bucket
    8 + floor(8 * ln(n/8) / ln(128/8)); n >= 128 into bucket 15.
    """
    rel = np.asarray(rel, dtype=np.int64)
    half = NUM_BUCKETS // 2                       # 16
    exact = half // 2                             # 8
    n = np.abs(rel)
    side = np.where(rel > 0, half, 0)
    # 8 + floor(8 ln(n/8) / ln 16) >= 8 + b  <=>  (n/8)^8 >= 16^b  <=>  n^8 >= 8^8 16^b : exact in
    # integers (n is clipped to 128 first, 128^8 = 2^56), so bucket edges do not depend on how a
    # floating-point logarithm rounds at n = 16, 32, 64.
    nc = np.minimum(n, MAX_DISTANCE).astype(np.int64)
    n8 = nc ** 8
    log_b = np.zeros_like(nc)
    for b in range(1, half - exact):
        log_b += (n8 >= (exact ** 8) * (16 ** b)).astype(np.int64)
    log_b = np.where(nc >= MAX_DISTANCE, half - 1, exact + log_b)
    return side + np.where(n < exact, n, log_b)


def position_bias(n, table):
    """bias[h][i][j] = table[bucket(j - i)][h] for a sequence of n tokens; table: [32][H]."""
    i = np.arange(n)[:, None]
    j = np.arange(n)[None, :]
    b = relative_position_bucket(j - i)              # [n][n]
    return np.transpose(np.asarray(table, F64)[b], (2, 0, 1))


def rms_norm(x, gain):
    return x / np.sqrt((x * x).mean(axis=-1, keepdims=True) + RMS_EPS) * gain


def gelu_tanh(x):
    return 0.5 * x * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (x + 0.044715 * x ** 3)))


def softmax_rows(s):
    m = s.max(axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / e.sum(axis=-1, keepdims=True)


class EncoderOracle:
    def __init__(self, arch, params):
        self.arch = arch
        self.p = {k: np.asarray(v, F64) for k, v in params.items()}

    def layer(self, x, l, bias, taps=None):
        a, p = self.arch, self.p
        H, dh = a["n_heads"], a["head_dim"]
        n = x.shape[0]
        pre = f"l{l}"
        h = rms_norm(x, p[pre + ".ln1.g"])
        q = (h @ p[pre + ".q.w"]).reshape(n, H, dh)
        k = (h @ p[pre + ".k.w"]).reshape(n, H, dh)
        v = (h @ p[pre + ".v.w"]).reshape(n, H, dh)
        o = np.empty((n, H, dh), F64)
        for hd in range(H):
            s = q[:, hd] @ k[:, hd].T + bias[hd]
            o[:, hd] = softmax_rows(s) @ v[:, hd]
        o = o.reshape(n, H * dh)
        x = x + o @ p[pre + ".o.w"]
        h2 = rms_norm(x, p[pre + ".ln2.g"])
        act = gelu_tanh(h2 @ p[pre + ".wi0.w"]) * (h2 @ p[pre + ".wi1.w"])
        y = x + act @ p[pre + ".wo.w"]
        if taps is not None:
            taps[pre + ".ln1"] = h; taps[pre + ".attn"] = o; taps[pre + ".x_attn"] = x
            taps[pre + ".act"] = act; taps[pre + ".x_out"] = y
        return y

    def forward(self, tokens, taps=None):
        """tokens: int array [n] -> condition [n][d_model]."""
        tokens = np.asarray(tokens, dtype=np.int64)
        x = self.p["embed"][tokens]
        bias = position_bias(len(tokens), self.p["rel_bias"])
        for l in range(self.arch["n_layers"]):
            x = self.layer(x, l, bias, taps)
        return rms_norm(x, self.p["final.g"])

"""Pins for the WIRING of the oracle's blocks: which modulation entry goes where, which slice
of a fused projection feeds which branch, where the gates and the affine norm sit.  Each test
builds weights (identities, zeros, selectors) for which the block collapses to a formula short
enough to evaluate by hand here with `math` / plain NumPy moments, or to an already pinned
elementary function (attention over equal scores = mean of V), so that a swapped index or a
dropped activation inside the block fails the test.  (The elementary functions themselves are
pinned in test_oracle_pins.py.)
"""
import math

import numpy as np

import synth
from oracle import dit_oracle as O


def small_arch(family="J", **kw):
    a = dict(family=family, n_blocks=1, n_single=0, hidden=32, n_heads=4, head_dim=8,
             mlp_hidden=64, latent_ch=2, patch=(1, 2, 2), cond_dim=12,
             rope_axes=(0, 0, 0), rope_theta=10000.0)
    if family == "F":
        a.update(n_blocks=0, n_single=1, rope_axes=(2, 4, 2))
    if family == "W":
        a.update(rope_axes=(4, 2, 2))
    a.update(kw)
    return a


def rand_params(arch, seed=7, std=0.3, bias_std=0.2, gain_std=0.2):
    p = synth.make_params(O.param_shapes(arch), seed, std, bias_std, gain_std)
    return {k: np.array(v, dtype=np.float64) for k, v in p.items()}


def rand_io(arch, f=1, h=4, w=6, n_cond=3, seed=5):
    lat = synth.gaussian(seed, "latent", arch["latent_ch"] * f * h * w).reshape(
        arch["latent_ch"], f, h, w).astype(np.float64)
    cond = synth.gaussian(seed + 1, "cond", n_cond * arch["cond_dim"]).reshape(
        n_cond, arch["cond_dim"]).astype(np.float64)
    return lat, cond


def _silu(x):
    return x / (1.0 + math.exp(-x))


def _gelu(x):
    return 0.5 * x * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * (x + 0.044715 * x ** 3)))


def _ln_rows(x):
    """LayerNorm of each row from the moments, written with Python sums."""
    out = np.empty_like(x)
    for r in range(x.shape[0]):
        row = [float(v) for v in x[r]]
        mu = sum(row) / len(row)
        var = sum((v - mu) ** 2 for v in row) / len(row)
        out[r] = [(v - mu) / math.sqrt(var + 1e-6) for v in row]
    return out


# ------------------------------------------------------------------------ conditioning
def test_conditioning_is_silu_of_the_two_layer_mlp_on_the_timestep_features():
    """With W1 = [I; 0] and W2 = I the conditioning vector is silu(silu(cos(tau f_k) + b1) + b2):
    the inner activation, the outer activation, both biases and the layer order are all visible
    (dropping the outer SiLU, or applying it before the second layer, changes the value)."""
    arch = small_arch("J")
    d = arch["hidden"]
    p = rand_params(arch)
    w1 = np.zeros((O.T_FREQ_DIM, d)); w1[:d, :d] = np.eye(d)
    p["t_embed.1.w"] = w1
    p["t_embed.2.w"] = np.eye(d)
    sigma = 0.3
    got = O.DiTOracle(arch, p).conditioning(sigma)
    b1, b2 = p["t_embed.1.b"], p["t_embed.2.b"]
    assert np.abs(b1).max() > 1e-2 and np.abs(b2).max() > 1e-2
    for k in range(d):
        f_k = math.exp(-math.log(10000.0) * k / 128.0)
        s = math.cos(1000.0 * sigma * f_k)             # first half of the feature vector: cosines
        want = _silu(_silu(s + b1[k]) + b2[k])
        assert abs(got[k] - want) < 1e-12, k
    # the sine half feeds through rows 128.. of W1
    w1 = np.zeros((O.T_FREQ_DIM, d)); w1[128:128 + d, :d] = np.eye(d)
    p["t_embed.1.w"] = w1
    got = O.DiTOracle(arch, p).conditioning(sigma)
    for k in range(d):
        f_k = math.exp(-math.log(10000.0) * k / 128.0)
        want = _silu(_silu(math.sin(1000.0 * sigma * f_k) + b1[k]) + b2[k])
        assert abs(got[k] - want) < 1e-12, k
    # a scaled second layer scales vec BEFORE the outer activation
    p["t_embed.2.w"] = 2.0 * np.eye(d)
    got2 = O.DiTOracle(arch, p).conditioning(sigma)
    for k in range(d):
        f_k = math.exp(-math.log(10000.0) * k / 128.0)
        want = _silu(2.0 * _silu(math.sin(1000.0 * sigma * f_k) + b1[k]) + b2[k])
        assert abs(got2[k] - want) < 1e-12, k


def test_velocity_feeds_the_conditioning_vector_to_the_blocks():
    """The vector the blocks modulate with is `conditioning(sigma)` itself (tap "m")."""
    arch = small_arch("J")
    p = rand_params(arch)
    m = O.DiTOracle(arch, p)
    lat, cond = rand_io(arch)
    taps = {}
    m.velocity(lat, cond, 0.7, taps)
    assert np.array_equal(taps["m"], m.conditioning(0.7))


# ------------------------------------------------------------------- joint block, MLP branch
def _joint_mods(p, m_vec, stream, d):
    mod = m_vec @ p[f"blk0.{stream}.mod.w"] + p[f"blk0.{stream}.mod.b"]
    return [mod[i * d:(i + 1) * d] for i in range(6)]


def test_joint_block_mlp_branch_uses_the_second_modulation_triple():
    """Entries 3, 4, 5 of the six-way modulation (shift2, scale2, gate2) act on the MLP branch
    and only there: doubling the gate2 columns doubles x_out - x_attn and leaves x_attn alone;
    changing shift2 or scale2 changes x_out but not x_attn; changing shift1, scale1 or gate1
    changes x_attn."""
    arch = small_arch("J")
    d = arch["hidden"]
    p = rand_params(arch)
    lat, cond = rand_io(arch)

    def run(params):
        t = {}
        O.DiTOracle(arch, params).velocity(lat, cond, 0.5, t)
        return t

    base = run(p)
    for s in ("img", "txt"):
        inc = base[f"blk0.{s}.x_out"] - base[f"blk0.{s}.x_attn"]
        assert np.abs(inc).max() > 1e-3

        def with_cols(lo, hi, factor=None, add=None):
            q = dict(p)
            w, b = p[f"blk0.{s}.mod.w"].copy(), p[f"blk0.{s}.mod.b"].copy()
            if factor is not None:
                w[:, lo:hi] *= factor; b[lo:hi] *= factor
            if add is not None:
                b[lo:hi] += add
            q[f"blk0.{s}.mod.w"], q[f"blk0.{s}.mod.b"] = w, b
            return run(q)

        t = with_cols(5 * d, 6 * d, factor=2.0)                       # gate2
        assert np.array_equal(t[f"blk0.{s}.x_attn"], base[f"blk0.{s}.x_attn"])
        assert np.allclose(t[f"blk0.{s}.x_out"] - t[f"blk0.{s}.x_attn"], 2 * inc, atol=1e-10)
        for lo in (3 * d, 4 * d):                                     # shift2, scale2
            t = with_cols(lo, lo + d, add=0.37)
            assert np.array_equal(t[f"blk0.{s}.x_attn"], base[f"blk0.{s}.x_attn"])
            assert np.abs(t[f"blk0.{s}.mlp_act"] - base[f"blk0.{s}.mlp_act"]).max() > 1e-3
        for lo in (0, d, 2 * d):                                      # shift1, scale1, gate1
            t = with_cols(lo, lo + d, add=0.37)
            assert np.abs(t[f"blk0.{s}.x_attn"] - base[f"blk0.{s}.x_attn"]).max() > 1e-4


def test_joint_block_mlp_branch_closed_form():
    """With mlp1 = [I | 0] (no bias) and mlp2 = [I; 0] (no bias) the branch is
    x_out = x_attn + gate2 * gelu(LN(x_attn) (1 + scale2) + shift2), evaluated here element by
    element from the row moments."""
    arch = small_arch("J")
    d, dff = arch["hidden"], arch["mlp_hidden"]
    p = rand_params(arch)
    for s in ("img", "txt"):
        w1 = np.zeros((d, dff)); w1[:, :d] = np.eye(d)
        w2 = np.zeros((dff, d)); w2[:d, :] = np.eye(d)
        p[f"blk0.{s}.mlp1.w"], p[f"blk0.{s}.mlp1.b"] = w1, np.zeros(dff)
        p[f"blk0.{s}.mlp2.w"], p[f"blk0.{s}.mlp2.b"] = w2, np.zeros(d)
    lat, cond = rand_io(arch)
    m = O.DiTOracle(arch, p)
    t = {}
    m.velocity(lat, cond, 0.5, t)
    for s in ("img", "txt"):
        _, _, _, sh2, sc2, g2 = _joint_mods(p, t["m"], s, d)
        xa = t[f"blk0.{s}.x_attn"]
        ln = _ln_rows(xa)
        want = np.empty_like(xa)
        for r in range(xa.shape[0]):
            for c in range(d):
                want[r, c] = xa[r, c] + g2[c] * _gelu(ln[r, c] * (1.0 + sc2[c]) + sh2[c])
        assert np.allclose(t[f"blk0.{s}.x_out"], want, atol=1e-10), s


def test_joint_block_attention_branch_closed_form():
    """With zero q/k projections (attention = mean of V over the joint sequence), v = the
    modulated input (qkv's V columns = I) and proj = I:
    x_attn = x + gate1 * (mean over [txt; img] rows of (LN(x) (1 + scale1) + shift1) + b_v + b_o),
    with each stream's own modulation in its own rows."""
    arch = small_arch("J")
    d = arch["hidden"]
    p = rand_params(arch)
    for s in ("img", "txt"):
        w = np.zeros((d, 3 * d)); w[:, 2 * d:] = np.eye(d)
        b = p[f"blk0.{s}.qkv.b"].copy(); b[:2 * d] = 0
        p[f"blk0.{s}.qkv.w"], p[f"blk0.{s}.qkv.b"] = w, b
        p[f"blk0.{s}.proj.w"] = np.eye(d)
    lat, cond = rand_io(arch)
    t = {}
    O.DiTOracle(arch, p).velocity(lat, cond, 0.5, t)
    v_rows = []
    for s, x0 in (("txt", t["x_txt0"]), ("img", t["x_img0"])):
        sh1, sc1 = _joint_mods(p, t["m"], s, d)[:2]
        v_rows.append(_ln_rows(x0) * (1.0 + sc1) + sh1 + p[f"blk0.{s}.qkv.b"][2 * d:])
    mean_v = np.concatenate(v_rows).mean(axis=0)
    for s, x0 in (("txt", t["x_txt0"]), ("img", t["x_img0"])):
        g1 = _joint_mods(p, t["m"], s, d)[2]
        want = x0 + g1 * (mean_v + p[f"blk0.{s}.proj.b"])
        assert np.allclose(t[f"blk0.{s}.x_attn"], want, atol=1e-10), s


# ----------------------------------------------------------------------- single-stream block
def _single_setup(select):
    """Family F with no double blocks and one single block whose attention is the mean of V
    (zero q/k columns), V = h (identity), u[:, :d] = h (identity); `select` picks which half of
    the concatenation [attention, GELU(u)] the second projection passes on."""
    arch = small_arch("F")
    d, dff = arch["hidden"], arch["mlp_hidden"]
    p = rand_params(arch)
    w1 = np.zeros((d, 3 * d + dff))
    w1[:, 2 * d:3 * d] = np.eye(d)            # v = h
    w1[:, 3 * d:4 * d] = np.eye(d)            # first d columns of u = h
    b1 = p["sgl0.lin1.b"].copy(); b1[:2 * d] = 0
    p["sgl0.lin1.w"], p["sgl0.lin1.b"] = w1, b1
    w2 = np.zeros((d + dff, d))
    if select == "attn":
        w2[:d] = np.eye(d)
    else:
        w2[d:2 * d] = np.eye(d)               # the first d columns of GELU(u)
    p["sgl0.lin2.w"] = w2
    return arch, p


def test_single_block_slices_and_concatenation():
    """x_out = x + g * ([attn, GELU(u)] W2 + b2) with [q, k, v, u] cut from one projection in
    that order: passing only the attention half must give x + g (mean(h + b_v) + b2), passing
    only the first d columns of the GELU half must give x + g (gelu(h + b_u) + b2) row by row.
    A GELU on the wrong slice, or the two halves swapped, fails one of the two."""
    for select in ("attn", "gelu"):
        arch, p = _single_setup(select)
        d = arch["hidden"]
        lat, cond = rand_io(arch)
        t = {}
        O.DiTOracle(arch, p).velocity(lat, cond, 0.5, t)
        x = np.concatenate([t["x_txt0"], t["x_img0"]])       # text rows first
        mod = t["m"] @ p["sgl0.mod.w"] + p["sgl0.mod.b"]
        sh, sc, g = mod[:d], mod[d:2 * d], mod[2 * d:]
        h = _ln_rows(x) * (1.0 + sc) + sh
        b1, b2 = p["sgl0.lin1.b"], p["sgl0.lin2.b"]
        if select == "attn":
            branch = np.tile((h + b1[2 * d:3 * d]).mean(axis=0), (x.shape[0], 1))
        else:
            branch = np.vectorize(_gelu)(h + b1[3 * d:4 * d])
        want = x + g * (branch + b2)
        assert np.allclose(t["sgl0.x_out"], want, atol=1e-10), select
        assert np.abs(t["sgl0.x_out"] - x).max() > 1e-3


# --------------------------------------------------------------------- family W cross-attention
def _w_case(**over):
    arch = small_arch("W")
    p = rand_params(arch)
    p.update(over)
    lat, cond = rand_io(arch, f=2, h=4, w=6, n_cond=5)
    return arch, p, lat, cond


def test_w_block_cross_attention_has_no_gate_and_no_modulation():
    """With a zero query projection every cross-attention score is 0, so each token receives
    mean_over_condition_tokens(c' W_v + b_v) W_xproj + b_xproj, the same for all rows, with no
    gate factor and independent of the timestep modulation."""
    arch, p, lat, cond = _w_case()
    d = arch["hidden"]
    p["blk0.xq.w"] = np.zeros((d, d)); p["blk0.xq.b"] = np.zeros(d)
    t = {}
    O.DiTOracle(arch, p).velocity(lat, cond, 0.5, t)
    cproj = cond @ p["c_embed.w"] + p["c_embed.b"]
    v = cproj @ p["blk0.xkv.w"][:, d:] + p["blk0.xkv.b"][d:]          # values are the SECOND half of xkv
    want = v.mean(axis=0) @ p["blk0.xproj.w"] + p["blk0.xproj.b"]
    inc = t["blk0.x_cross"] - t["blk0.x_attn"]
    assert np.allclose(inc, np.tile(want, (inc.shape[0], 1)), atol=1e-10)
    assert np.abs(want).max() > 1e-3
    # every modulation entry may change: the increment stays
    q = dict(p)
    q["blk0.mod_table"] = p["blk0.mod_table"] + 0.5
    q["t_proj.b"] = p["t_proj.b"] - 0.25
    t2 = {}
    O.DiTOracle(arch, q).velocity(lat, cond, 0.5, t2)
    assert np.allclose(t2["blk0.x_cross"] - t2["blk0.x_attn"], inc, atol=1e-10)
    assert np.abs(t2["blk0.x_attn"] - t["blk0.x_attn"]).max() > 1e-4      # ... while the gated branches move
    # and with q = 0 the norm's affine parameters cannot matter either
    q = dict(p)
    q["blk0.xnorm.g"] = p["blk0.xnorm.g"] * 3.0
    q["blk0.xnorm.b"] = p["blk0.xnorm.b"] + 1.0
    t3 = {}
    O.DiTOracle(arch, q).velocity(lat, cond, 0.5, t3)
    assert np.allclose(t3["blk0.x_cross"], t["blk0.x_cross"], atol=1e-10)


def test_w_block_cross_attention_pre_norm_is_layer_norm_with_affine():
    """gain 0 and a constant beta make the normalised input the same vector beta for every
    token, whatever x is: every row's query is then rms_norm_heads(beta W_q + b_q) and every row
    of the cross-attention output equals the (already pinned) attention of that one query over
    the condition's keys and values.  Without the affine, or with it applied before the
    normalisation, rows would differ."""
    arch, p, lat, cond = _w_case()
    d, H, dh = arch["hidden"], arch["n_heads"], arch["head_dim"]
    beta = synth.gaussian(31, "beta", d).astype(np.float64)
    p["blk0.xnorm.g"] = np.zeros(d)
    p["blk0.xnorm.b"] = beta
    t = {}
    O.DiTOracle(arch, p).velocity(lat, cond, 0.5, t)
    cproj = cond @ p["c_embed.w"] + p["c_embed.b"]
    kv = cproj @ p["blk0.xkv.w"] + p["blk0.xkv.b"]
    k, v = kv[:, :d], kv[:, d:]
    q = (beta @ p["blk0.xq.w"] + p["blk0.xq.b"]).reshape(1, H, dh)
    qn = (q / np.sqrt((q * q).mean(-1, keepdims=True) + 1e-6) * p["blk0.xqnorm.g"]).reshape(1, d)
    kh = k.reshape(-1, H, dh)
    kn = (kh / np.sqrt((kh * kh).mean(-1, keepdims=True) + 1e-6) * p["blk0.xknorm.g"]).reshape(-1, d)
    row = O.multi_head_attention(qn, kn, v, H)[0]
    assert np.allclose(t["blk0.xattn"], np.tile(row, (t["blk0.xattn"].shape[0], 1)), atol=1e-10)
    # sensitivity: a non-zero gain makes rows differ (the norm really sees x)
    p["blk0.xnorm.g"] = np.ones(d)
    t2 = {}
    O.DiTOracle(arch, p).velocity(lat, cond, 0.5, t2)
    assert np.abs(t2["blk0.xattn"] - t2["blk0.xattn"][0]).max() > 1e-4


def test_w_block_modulation_is_table_plus_projected_timestep_in_six_rows():
    """e = table + reshape(m W_tp + b_tp, [6, d]) with rows (shift1, scale1, gate1, shift2,
    scale2, gate2): zeroing row 2 of the sum switches the self-attention branch off (x_attn =
    x_in), zeroing row 5 switches the MLP branch off (x_out = x_cross), and the other rows do
    neither."""
    arch, p, lat, cond = _w_case()
    d = arch["hidden"]
    m = O.DiTOracle(arch, p)
    base = (m.conditioning(0.5) @ p["t_proj.w"] + p["t_proj.b"]).reshape(6, d)
    for row, (a, b) in ((2, ("x_img0", "blk0.x_attn")), (5, ("blk0.x_cross", "blk0.x_out"))):
        q = dict(p)
        tab = p["blk0.mod_table"].copy()
        tab[row] = -base[row]
        q["blk0.mod_table"] = tab
        t = {}
        O.DiTOracle(arch, q).velocity(lat, cond, 0.5, t)
        assert np.allclose(t[b], t[a], atol=1e-12), row
        other = ("blk0.x_cross", "blk0.x_out") if row == 2 else ("x_img0", "blk0.x_attn")
        assert np.abs(t[other[1]] - t[other[0]]).max() > 1e-4


def test_w_block_cross_attention_ignores_the_timestep_modulation():
    """With a live query path: shift2/scale2/gate2 (rows 3-5) act only after the cross-attention,
    so changing them leaves its output bit-identical; with the self-attention gate (row 2) held
    at zero the block input reaches the cross-attention untouched, and then shift1/scale1 (rows
    0, 1) cannot change its output either."""
    arch, p, lat, cond = _w_case()
    d = arch["hidden"]
    base = (O.DiTOracle(arch, p).conditioning(0.5) @ p["t_proj.w"] + p["t_proj.b"]).reshape(6, d)

    def run(tab):
        q = dict(p); q["blk0.mod_table"] = tab
        t = {}
        O.DiTOracle(arch, q).velocity(lat, cond, 0.5, t)
        return t

    t0 = run(p["blk0.mod_table"])
    tab = p["blk0.mod_table"].copy(); tab[3:6] += 0.4
    t1 = run(tab)
    assert np.array_equal(t1["blk0.xattn"], t0["blk0.xattn"]) and np.array_equal(t1["blk0.x_cross"], t0["blk0.x_cross"])
    assert np.abs(t1["blk0.x_out"] - t0["blk0.x_out"]).max() > 1e-4
    tab = p["blk0.mod_table"].copy(); tab[2] = -base[2]
    t2 = run(tab)
    tab2 = tab.copy(); tab2[0:2] += 0.4
    t3 = run(tab2)
    assert np.allclose(t2["blk0.x_attn"], t2["x_img0"], atol=1e-12)
    assert np.allclose(t3["blk0.xattn"], t2["blk0.xattn"], atol=1e-12)
    assert np.abs(t2["blk0.xattn"] - t2["blk0.xattn"][0]).max() > 1e-4       # the query path is live

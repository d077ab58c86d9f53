"""Pins for the CPU oracle: closed forms, invariants, brute force on tiny inputs and
special cases that reduce to a textbook definition.  None of these retype the oracle's
own formula; each is chosen so that a plausible slip (dropped term, wrong sign or index,
transposed operand) makes it fail.  The paper prints no worked numbers for the Diffuse
stage (section 2.1 has only the two-term update equation), so there are no paper values
to pin to.
"""
import math

import numpy as np
import pytest

import synth
from oracle import dit_oracle as O

RNG = np.random.default_rng(1234)


def small_arch(family="J", **kw):
    a = dict(family=family, n_blocks=2, n_single=0, hidden=32, n_heads=4, head_dim=8,
             mlp_hidden=64, latent_ch=2, patch=(1, 2, 2), cond_dim=12,
             rope_axes=(0, 0, 0), rope_theta=10000.0)
    if family == "F":
        a.update(n_single=2, rope_axes=(2, 4, 2))
    if family == "W":
        a.update(rope_axes=(4, 2, 2))
    a.update(kw)
    return a


def rand_params(arch, seed=7, std=0.3, bias_std=0.2, gain_std=0.2):
    return synth.make_params(O.param_shapes(arch), seed, std, bias_std, gain_std)


def rand_io(arch, f=1, h=4, w=6, n_cond=3, seed=5):
    lat = synth.gaussian(seed, "latent", arch["latent_ch"] * f * h * w).reshape(
        arch["latent_ch"], f, h, w).astype(np.float64)
    cond = synth.gaussian(seed + 1, "cond", n_cond * arch["cond_dim"]).reshape(
        n_cond, arch["cond_dim"]).astype(np.float64)
    return lat, cond


# ---------------------------------------------------------------------------- softmax
def test_softmax_rows_sum_to_one_and_shift_invariant():
    s = RNG.normal(size=(7, 33)) * 10
    p = O.softmax_rows(s)
    assert np.allclose(p.sum(-1), 1.0, atol=1e-12)
    assert (p >= 0).all()
    assert np.allclose(O.softmax_rows(s + 123.456), p, atol=1e-12)
    # huge logits must not overflow (needs the max subtraction)
    assert np.isfinite(O.softmax_rows(s + 1e4)).all()


def test_softmax_matches_online_tiled_evaluation():
    """The tiled running-max/running-sum recurrence gives the same attention output."""
    n, dh = 37, 8
    q, k, v = (RNG.normal(size=(n, dh)) for _ in range(3))
    ref = O.attention(q, k, v)
    for tile in (1, 5, 16, 64):
        m = np.full(n, -np.inf)
        l = np.zeros(n)
        acc = np.zeros((n, dh))
        for lo in range(0, n, tile):
            s = q @ k[lo:lo + tile].T / math.sqrt(dh)
            m_new = np.maximum(m, s.max(-1))
            p = np.exp(s - m_new[:, None])
            corr = np.exp(m - m_new)
            l = l * corr + p.sum(-1)
            acc = acc * corr[:, None] + p @ v[lo:lo + tile]
            m = m_new
        assert np.allclose(acc / l[:, None], ref, atol=1e-12)


# -------------------------------------------------------------------------- attention
def test_attention_identical_keys_gives_mean_of_v():
    n, dh = 9, 8
    k = np.tile(RNG.normal(size=(1, dh)), (n, 1))
    q, v = RNG.normal(size=(5, dh)), RNG.normal(size=(n, dh))
    assert np.allclose(O.attention(q, k, v), np.tile(v.mean(0), (5, 1)), atol=1e-12)


def test_attention_single_key_returns_that_row():
    q, k, v = RNG.normal(size=(4, 8)), RNG.normal(size=(1, 8)), RNG.normal(size=(1, 8))
    assert np.allclose(O.attention(q, k, v), np.tile(v, (4, 1)), atol=1e-14)


def test_attention_brute_force_python_loops():
    nq, nk, dh = 5, 7, 4
    q, k, v = RNG.normal(size=(nq, dh)), RNG.normal(size=(nk, dh)), RNG.normal(size=(nk, dh))
    out = O.attention(q, k, v)
    for i in range(nq):
        logits = [sum(q[i, c] * k[j, c] for c in range(dh)) / math.sqrt(dh) for j in range(nk)]
        z = sum(math.exp(x) for x in logits)
        for c in range(dh):
            want = sum(math.exp(logits[j]) / z * v[j, c] for j in range(nk))
            assert abs(out[i, c] - want) < 1e-12


def test_attention_one_hot_limit_selects_matching_value():
    """Keys orthogonal and sharply scaled: each query retrieves the value of its own key."""
    dh = 8
    k = np.eye(dh) * 200.0
    v = RNG.normal(size=(dh, dh))
    q = np.eye(dh)[[3, 0, 6]] * 1.0
    assert np.allclose(O.attention(q, k, v), v[[3, 0, 6]], atol=1e-10)


def test_multi_head_attention_heads_do_not_mix():
    n, H, dh = 6, 3, 4
    q, k, v = (RNG.normal(size=(n, H * dh)) for _ in range(3))
    base = O.multi_head_attention(q, k, v, H)
    v2 = v.copy()
    v2[:, dh:2 * dh] += 1.0  # only head 1 changes, and softmax rows sum to 1 -> +1 there
    out = O.multi_head_attention(q, k, v2, H)
    assert np.array_equal(out[:, :dh], base[:, :dh])
    assert np.array_equal(out[:, 2 * dh:], base[:, 2 * dh:])
    assert np.allclose(out[:, dh:2 * dh], base[:, dh:2 * dh] + 1.0, atol=1e-12)


# ------------------------------------------------------------------------------ norms
def test_layer_norm_moments_and_scale_invariance():
    x = RNG.normal(size=(5, 64)) * 3 + 2
    y = O.layer_norm(x)
    assert np.allclose(y.mean(-1), 0, atol=1e-12)
    assert np.allclose(y.var(-1), 1, atol=1e-5)
    assert np.allclose(O.layer_norm(7.5 * x), y, atol=1e-6)
    assert np.allclose(O.layer_norm(x + 11.0), y, atol=1e-9)
    # textbook case: [1, 3] has mean 2 and variance 1
    assert np.allclose(O.layer_norm(np.array([[1.0, 3.0]])), [[-1.0, 1.0]], atol=1e-6)


def test_rms_norm_unit_rms_and_gain():
    x = RNG.normal(size=(5, 16)) * 4
    y = O.rms_norm(x, np.ones(16))
    assert np.allclose(np.sqrt((y * y).mean(-1)), 1, atol=1e-6)
    g = RNG.normal(size=16)
    assert np.allclose(O.rms_norm(x, g), y * g, atol=1e-12)
    # no mean subtraction: [3, 4] -> rms = sqrt(12.5)
    assert np.allclose(O.rms_norm(np.array([[3.0, 4.0]]), np.ones(2)),
                       np.array([[3.0, 4.0]]) / math.sqrt(12.5), atol=1e-6)


def test_modulate_zero_is_layer_norm_and_affine_in_shift_scale():
    x = RNG.normal(size=(4, 32))
    z = np.zeros(32)
    assert np.array_equal(O.modulate(x, z, z), O.layer_norm(x))
    sh, sc = RNG.normal(size=32), RNG.normal(size=32)
    assert np.allclose(O.modulate(x, sh, sc) - O.modulate(x, z, sc), np.tile(sh, (4, 1)), atol=1e-12)
    assert np.allclose(O.modulate(x, z, np.ones(32)), 2 * O.layer_norm(x), atol=1e-12)


# --------------------------------------------------------------------- activations
def test_gelu_tanh_against_erf_form_and_symmetry():
    x = np.linspace(-6, 6, 241)
    exact = np.array([0.5 * t * (1 + math.erf(t / math.sqrt(2))) for t in x])
    assert np.max(np.abs(O.gelu_tanh(x) - exact)) < 1e-3
    assert np.allclose(O.gelu_tanh(x) - O.gelu_tanh(-x), x, atol=1e-12)
    assert O.gelu_tanh(np.array([0.0]))[0] == 0.0
    assert abs(O.gelu_tanh(np.array([10.0]))[0] - 10.0) < 1e-9


def test_silu_closed_forms():
    x = np.linspace(-8, 8, 33)
    assert np.allclose(O.silu(x) - O.silu(-x), x, atol=1e-12)
    assert O.silu(np.array([0.0]))[0] == 0.0
    assert abs(O.silu(np.array([math.log(3.0)]))[0] - math.log(3.0) * 0.75) < 1e-12


# ------------------------------------------------------------------------ embeddings
def test_timestep_features_known_values():
    s = O.timestep_features(0.0)
    assert np.array_equal(s[:128], np.ones(128)) and np.array_equal(s[128:], np.zeros(128))
    s = O.timestep_features(0.0005)  # tau = 0.5
    assert abs(s[0] - math.cos(0.5)) < 1e-12 and abs(s[128] - math.sin(0.5)) < 1e-12
    # frequency k = 64 is 1e4^(-1/2) = 0.01
    s = O.timestep_features(0.1)  # tau = 100 -> angle 1.0 at k = 64
    assert abs(s[64] - math.cos(1.0)) < 1e-9 and abs(s[128 + 64] - math.sin(1.0)) < 1e-9
    assert np.allclose(s[:128] ** 2 + s[128:] ** 2, 1.0, atol=1e-12)


def test_sincos_pe_layout():
    d, gh, gw = 16, 3, 5
    pe = O.sincos_pe(gh, gw, d)
    assert pe.shape == (gh * gw, d)
    assert np.allclose(pe[0], [0, 0, 0, 0, 1, 1, 1, 1, 0, 0, 0, 0, 1, 1, 1, 1])
    for i in range(gh):
        for j in range(gw):
            row = pe[i * gw + j]
            for k in range(4):
                w = 10000.0 ** (-k / 4)
                want = [math.sin(i * w), math.cos(i * w), math.sin(j * w), math.cos(j * w)]
                got = [row[k], row[4 + k], row[8 + k], row[12 + k]]
                assert np.allclose(got, want, atol=1e-12)


def test_patchify_indexing_and_round_trip():
    c, f, h, w = 3, 4, 6, 8
    patch = (2, 2, 2)
    x = RNG.normal(size=(c, f, h, w))
    p = O.patchify(x, patch)
    gf, gh, gw = f // 2, h // 2, w // 2
    assert p.shape == (gf * gh * gw, c * 8)
    for _ in range(200):
        ci, fi, hi, wi = (int(RNG.integers(n)) for n in (c, f, h, w))
        tok = ((fi // 2) * gh + hi // 2) * gw + wi // 2
        feat = ((ci * 2 + fi % 2) * 2 + hi % 2) * 2 + wi % 2
        assert p[tok, feat] == x[ci, fi, hi, wi]
    assert np.array_equal(O.unpatchify(p, x.shape, patch), x)


# ------------------------------------------------------------------------------- RoPE
def test_rope_properties():
    n, H, dh = 6, 2, 8
    axes, theta = (4, 2, 2), 10000.0
    x = RNG.normal(size=(n, H, dh))
    pos = RNG.integers(0, 20, size=(n, 3)).astype(float)
    y = O.rope(x, pos, axes, theta)
    assert np.allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), atol=1e-12)
    assert np.array_equal(O.rope(x, np.zeros((n, 3)), axes, theta), x)
    # relative-position property per axis
    q, k = RNG.normal(size=(1, 1, dh)), RNG.normal(size=(1, 1, dh))
    def dot(pq, pk):
        return float((O.rope(q, np.array([pq], float), axes, theta)
                      * O.rope(k, np.array([pk], float), axes, theta)).sum())
    assert abs(dot([3, 5, 7], [1, 2, 3]) - dot([12, 13, 14], [10, 10, 10])) < 1e-10
    assert abs(dot([3, 5, 7], [1, 2, 3]) - dot([3, 5, 8], [1, 2, 3])) > 1e-6


def test_rope_hand_computed_angles():
    """Chunk widths (4, 2, 2): pairs (0,1),(2,3) turn with the frame position at rates
    1 and theta^(-1/2); pair (4,5) with the row; pair (6,7) with the column, rate 1."""
    theta = 10000.0
    x = np.zeros((1, 1, 8))
    x[0, 0, [0, 2, 4, 6]] = 1.0
    y = O.rope(x, np.array([[2.0, 3.0, 0.5]]), (4, 2, 2), theta)[0, 0]
    want = [math.cos(2.0), math.sin(2.0), math.cos(2.0 * 0.01), math.sin(2.0 * 0.01),
            math.cos(3.0), math.sin(3.0), math.cos(0.5), math.sin(0.5)]
    assert np.allclose(y, want, atol=1e-12)
    # quarter turn sends (0, 1) to (-1, 0): fixes the sign convention
    x = np.zeros((1, 1, 2)); x[0, 0, 1] = 1.0
    y = O.rope(x, np.array([[math.pi / 2, 0, 0]]), (2, 0, 0), theta)[0, 0]
    assert np.allclose(y, [-1.0, 0.0], atol=1e-12)


# ----------------------------------------------------------------------------- linear
def test_linear_identity_and_triple_loop():
    arch = small_arch()
    p = rand_params(arch)
    d = arch["hidden"]
    p["t_embed.2.w"] = np.eye(d)
    m = O.DiTOracle(arch, p)
    x = RNG.normal(size=(3, d))
    assert np.allclose(m._lin(x, "t_embed.2"), x + p["t_embed.2.b"], atol=1e-12)
    # non-square: y[i, o] = sum_k x[i, k] W[k, o] + b[o]
    w, b = np.asarray(p["blk0.img.mlp1.w"], float), np.asarray(p["blk0.img.mlp1.b"], float)
    y = m._lin(x, "blk0.img.mlp1")
    for i in range(3):
        for o in (0, 5, 63):
            assert abs(y[i, o] - (sum(x[i, k] * w[k, o] for k in range(d)) + b[o])) < 1e-10


# ------------------------------------------------------------------- update / sampler
def test_update_coefficients_closed_forms():
    assert O.update_coefficients(0, 0.75, 0.5) == (1.0, -0.25)
    a, b = O.update_coefficients(1, 0.6, 0.0)  # abar: 0.64 -> 1
    assert abs(a - 1 / 0.8) < 1e-12 and abs(b - (0.0 - 0.6 / 0.8)) < 1e-12
    # DDIM moves a sample x = sqrt(abar) x0 + sigma eps exactly along the line when eps is exact
    x0, eps = RNG.normal(size=5), RNG.normal(size=5)
    sc, sn = 0.9, 0.4
    xc = math.sqrt(1 - sc * sc) * x0 + sc * eps
    a, b = O.update_coefficients(1, sc, sn)
    assert np.allclose(a * xc + b * eps, math.sqrt(1 - sn * sn) * x0 + sn * eps, atol=1e-12)
    # Euler is exact for the straight flow x = (1-s) x0 + s eps with velocity eps - x0
    xc = (1 - sc) * x0 + sc * eps
    a, b = O.update_coefficients(0, sc, sn)
    assert np.allclose(a * xc + b * (eps - x0), (1 - sn) * x0 + sn * eps, atol=1e-12)
    with pytest.raises(ValueError):
        O.update_coefficients(1, 1.0, 0.5)


@pytest.mark.parametrize("family", ["J", "F", "W"])
def test_zero_weights_give_zero_velocity_and_closed_form_sampler(family):
    arch = small_arch(family)
    p = {k: np.zeros_like(v) for k, v in rand_params(arch).items()}
    m = O.DiTOracle(arch, p)
    lat, cond = rand_io(arch)
    assert np.array_equal(m.velocity(lat, cond, 0.7), np.zeros_like(lat))
    sig = synth.default_sigmas(5, 2.0)
    assert np.array_equal(m.sample(lat, cond, sig, kind=0), lat)
    sig_d = sig * 0.9
    want = lat * math.sqrt((1 - sig_d[-1] ** 2) / (1 - sig_d[0] ** 2))
    assert np.allclose(m.sample(lat, cond, sig_d, kind=1), want, atol=1e-12)


@pytest.mark.parametrize("family", ["J", "F", "W"])
def test_zero_weights_with_output_bias_shift_by_constant(family):
    """x = 0 => LN(x) = 0 => the final layer emits its bias; Euler from sigma 1 to 0 then
    moves the latent by exactly -unpatchify(b_out) whatever T and the schedule shift."""
    arch = small_arch(family)
    p = {k: np.zeros_like(v) for k, v in rand_params(arch).items()}
    p["final.b"] = RNG.normal(size=p["final.b"].shape)
    m = O.DiTOracle(arch, p)
    lat, cond = rand_io(arch)
    gh, gw = lat.shape[2] // 2, lat.shape[3] // 2
    vconst = O.unpatchify(np.tile(p["final.b"], (gh * gw, 1)), lat.shape, arch["patch"])
    if family == "J":
        # the position code makes x nonzero; switch it off through a zero embed: x = PE,
        # so use the F/W families for the strict constant, and only check finiteness here
        assert np.isfinite(m.velocity(lat, cond, 0.3)).all()
        return
    assert np.allclose(m.velocity(lat, cond, 0.3), vconst, atol=1e-12)
    for T, shift in ((3, 1.0), (7, 3.0)):
        out = m.sample(lat, cond, synth.default_sigmas(T, shift), kind=0)
        assert np.allclose(out, lat - vconst, atol=1e-12)


@pytest.mark.parametrize("family", ["J", "F", "W"])
def test_zero_gates_reduce_to_final_layer_on_embedded_input(family):
    """With every modulation matrix and table zero all gates vanish, so the blocks are the
    identity (family W keeps its ungated cross-attention, so its projection is zeroed too)
    and the output is the final layer applied to the embedded latent."""
    arch = small_arch(family)
    p = rand_params(arch)
    for k in p:
        if ".mod." in k or "mod_table" in k or k.startswith("t_proj") or ".xproj." in k:
            p[k] = np.zeros_like(p[k])
    m = O.DiTOracle(arch, p)
    lat, cond = rand_io(arch)
    tok = O.patchify(lat, arch["patch"]) @ p["x_embed.w"].astype(float) + p["x_embed.b"]
    if family == "J":
        tok = tok + O.sincos_pe(lat.shape[2] // 2, lat.shape[3] // 2, arch["hidden"])
    mu = tok.mean(-1, keepdims=True)
    ln = (tok - mu) / np.sqrt(tok.var(-1, keepdims=True) + 1e-6)
    y = ln @ p["final.w"].astype(float) + p["final.b"]
    want = O.unpatchify(y, lat.shape, arch["patch"])
    assert np.allclose(m.velocity(lat, cond, 0.4), want, atol=1e-10)


def test_sample_equals_repeated_steps():
    arch = small_arch("J")
    m = O.DiTOracle(arch, rand_params(arch))
    lat, cond = rand_io(arch)
    sig = synth.default_sigmas(3, 1.5)
    x = lat
    for j in range(3):
        x, _ = m.step(x, cond, sig[j], sig[j + 1])
    assert np.array_equal(m.sample(lat, cond, sig), x)


# ------------------------------------------------------------------- model structure
@pytest.mark.parametrize("family", ["J", "F", "W"])
def test_condition_and_timestep_influence_output(family):
    arch = small_arch(family)
    m = O.DiTOracle(arch, rand_params(arch))
    lat, cond = rand_io(arch)
    v = m.velocity(lat, cond, 0.5)
    assert np.isfinite(v).all() and np.abs(v).max() > 1e-3
    c2 = cond.copy(); c2[1, 3] += 0.5
    assert np.abs(m.velocity(lat, c2, 0.5) - v).max() > 1e-6
    assert np.abs(m.velocity(lat, cond, 0.6) - v).max() > 1e-6


def test_permutation_equivariance_without_position_code():
    """Family F with all rotary widths zero has no position information: permuting image
    tokens permutes the output tokens the same way."""
    arch = small_arch("F", rope_axes=(0, 0, 0))
    m = O.DiTOracle(arch, rand_params(arch))
    lat, cond = rand_io(arch)
    tok = O.patchify(lat, arch["patch"])
    perm = RNG.permutation(tok.shape[0])
    lat2 = O.unpatchify(tok[perm], lat.shape, arch["patch"])
    v1 = O.patchify(m.velocity(lat, cond, 0.5), arch["patch"])
    v2 = O.patchify(m.velocity(lat2, cond, 0.5), arch["patch"])
    assert np.allclose(v2, v1[perm], atol=1e-10)
    # and with the rotary code switched on the same permutation must NOT commute
    arch_r = small_arch("F")
    mr = O.DiTOracle(arch_r, rand_params(arch_r))
    w1 = O.patchify(mr.velocity(lat, cond, 0.5), arch["patch"])
    w2 = O.patchify(mr.velocity(lat2, cond, 0.5), arch["patch"])
    assert np.abs(w2 - w1[perm]).max() > 1e-6


def test_joint_attention_runs_over_text_and_image_tokens():
    """With the q and k projections zero all scores are equal, so every token's attention
    output is the mean of V over the whole [text; image] sequence of the request."""
    arch = small_arch("J", n_blocks=1)
    p = rand_params(arch)
    d = arch["hidden"]
    for s in ("txt", "img"):
        p[f"blk0.{s}.qkv.w"] = p[f"blk0.{s}.qkv.w"].copy()
        p[f"blk0.{s}.qkv.b"] = p[f"blk0.{s}.qkv.b"].copy()
        p[f"blk0.{s}.qkv.w"][:, :2 * d] = 0
        p[f"blk0.{s}.qkv.b"][:2 * d] = 0
    m = O.DiTOracle(arch, p)
    lat, cond = rand_io(arch)
    taps = {}
    m.velocity(lat, cond, 0.5, taps)
    n = cond.shape[0] + (lat.shape[2] // 2) * (lat.shape[3] // 2)
    assert taps["blk0.v"].shape == (n, d)
    assert np.allclose(taps["blk0.attn"], np.tile(taps["blk0.v"].mean(0), (n, 1)), atol=1e-12)
    # text rows come first in the joint sequence
    h_txt = taps["blk0.txt.qkv"][:, 2 * d:]
    assert np.array_equal(taps["blk0.v"][:cond.shape[0]], h_txt)


def test_qk_norm_gives_unit_rms_heads():
    arch = small_arch("J", n_blocks=1)
    p = rand_params(arch, gain_std=0.0)
    m = O.DiTOracle(arch, p)
    lat, cond = rand_io(arch)
    taps = {}
    m.velocity(lat, cond, 0.5, taps)
    for name in ("blk0.q", "blk0.k"):
        t = taps[name].reshape(-1, arch["n_heads"], arch["head_dim"])
        assert np.allclose(np.sqrt((t * t).mean(-1)), 1.0, atol=1e-4)


def test_gate_scales_branch_linearly():
    """x_out - x_in of the attention branch is linear in the gate g1: doubling the gate
    columns of the modulation matrix doubles the residual increment."""
    arch = small_arch("J", n_blocks=1)
    p = rand_params(arch)
    d = arch["hidden"]
    lat, cond = rand_io(arch)
    t1, t2 = {}, {}
    O.DiTOracle(arch, p).velocity(lat, cond, 0.5, t1)
    p2 = dict(p)
    w, b = p["blk0.img.mod.w"].copy(), p["blk0.img.mod.b"].copy()
    w[:, 2 * d:3 * d] *= 2
    b[2 * d:3 * d] *= 2
    p2["blk0.img.mod.w"], p2["blk0.img.mod.b"] = w, b
    O.DiTOracle(arch, p2).velocity(lat, cond, 0.5, t2)
    inc1 = t1["blk0.img.x_attn"] - t1["x_img0"]
    inc2 = t2["blk0.img.x_attn"] - t2["x_img0"]
    assert np.allclose(inc2, 2 * inc1, atol=1e-10)
    assert np.abs(inc1).max() > 1e-3


def test_parameter_counts_match_model_classes():
    """2 B-class, 12 B-class and 13 B-class diffusion transformers (the paper's pipeline
    table lists Sd3-DiT 2 B, Flux-DiT 12 B, HYV-DiT 13 B)."""
    def count(name):
        return sum(int(np.prod(s)) for s, _ in O.param_shapes(synth.CONFIGS[name]["arch"]).values())
    assert abs(count("sd3") / 2.04e9 - 1) < 0.02
    assert abs(count("flux") / 1.18e10 - 1) < 0.02
    assert abs(count("wan") / 1.42e10 - 1) < 0.02
    assert abs(count("tiny") / 4.9e6 - 1) < 0.1


# --------------------------------------------------------------------------- generator
def test_generator_is_counter_based_and_gaussian():
    a = synth.gaussian(3, "w", 1000)
    b = synth.gaussian(3, "w", 400, start=600)
    assert np.array_equal(a[600:], b)
    assert not np.array_equal(a, synth.gaussian(4, "w", 1000))
    assert not np.array_equal(a, synth.gaussian(3, "v", 1000))
    g = synth.gaussian(11, "big", 400000).astype(np.float64)
    assert abs(g.mean()) < 0.01 and abs(g.std() - 1) < 0.01
    assert abs((g ** 4).mean() - 3.0) < 0.1  # Gaussian kurtosis
    assert synth.fnv1a64("a") == 0xAF63DC4C8601EC8C  # published FNV-1a test vector


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -8 + 2 ** -20, -2.5],
                 np.float32)
    want = np.array([1.0, 1.0, 1.0 + 2 ** -6, 1.0 + 2 ** -7, -2.5], np.float32)
    assert np.array_equal(synth.round_bf16(x), want)


def test_tiny_config_regression_file():
    """The stored samples were written by tests/golden/make_golden.py from the oracle alone;
    this guards the oracle (and the generators) against silent change."""
    import importlib.util
    import os
    here = os.path.dirname(os.path.abspath(__file__))
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(here, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    idx, v0, x0 = mod.compute()
    tab = np.loadtxt(os.path.join(here, "golden", "tiny_oracle.txt"))
    assert np.array_equal(tab[:, 0].astype(int), idx)
    assert np.allclose(tab[:, 1], v0, rtol=0, atol=1e-12)
    assert np.allclose(tab[:, 2], x0, rtol=0, atol=1e-12)


def test_row_sampled_last_block_equals_full_evaluation():
    """The row-restricted evaluation of the last block is the full evaluation on those rows."""
    arch = small_arch("W", n_blocks=2)
    m = O.DiTOracle(arch, rand_params(arch))
    lat, cond = rand_io(arch, f=2, h=4, w=6)
    taps = {}
    m.velocity(lat, cond, 0.5, taps)
    rows = np.array([0, 3, 7, 11])
    assert np.allclose(m.final_rows_w(lat, cond, 0.5, rows), taps["final"][rows], atol=1e-12)

"""Pins of the Encode-stage oracle (T5-v1.1-style encoder) against hand-derived values,
closed forms and invariants."""
import os

import numpy as np
import pytest

import synth
from oracle import encoder_oracle as E

HERE = os.path.dirname(os.path.abspath(__file__))
ARCH = synth.ENCODERS["t5_tiny"]


def _params(arch=ARCH, seed=1, std=0.05, gain_std=0.1):
    return synth.make_params(E.param_shapes(arch), seed, std, 0.0, gain_std)


def test_bucket_edges_match_the_hand_derived_table():
    rows = [tuple(map(int, l.split())) for l in open(os.path.join(HERE, "golden", "t5_bucket_edges.txt")) if l[0] != "#"]
    assert [b for b, _ in rows] == list(range(8, 16))
    for (b, first), nxt in zip(rows, [r[1] for r in rows[1:]] + [10 ** 6]):
        for n in (first, nxt - 1 if nxt < 10 ** 6 else 5000):
            assert E.relative_position_bucket(-n) == b            # key before the query
            assert E.relative_position_bucket(n) == 16 + b        # key after the query
        if first > 8:
            assert E.relative_position_bucket(-(first - 1)) == b - 1


def test_bucket_exact_range_symmetry_and_monotonicity():
    for n in range(8):
        assert E.relative_position_bucket(-n) == n
        assert E.relative_position_bucket(n) == (16 + n if n else 0)
    r = np.arange(1, 400)
    after, before = E.relative_position_bucket(r), E.relative_position_bucket(-r)
    assert np.array_equal(after, before + 16)
    assert np.all(np.diff(before) >= 0) and before.max() == 15 and np.all(before[127:] == 15)
    # away from the edges the floating-point form of the published rule agrees
    for n in (9, 10, 14, 20, 28, 40, 55, 80, 110):
        assert E.relative_position_bucket(-n) == 8 + int(np.floor(8 * np.log(n / 8) / np.log(16)))


def test_position_bias_is_a_toeplitz_lookup():
    table = np.arange(32 * 3, dtype=float).reshape(32, 3)
    b = E.position_bias(6, table)
    assert b.shape == (3, 6, 6)
    for h in range(3):
        for i in range(6):
            for j in range(6):
                assert b[h, i, j] == table[E.relative_position_bucket(j - i), h]
    assert b[1, 2, 2] == table[0, 1] and b[1, 2, 5] == table[19, 1] and b[1, 5, 2] == table[3, 1]


def test_rms_norm_has_no_mean_subtraction():
    x = np.full((2, 8), 3.0)
    assert np.allclose(E.rms_norm(x, np.ones(8)), 1.0, atol=1e-6)             # LayerNorm would give 0
    x = np.array([[3.0, -4.0]])
    assert np.allclose(E.rms_norm(x, np.array([2.0, 1.0])), [[2 * 3 / np.sqrt(12.5), -4 / np.sqrt(12.5)]], atol=1e-6)


def test_gelu_matches_erf_form_loosely_and_identities():
    from math import erf
    x = np.linspace(-4, 4, 41)
    ref = np.array([0.5 * v * (1 + erf(v / np.sqrt(2))) for v in x])
    assert np.abs(E.gelu_tanh(x) - ref).max() < 3e-3
    assert np.allclose(E.gelu_tanh(x) - E.gelu_tanh(-x), x)                    # gelu(x) - gelu(-x) = x


def test_zero_weights_give_the_normalised_embedding():
    p = _params()
    for k in p:
        if k.endswith(".w"):
            p[k] = np.zeros_like(p[k])
    tok = synth.make_tokens([9], ARCH["vocab"])[0]
    y = E.EncoderOracle(ARCH, p).forward(tok)
    x = p["embed"][tok].astype(np.float64)
    want = x / np.sqrt((x * x).mean(-1, keepdims=True) + 1e-6) * p["final.g"]
    assert np.allclose(y, want, atol=1e-12)


def test_single_token_attention_returns_its_value_and_scores_are_unscaled():
    p = _params()
    tok = np.array([5])
    taps = {}
    E.EncoderOracle(ARCH, p).forward(tok, taps)
    h = taps["l0.ln1"].astype(np.float64)
    assert np.allclose(taps["l0.attn"], h @ p["l0.v.w"].astype(np.float64), atol=1e-12)
    # two tokens, one head: probabilities follow exp(q.k + bias) with NO 1/sqrt(d) factor
    arch = dict(ARCH, n_heads=1, n_layers=1)
    p = _params(arch, std=0.2)
    tok = np.array([3, 8])
    taps = {}
    E.EncoderOracle(arch, p).forward(tok, taps)
    h = taps["l0.ln1"]
    q, k, v = (h @ p[f"l0.{n}.w"].astype(np.float64) for n in "qkv")
    tb = p["rel_bias"].astype(np.float64)
    s00, s01 = q[0] @ k[0] + tb[0, 0], q[0] @ k[1] + tb[17, 0]
    w = np.exp(s01 - s00); want = (v[0] + w * v[1]) / (1 + w)
    assert np.allclose(taps["l0.attn"][0], want, rtol=1e-9, atol=1e-12)


def test_bias_shift_invariance_and_position_dependence():
    p = _params()
    tok = synth.make_tokens([12], ARCH["vocab"])[0]
    y0 = E.EncoderOracle(ARCH, p).forward(tok)
    p2 = dict(p); p2["rel_bias"] = p["rel_bias"] + 3.0                         # softmax ignores a constant
    assert np.allclose(E.EncoderOracle(ARCH, p2).forward(tok), y0, atol=1e-10)
    perm = np.random.default_rng(0).permutation(12)
    p3 = dict(p); p3["rel_bias"] = np.zeros_like(p["rel_bias"])               # without the bias: permutation equivariant
    m = E.EncoderOracle(ARCH, p3)
    assert np.allclose(m.forward(tok[perm]), m.forward(tok)[perm], atol=1e-10)
    m = E.EncoderOracle(ARCH, dict(p, rel_bias=p["rel_bias"] * 40))
    assert not np.allclose(m.forward(tok[perm]), m.forward(tok)[perm], atol=1e-3)


def test_gated_mlp_closed_form():
    arch = dict(ARCH, n_layers=1)
    p = _params(arch)
    for n in "qkvo":
        p[f"l0.{n}.w"] = np.zeros_like(p[f"l0.{n}.w"])
    p["l0.wi1.w"] = np.zeros_like(p["l0.wi1.w"])                               # gate operand 0 -> MLP adds nothing
    tok = synth.make_tokens([7], arch["vocab"])[0]
    taps = {}
    E.EncoderOracle(arch, p).forward(tok, taps)
    assert np.allclose(taps["l0.x_out"], p["embed"][tok], atol=1e-12)
    p = _params(arch)
    taps = {}
    E.EncoderOracle(arch, p).forward(tok, taps)
    h2 = E.rms_norm(taps["l0.x_attn"], p["l0.ln2.g"].astype(np.float64))
    a, b = h2 @ p["l0.wi0.w"].astype(np.float64), h2 @ p["l0.wi1.w"].astype(np.float64)
    assert np.allclose(taps["l0.act"], 0.5 * a * (1 + np.tanh(0.7978845608028654 * (a + 0.044715 * a ** 3))) * b, atol=1e-12)


def test_parameter_count_of_the_xxl_configuration():
    shapes = E.param_shapes(synth.ENCODERS["t5_xxl"])
    n = sum(int(np.prod(s)) for s, _ in shapes.values())
    assert 4.7e9 < n < 4.9e9                                                    # the paper's table: 4.8 B

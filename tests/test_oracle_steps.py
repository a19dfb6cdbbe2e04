"""Pins for each step of the oracle against facts fixed by the mathematics or by
an independent library routine: closed forms, invariants, special cases.
Each test is chosen so that a plausible slip (dropped term, wrong sign or index,
transposed operand) fails it."""
import math

import numpy as np
import pytest
import scipy.special
import torch


def f16(a):
    return np.asarray(a, dtype=np.float16)


# ---- LayerNorm ----------------------------------------------------------
def test_layernorm_pre_affine_has_zero_mean_and_unit_variance(orc):
    rng = np.random.default_rng(1)
    x = rng.standard_normal(2560) * 3.0 + 1.5
    y = orc.layernorm(x, None, None, eps=1e-5)
    assert abs(y.mean()) < 1e-12
    var = x.var()
    assert abs(y.var() - var / (var + 1e-5)) < 1e-12   # eps sits inside the root


def test_layernorm_matches_library_routine(orc):
    rng = np.random.default_rng(2)
    x = rng.standard_normal(512)
    g = f16(1 + 0.02 * rng.standard_normal(512))
    b = f16(0.02 * rng.standard_normal(512))
    want = torch.nn.functional.layer_norm(torch.from_numpy(x), (512,),
                                          torch.from_numpy(g.astype(np.float64)),
                                          torch.from_numpy(b.astype(np.float64)), 1e-5).numpy()
    assert np.abs(orc.layernorm(x, g, b, 1e-5) - want).max() < 1e-12


def test_layernorm_special_cases(orc):
    rng = np.random.default_rng(3)
    beta = f16(rng.standard_normal(64))
    gamma = f16(rng.standard_normal(64))
    # constant input -> exactly beta
    assert np.array_equal(orc.layernorm(np.full(64, 3.25), gamma, beta), beta.astype(np.float64))
    # scale invariance for c > 0 (up to eps), sign flip for c < 0
    x = rng.standard_normal(64)
    y = orc.layernorm(x, None, None, eps=0.0)
    assert np.abs(orc.layernorm(7.0 * x, None, None, eps=0.0) - y).max() < 1e-12
    assert np.abs(orc.layernorm(-2.0 * x, None, None, eps=0.0) + y).max() < 1e-12
    # a large eps must shrink the output: eps is added to the variance, not the std
    x2 = np.array([1.0, -1.0, 1.0, -1.0])
    assert np.allclose(orc.layernorm(x2, None, None, eps=3.0), x2 / 2.0)


# ---- GEMV ---------------------------------------------------------------
def test_gemv_matches_numpy_float64(orc):
    rng = np.random.default_rng(4)
    W = f16(0.02 * rng.standard_normal((96, 160)))
    b = f16(0.02 * rng.standard_normal(96))
    v = rng.standard_normal(160)
    want = W.astype(np.float64) @ v + b.astype(np.float64)
    assert np.abs(orc.gemv(W, b, v) - want).max() < 1e-13
    assert np.abs(orc.gemv(W, None, v) - W.astype(np.float64) @ v).max() < 1e-13


def test_gemv_orientation_by_one_hot(orc):
    W = np.zeros((5, 7), dtype=np.float16)
    W[3, 6] = 2.0           # out[3] = 2 * v[6], nothing else
    v = np.arange(7, dtype=np.float64) + 1
    out = orc.gemv(W, None, v)
    want = np.zeros(5)
    want[3] = 14.0
    assert np.array_equal(out, want)


# ---- RoPE ---------------------------------------------------------------
def test_rope_identity_at_position_zero(orc):
    u = np.random.default_rng(5).standard_normal(80)
    assert np.array_equal(orc.rope(u, 20, 0), u)


def test_rope_hand_value_pins_half_split_pairing_and_frequency(orc):
    # r = 4: pairs are (0, 2) and (1, 3); theta_0 = 1, theta_1 = base^(-2/4) = 0.01
    out = orc.rope(np.array([1.0, 0.0, 0.0, 0.0, 5.0, 6.0]), 4, 1)
    assert np.allclose(out, [math.cos(1), 0, math.sin(1), 0, 5, 6], atol=1e-15)
    out = orc.rope(np.array([0.0, 1.0, 0.0, 0.0]), 4, 3)
    assert np.allclose(out, [0, math.cos(0.03), 0, math.sin(0.03)], atol=1e-15)
    # second element of a pair rotates the other way round: (0,1) -> (-sin, cos)
    out = orc.rope(np.array([0.0, 0.0, 1.0, 0.0]), 4, 2)
    assert np.allclose(out, [-math.sin(2), 0, math.cos(2), 0], atol=1e-15)


def test_rope_preserves_pair_norms_and_passes_the_rest(orc):
    rng = np.random.default_rng(6)
    u = rng.standard_normal(80)
    out = orc.rope(u, 20, 4095)
    assert np.array_equal(out[20:], u[20:])
    assert np.allclose(out[:10] ** 2 + out[10:20] ** 2, u[:10] ** 2 + u[10:20] ** 2, rtol=1e-13)
    assert not np.allclose(out[:20], u[:20])


def test_rope_inner_product_depends_on_relative_position(orc):
    rng = np.random.default_rng(7)
    q, k = rng.standard_normal(64), rng.standard_normal(64)
    a = orc.rope(q, 16, 900) @ orc.rope(k, 16, 880)
    b = orc.rope(q, 16, 120) @ orc.rope(k, 16, 100)
    assert abs(a - b) < 1e-10
    c = orc.rope(q, 16, 120) @ orc.rope(k, 16, 101)
    assert abs(a - c) > 1e-3


# ---- attention ----------------------------------------------------------
def test_attention_single_token_returns_v(orc):
    rng = np.random.default_rng(8)
    K = f16(rng.standard_normal((1, 80)))
    V = f16(rng.standard_normal((1, 80)))
    o = orc.attention_head(rng.standard_normal(80), K, V, 1)
    assert np.array_equal(o, V[0].astype(np.float64))


def test_attention_softmax_rows_sum_to_one_and_shift_invariance(orc):
    rng = np.random.default_rng(9)
    K = f16(rng.standard_normal((300, 64)))
    V = f16(rng.standard_normal((300, 64)))
    q = rng.standard_normal(64) * 3
    o, p = orc.attention_head(q, K, V, 300, return_probs=True)
    assert abs(p.sum() - 1.0) < 1e-12 and (p >= 0).all()
    # probabilities equal the library softmax of q.K/sqrt(d)
    s = K.astype(np.float64) @ q / math.sqrt(64)
    assert np.abs(p - scipy.special.softmax(s)).max() < 1e-14
    assert np.abs(o - scipy.special.softmax(s) @ V.astype(np.float64)).max() < 1e-13
    # q = 0 -> uniform weights -> mean of V
    o0 = orc.attention_head(np.zeros(64), K, V, 300)
    assert np.abs(o0 - V.astype(np.float64).mean(0)).max() < 1e-13


def test_attention_dominant_score_and_poisoned_tail(orc):
    rng = np.random.default_rng(10)
    K = f16(rng.standard_normal((40, 64)) * 0.1)
    V = f16(rng.standard_normal((40, 64)))
    q = np.zeros(64)
    q[0] = 8.0
    K[17, 0] = 400.0            # score 400 above the others
    o = orc.attention_head(q, K, V, 30)
    assert np.abs(o - V[17].astype(np.float64)).max() < 1e-12
    # rows at or beyond n_pos must never be read
    K[30:] = np.nan
    V[30:] = np.nan
    assert np.array_equal(orc.attention_head(q, K, V, 30), o)


def test_attention_scale_is_one_over_sqrt_head_dim(orc):
    # two keys, scores (ln 3 * sqrt(d), 0) / sqrt(d) -> probabilities (3/4, 1/4)
    d = 80
    K = np.zeros((2, d), dtype=np.float16)
    K[0, 0] = 1.0
    V = np.zeros((2, d), dtype=np.float16)
    V[0, 0] = 1.0
    V[1, 1] = 1.0
    q = np.zeros(d)
    q[0] = math.log(3.0) * math.sqrt(d)
    o = orc.attention_head(q, K, V, 2)
    assert abs(o[0] - 0.75) < 1e-12 and abs(o[1] - 0.25) < 1e-12


# ---- GELU ---------------------------------------------------------------
def test_gelu_closed_forms(orc):
    z = np.linspace(-9, 9, 3601)
    g = orc.gelu(z)
    want = 0.5 * z * (1 + scipy.special.erf(z / math.sqrt(2)))
    assert np.abs(g - want).max() < 1e-15
    assert orc.gelu(np.array([0.0]))[0] == 0.0
    assert np.abs(orc.gelu(z) - orc.gelu(-z) - z).max() < 1e-14       # odd part is z/2
    assert abs(orc.gelu(np.array([30.0]))[0] - 30.0) < 1e-12
    assert abs(orc.gelu(np.array([-30.0]))[0]) < 1e-12
    # the tanh approximation differs by about 1e-4 near z = 2; make sure we are the erf form
    t = 0.5 * 2.0 * (1 + math.tanh(math.sqrt(2 / math.pi) * (2.0 + 0.044715 * 8.0)))
    assert abs(orc.gelu(np.array([2.0]))[0] - t) > 5e-5
    # standard normal CDF: gelu(z) = z * Phi(z)
    assert abs(orc.gelu(np.array([1.0]))[0] - 0.8413447460685429) < 1e-15

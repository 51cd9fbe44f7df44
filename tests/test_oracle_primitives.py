"""Pins of the oracle's primitives against closed forms, library routines and
the values the paper's equations fix.  CPU only."""
import math

import numpy as np
import pytest
from scipy.special import softmax

import oracle as orc
from sb_inputs import round_to_bf16, bf16_to_f32

BITS = [64, 32]


def tol(bits):
    return 1e-12 if bits == 64 else 2e-5


@pytest.mark.parametrize("bits", BITS)
def test_matvec_equals_numpy_matmul(bits):
    g = np.random.default_rng(0)
    W = g.standard_normal((37, 53)).astype(np.float32)   # non-square: a transposed read fails
    x = g.standard_normal(53)
    y = orc.matvec(W, x, bits)
    ref = W.astype(np.float64) @ x
    assert np.allclose(y, ref, rtol=0, atol=tol(bits) * 50)


@pytest.mark.parametrize("bits", BITS)
def test_matvec_bf16_weights_are_upcast_exactly(bits):
    g = np.random.default_rng(1)
    Wb = round_to_bf16(g.standard_normal((19, 64)).astype(np.float32))
    x = g.standard_normal(64)
    y = orc.matvec(Wb, x, bits)
    ref = bf16_to_f32(Wb).astype(np.float64) @ x
    assert np.allclose(y, ref, rtol=0, atol=tol(bits) * 50)
    # one-hot x picks out a column: exact in any precision
    e = np.zeros(64); e[7] = 1.0
    assert np.array_equal(orc.matvec(Wb, e, bits), bf16_to_f32(Wb)[:, 7].astype(np.float64))


def test_bf16_rounding_is_nearest_even():
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: even mantissa (1.0) wins
    a = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -9, -(1.0 + 2.0 ** -8)], np.float32)
    r = bf16_to_f32(round_to_bf16(a))
    assert r.tolist() == [1.0, 1.0 + 2.0 ** -6, 1.0, -1.0]


@pytest.mark.parametrize("bits", BITS)
def test_rmsnorm_hand_values(bits):
    out = orc.rmsnorm(np.array([3.0, 4.0]), np.array([1.0, 2.0], np.float32), 0.0, bits)
    rms = math.sqrt(12.5)
    assert np.allclose(out, [3 / rms, 8 / rms], atol=tol(bits))
    # a constant vector normalises to sign * g (eps -> 0)
    g = np.linspace(0.5, 1.5, 16).astype(np.float32)
    assert np.allclose(orc.rmsnorm(np.full(16, -7.0), g, 0.0, bits), -g, atol=tol(bits) * 4)
    # eps enters under the root, added to the mean square
    out = orc.rmsnorm(np.array([1.0, 1.0]), np.ones(2, np.float32), 3.0, bits)
    assert np.allclose(out, [0.5, 0.5], atol=tol(bits))


@pytest.mark.parametrize("bits", BITS)
def test_swiglu_closed_forms_and_library_routine(bits):
    """silu(g) * v: hand values, the identities silu(g) - silu(-g) = g and silu(g) + silu(-g) =
    g tanh(g / 2), the limits, operand order (gate first, up second), and torch's own silu."""
    import torch
    t = tol(bits)
    # silu(0) = 0; silu(ln 3) = ln 3 * 3/4; the up value multiplies
    out = orc.swiglu(np.array([0.0, math.log(3.0), 5.0, 2.0]), bits)       # gates 0, ln 3; ups 5, 2
    assert np.allclose(out, [0.0, math.log(3.0) * 0.75 * 2.0], atol=t)
    g = np.linspace(-9.0, 9.0, 37)
    one = np.ones_like(g)
    sp, sm = orc.swiglu(np.concatenate([g, one]), bits), orc.swiglu(np.concatenate([-g, one]), bits)
    assert np.allclose(sp - sm, g, atol=t * 10)
    assert np.allclose(sp + sm, g * np.tanh(g / 2), atol=t * 10)
    # large gates pass through, very negative ones close
    assert np.allclose(orc.swiglu(np.array([40.0, -40.0, 1.5, 1.5]), bits), [60.0, 0.0], atol=1e-12 if bits == 64 else 1e-5)
    # gate and up are not interchangeable
    assert not np.allclose(orc.swiglu(np.array([1.0, 3.0]), bits), orc.swiglu(np.array([3.0, 1.0]), bits))
    r = np.random.default_rng(5)
    gu = r.standard_normal(2 * 300) * 3
    ref = (torch.nn.functional.silu(torch.from_numpy(gu[:300])) * torch.from_numpy(gu[300:])).numpy()
    assert np.allclose(orc.swiglu(gu, bits), ref, atol=t * 30, rtol=t * 10)


@pytest.mark.parametrize("bits", BITS)
def test_rope_rotation_hand_values(bits):
    # hd = 2: one pair, theta_0 = 1, so position p rotates (1,0) by p radians
    v = orc.rope_apply(np.array([1.0, 0.0]), 1, 10000.0, bits)
    assert np.allclose(v, [math.cos(1.0), math.sin(1.0)], atol=1e-7)
    # hd = 4: pairs (0,2) and (1,3); theta_1 = base^(-2/4) = 0.01 for base 1e4
    v = orc.rope_apply(np.array([0.0, 1.0, 0.0, 0.0]), 50, 10000.0, bits)
    assert np.allclose(v, [0.0, math.cos(0.5), 0.0, math.sin(0.5)], atol=1e-7)
    # position 0 is the identity
    x = np.random.default_rng(2).standard_normal(64)
    assert np.array_equal(orc.rope_apply(x, 0, 10000.0, bits), x.astype(np.float64 if bits == 64 else np.float32))


def test_rope_scores_depend_on_relative_position_only():
    g = np.random.default_rng(3)
    q, k = g.standard_normal(64), g.standard_normal(64)
    def score(m, n):
        return float(orc.rope_apply(q, m, 10000.0) @ orc.rope_apply(k, n, 10000.0))
    assert abs(score(5, 3) - score(12, 10)) < 1e-5
    assert abs(score(7, 7) - float(q @ k)) < 1e-5
    assert abs(score(5, 3) - score(3, 5)) > 1e-3      # not symmetric: direction matters
    # norm preserved
    assert abs(np.linalg.norm(orc.rope_apply(q, 9, 10000.0)) - np.linalg.norm(q)) < 1e-5


@pytest.mark.parametrize("bits", BITS)
def test_attention_head_special_cases(bits):
    g = np.random.default_rng(4)
    hd = 8
    q = g.standard_normal(hd)
    K = g.standard_normal((5, hd)).astype(np.float32)
    V = g.standard_normal((5, hd)).astype(np.float32)
    # one key: the output is its value row
    assert np.allclose(orc.attention_head(q, K[:1], V[:1], bits), V[0], atol=tol(bits))
    # zero query: uniform weights, output is the mean of V
    assert np.allclose(orc.attention_head(np.zeros(hd), K, V, bits), V.mean(0), atol=tol(bits) * 10)
    # library softmax with the 1/sqrt(hd) scale
    p = softmax((K.astype(np.float64) @ q) / math.sqrt(hd))
    assert np.allclose(orc.attention_head(q, K, V, bits), p @ V.astype(np.float64), atol=tol(bits) * 20)
    # hand value: hd=4, q=(2,0,0,0), keys e0 and 0 -> scores (1, 0)
    q4 = np.array([2.0, 0, 0, 0]); K4 = np.array([[1, 0, 0, 0], [0, 0, 0, 0]], np.float32)
    V4 = np.array([[1, 0, 0, 0], [0, 1, 0, 0]], np.float32)
    w0 = math.e / (1 + math.e)
    assert np.allclose(orc.attention_head(q4, K4, V4, bits), [w0, 1 - w0, 0, 0], atol=tol(bits))


@pytest.mark.parametrize("bits", BITS)
def test_act_confidence_closed_forms(bits):
    V = 1000
    # Eq. 2 with T = 1 is the plain softmax maximum
    z = np.random.default_rng(5).standard_normal(V) * 3
    am, p = orc.act(z, 1.0, bits)
    sm = softmax(z)
    assert am == int(np.argmax(z)) and abs(p - sm.max()) < tol(bits) * 10
    # general T: softmax of z/T
    for T in (2.0, 1.3, 0.7):
        am2, pT = orc.act(z, T, bits)
        assert am2 == am                      # arg max does not depend on T
        assert abs(pT - softmax(z / T).max()) < tol(bits) * 10
    # one hot logit a, the rest 0: p = e^{a/T} / (e^{a/T} + V - 1)
    z1 = np.zeros(V); z1[123] = 4.0
    for T in (1.0, 2.0):
        am3, p3 = orc.act(z1, T, bits)
        e = math.exp(4.0 / T)
        assert am3 == 123 and abs(p3 - e / (e + V - 1)) < tol(bits)
    # T -> infinity flattens to 1/V; confidence decreases as T grows
    assert abs(orc.act(z, 1e9, bits)[1] - 1.0 / V) < 1e-6
    ps = [orc.act(z, T, bits)[1] for T in (0.5, 1.0, 1.5, 2.0, 4.0)]
    assert all(a > b for a, b in zip(ps, ps[1:]))
    # ties: lowest index wins
    zt = np.zeros(10); zt[3] = zt[7] = 2.0
    assert orc.act(zt, 1.0, bits)[0] == 3


def test_temperature_schedule_eq1(golden):
    gd = golden("paper_equations.txt")
    T = orc.temperature_schedule(gd["eq1_alpha"][0], gd["eq1_L"][0], gd["eq1_L"][0])
    for l, want in zip(gd["eq1_layers"], gd["eq1_T"]):
        assert abs(float(T[l - 1]) - want) < 1e-6
    assert float(T[-1]) == 1.0                    # T_L = 1: the base model's distribution
    assert all(a > b for a, b in zip(T, T[1:]))   # hotter in shallow layers


def test_speedup_model_eq3_to_eq5(golden):
    gd = golden("paper_equations.txt")
    assert abs(orc.round_time(32, 10, 8) - gd["eq3_value"][0]) < 1e-12
    assert abs(orc.expected_accept(0.9, 8) - gd["eq4_value"][0]) < 1e-6
    assert abs(orc.speedup(32, 10, 8, 0.9) - gd["eq5_value"][0]) < 1e-6
    # Eq. 4's two sides agree for other parameters (the oracle evaluates the sum)
    for a in (0.1, 0.5, 0.77):
        for w in (1, 3, 8):
            assert abs(orc.expected_accept(a, w) - a * (1 - a ** w) / (1 - a)) < 1e-12
    # Monte Carlo under the geometric-acceptance assumption
    g = np.random.default_rng(6)
    a, w = 0.8, 6
    acc = (g.random((200000, w)) < a)
    n_acc = np.where(acc.all(1), w, acc.argmin(1))
    assert abs(n_acc.mean() - orc.expected_accept(a, w)) < 0.02

"""Pins for the oracle's elementwise pieces and attention: closed forms, hand
values, invariants and brute force with explicit scalar loops."""
import math

import numpy as np
import pytest

from oracle import mdi_oracle as O

rng = np.random.default_rng(7)


# ---------------------------------------------------------------- norms
def test_layernorm_hand_values():
    # x = 1,2,3,4: mean 2.5, biased variance 1.25
    y = O.layernorm(np.array([[1.0, 2.0, 3.0, 4.0]]), 1.0, 0.0, 0.0)
    s = math.sqrt(1.25)
    np.testing.assert_allclose(y[0], [-1.5 / s, -0.5 / s, 0.5 / s, 1.5 / s], rtol=1e-15)
    # gain and bias act after the normalisation
    y2 = O.layernorm(np.array([[1.0, 2.0, 3.0, 4.0]]), np.array([2.0, 2.0, 2.0, 2.0]), np.array([1.0, 0, 0, 0]), 0.0)
    np.testing.assert_allclose(y2[0], [2 * -1.5 / s + 1, 2 * -0.5 / s, 2 * 0.5 / s, 2 * 1.5 / s], rtol=1e-15)


def test_layernorm_moments_and_scale_invariance():
    x = rng.standard_normal((5, 64))
    y = O.layernorm(x, 1.0, 0.0, 0.0)
    np.testing.assert_allclose(y.mean(-1), 0, atol=1e-14)
    np.testing.assert_allclose((y * y).mean(-1), 1, rtol=1e-12)
    np.testing.assert_allclose(O.layernorm(3.7 * x, 1.0, 0.0, 0.0), y, rtol=1e-12, atol=1e-14)
    # eps enters under the root, next to the variance
    v = x.var(-1, keepdims=True)
    np.testing.assert_allclose(O.layernorm(x, 1.0, 0.0, 0.5), y * np.sqrt(v / (v + 0.5)), rtol=1e-12, atol=1e-14)


def test_rmsnorm_hand_values_and_invariants():
    y = O.rmsnorm(np.array([[3.0, 4.0]]), 1.0, 0.0)          # rms = sqrt(12.5)
    np.testing.assert_allclose(y[0], [3 / math.sqrt(12.5), 4 / math.sqrt(12.5)], rtol=1e-15)
    x = rng.standard_normal((4, 32)) + 2.0                    # non-zero mean: no centring happens
    y = O.rmsnorm(x, 1.0, 0.0)
    np.testing.assert_allclose((y * y).mean(-1), 1, rtol=1e-12)
    np.testing.assert_allclose(O.rmsnorm(0.3 * x, 1.0, 0.0), y, rtol=1e-12)
    g = rng.standard_normal(32)
    np.testing.assert_allclose(O.rmsnorm(x, g, 0.0), y * g, rtol=1e-12)
    ms = (x * x).mean(-1, keepdims=True)
    np.testing.assert_allclose(O.rmsnorm(x, 1.0, 0.25), x / np.sqrt(ms + 0.25), rtol=1e-12)


# ---------------------------------------------------------------- activations
def test_activation_known_values():
    x = np.array([0.0, 1.0, -1.0, 10.0, -10.0])
    # x * Phi(x) with Phi(1) = 0.8413447460685429 (standard normal CDF)
    np.testing.assert_allclose(O.gelu_erf(x), [0, 0.8413447460685429, -0.15865525393145707, 10.0, 0.0], atol=1e-12)
    # tanh form at 1: 0.5*(1+tanh(sqrt(2/pi)*1.044715)) = 0.8411919906082768
    np.testing.assert_allclose(O.gelu_tanh(x), [0, 0.8411919906082768, -0.15880800939172324, 10.0, 0.0], atol=1e-12)
    # logistic(1) = 0.7310585786300049
    np.testing.assert_allclose(O.silu(x), [0, 0.7310585786300049, -0.2689414213699951, 10 / (1 + math.exp(-10)), -10 / (1 + math.exp(10))], rtol=1e-13)
    xs = np.linspace(-6, 6, 2001)
    assert np.abs(O.gelu_tanh(xs) - O.gelu_erf(xs)).max() < 1e-3      # the two variants stay close


def test_softmax_rows():
    s = rng.standard_normal((6, 37)) * 5
    p = O.softmax_rows(s)
    np.testing.assert_allclose(p.sum(-1), 1.0, atol=1e-12)
    assert (p >= 0).all()
    np.testing.assert_allclose(O.softmax_rows(np.array([[0.0, math.log(2.0)]])), [[1 / 3, 2 / 3]], rtol=1e-15)
    np.testing.assert_allclose(O.softmax_rows(s + 1000.0), p, rtol=1e-12)   # shift invariance, no overflow
    np.testing.assert_allclose(O.pmf(s[0]).sum(), 1.0, atol=1e-12)


# ---------------------------------------------------------------- RoPE
def test_rope_pairing_and_angles():
    h = 4
    x = np.zeros((1, 1, h)); x[0, 0, 0] = 1.0                  # unit vector on lane 0, partner is lane h/2
    y = O.rope_rotate(x, [3], 10000.0)                         # i = 0: theta = 1, angle = 3
    np.testing.assert_allclose(y[0, 0], [math.cos(3), 0, math.sin(3), 0], atol=1e-15)
    x = np.zeros((1, 1, h)); x[0, 0, 1] = 1.0                  # i = 1: theta = 10000**(-2/4) = 0.01
    y = O.rope_rotate(x, [50], 10000.0)
    np.testing.assert_allclose(y[0, 0], [0, math.cos(0.5), 0, math.sin(0.5)], atol=1e-14)
    x = np.zeros((1, 1, h)); x[0, 0, 3] = 1.0                  # second element of pair 1
    y = O.rope_rotate(x, [50], 10000.0)
    np.testing.assert_allclose(y[0, 0], [0, -math.sin(0.5), 0, math.cos(0.5)], atol=1e-14)


def test_rope_invariants():
    q = rng.standard_normal((5, 3, 16)); k = rng.standard_normal((5, 3, 16))
    np.testing.assert_array_equal(O.rope_rotate(q, np.zeros(5), 500000.0), q)      # position 0 is the identity
    pos = np.array([0, 1, 7, 100, 4000])
    qr = O.rope_rotate(q, pos, 10000.0)
    np.testing.assert_allclose((qr * qr).sum(-1), (q * q).sum(-1), rtol=1e-12)     # a rotation
    # scores depend on the position difference only
    s1 = np.einsum("thd,thd->th", O.rope_rotate(q, pos + 3, 1e4), O.rope_rotate(k, pos, 1e4))
    s2 = np.einsum("thd,thd->th", O.rope_rotate(q, pos + 20, 1e4), O.rope_rotate(k, pos + 17, 1e4))
    np.testing.assert_allclose(s1, s2, rtol=1e-9, atol=1e-11)


# ---------------------------------------------------------------- attention
def brute_attention(q, k, v, pos0):
    """Scalar triple loops, float64, no numpy arithmetic."""
    T, H, h = q.shape
    c, K, _ = k.shape
    out = [[[0.0] * h for _ in range(H)] for _ in range(T)]
    for t in range(T):
        for j in range(H):
            kv = j // (H // K)
            scores = []
            for u in range(pos0 + t + 1):
                acc = 0.0
                for e in range(h):
                    acc += float(q[t, j, e]) * float(k[u, kv, e])
                scores.append(acc / math.sqrt(h))
            m = max(scores)
            w = [math.exp(s - m) for s in scores]
            z = sum(w)
            for e in range(h):
                out[t][j][e] = sum(w[u] * float(v[u, kv, e]) for u in range(len(w))) / z
    return np.array(out)


@pytest.mark.parametrize("H,K", [(4, 1), (4, 2), (4, 4), (1, 1), (3, 3)])
@pytest.mark.parametrize("T,pos0", [(8, 0), (1, 7), (3, 5)])
def test_attention_vs_brute_force(H, K, T, pos0):
    h = 4
    c = pos0 + T
    q = rng.standard_normal((T, H, h)); k = rng.standard_normal((c, K, h)); v = rng.standard_normal((c, K, h))
    np.testing.assert_allclose(O.causal_attention(q, k, v, pos0), brute_attention(q, k, v, pos0), rtol=1e-12, atol=1e-13)


def test_attention_special_cases():
    T, H, K, h = 6, 4, 2, 8
    q = rng.standard_normal((T, H, h)); k = rng.standard_normal((T, K, h)); v = rng.standard_normal((T, K, h))
    o = O.causal_attention(q, k, v, 0)
    # position 0 attends to itself only: weight 1, output v_0
    for j in range(H):
        np.testing.assert_allclose(o[0, j], v[0, j // 2], rtol=1e-15)
    # zero queries: uniform weights, output is the prefix mean of V
    o0 = O.causal_attention(np.zeros_like(q), k, v, 0)
    for t in range(T):
        np.testing.assert_allclose(o0[t, 3], v[:t + 1, 1].mean(0), rtol=1e-12)
    # causality: changing token 4 leaves rows 0..3 untouched
    k2, v2 = k.copy(), v.copy(); k2[4] += 1.0; v2[4] -= 2.0
    o2 = O.causal_attention(q, k2, v2, 0)
    np.testing.assert_array_equal(o2[:4], o[:4])
    assert np.abs(o2[4:] - o[4:]).max() > 1e-3
    # grouped heads equal full multi-head attention with each kv head repeated
    o_mha = O.causal_attention(q, np.repeat(k, 2, axis=1), np.repeat(v, 2, axis=1), 0)
    np.testing.assert_allclose(o_mha, o, rtol=1e-15)
    # the 1/sqrt(h) scale: one query, two keys with known scores
    qq = np.zeros((1, 1, 4)); qq[0, 0, 0] = 2.0
    kk = np.zeros((2, 1, 4)); kk[1, 0, 0] = math.log(3.0)      # scores 0 and 2*ln3/2 = ln 3
    vv = np.zeros((2, 1, 4)); vv[0, 0, 0] = 1.0; vv[1, 0, 1] = 1.0
    np.testing.assert_allclose(O.causal_attention(qq, kk, vv, 1)[0, 0], [0.25, 0.75, 0, 0], rtol=1e-14)


def test_greedy_rule():
    assert O.greedy(np.full(17, 0.25)) == 0                       # exact ties: lowest index
    z = np.zeros(17); z[11] = 1e-9
    assert O.greedy(z) == 11
    z[5] = 1e-9
    assert O.greedy(z) == 5

"""Pins for the oracle's elementary operators: plain-Python brute force on tiny inputs,
library routines (torch CPU, scipy) they must reduce to, and closed-form special cases."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F
from scipy.special import erf

from oracle import block as ob


def _loops_attention(q, k, v):
    h, nq, hd = len(q), len(q[0]), len(q[0][0])
    nk = len(k[0])
    out = [[[0.0] * hd for _ in range(nq)] for _ in range(h)]
    for a in range(h):
        for i in range(nq):
            s = [sum(q[a][i][c] * k[a][j][c] for c in range(hd)) / math.sqrt(hd) for j in range(nk)]
            mx = max(s)
            e = [math.exp(t - mx) for t in s]
            z = sum(e)
            for c in range(hd):
                out[a][i][c] = sum(e[j] * v[a][j][c] for j in range(nk)) / z
    return np.array(out)


def test_attention_brute_force_tiny():
    rng = np.random.default_rng(0)
    q, k, v = rng.normal(size=(2, 5, 4)), rng.normal(size=(2, 7, 4)), rng.normal(size=(2, 7, 4))
    np.testing.assert_allclose(ob.attention(q, k, v), _loops_attention(q.tolist(), k.tolist(), v.tolist()),
                               rtol=1e-12, atol=1e-14)


def test_attention_equals_library_sdpa():
    rng = np.random.default_rng(1)
    q, k, v = rng.normal(size=(3, 33, 16)), rng.normal(size=(3, 50, 16)), rng.normal(size=(3, 50, 16))
    ref = F.scaled_dot_product_attention(torch.from_numpy(q), torch.from_numpy(k), torch.from_numpy(v)).numpy()
    np.testing.assert_allclose(ob.attention(q, k, v), ref, rtol=1e-10, atol=1e-12)


def test_softmax_rows_sum_to_one_and_shift_invariant():
    rng = np.random.default_rng(2)
    s = rng.normal(size=(64, 300)) * 30
    p = ob.softmax_rows(s)
    assert np.abs(p.sum(-1) - 1).max() < 1e-12
    np.testing.assert_allclose(ob.softmax_rows(s + 1000.0), p, rtol=1e-9)
    assert np.isfinite(ob.softmax_rows(s * 100)).all()


def test_attention_special_cases():
    rng = np.random.default_rng(3)
    q, k = rng.normal(size=(1, 6, 8)), rng.normal(size=(1, 9, 8))
    v_same = np.tile(rng.normal(size=(1, 1, 8)), (1, 9, 1))
    np.testing.assert_allclose(ob.attention(q, k, v_same), np.tile(v_same[:, :1], (1, 6, 1)), atol=1e-13)
    v = rng.normal(size=(1, 9, 8))
    perm = rng.permutation(9)
    np.testing.assert_allclose(ob.attention(q, k[:, perm], v[:, perm]), ob.attention(q, k, v), atol=1e-13)
    # one key dominates: output tends to that key's value row
    kd = k.copy()
    kd[0, 4] = q[0, 2] * 200
    assert np.abs(ob.attention(q, kd, v)[0, 2] - v[0, 4]).max() < 1e-9
    # zero queries: uniform average of the values
    np.testing.assert_allclose(ob.attention(np.zeros_like(q), k, v)[0, 0], v[0].mean(0), atol=1e-13)


def test_layernorm_against_library_and_moments():
    rng = np.random.default_rng(4)
    x = rng.normal(size=(10, 96)) * 3 + 1.5
    ref = F.layer_norm(torch.from_numpy(x), (96,), eps=1e-6).numpy()
    y = ob.layernorm(x)
    np.testing.assert_allclose(y, ref, rtol=1e-10, atol=1e-12)
    assert np.abs(y.mean(-1)).max() < 1e-12
    assert np.abs(y.var(-1) - 1).max() < 1e-5          # eps makes it just under 1


def test_rmsnorm_loops():
    rng = np.random.default_rng(5)
    x, w = rng.normal(size=(3, 4, 8)), rng.normal(size=8)
    y = ob.rmsnorm(x, w)
    for a in range(3):
        for b in range(4):
            ms = sum(float(t) ** 2 for t in x[a, b]) / 8
            for c in range(8):
                assert y[a, b, c] == pytest.approx(x[a, b, c] / math.sqrt(ms + 1e-6) * w[c], rel=1e-12)
    if hasattr(F, "rms_norm"):
        ref = F.rms_norm(torch.from_numpy(x), (8,), torch.from_numpy(w), eps=1e-6).numpy()
        np.testing.assert_allclose(y, ref, rtol=1e-10)


def test_gelu_tanh_against_library_and_exact_gelu():
    x = np.linspace(-8, 8, 4001)
    ref = F.gelu(torch.from_numpy(x), approximate="tanh").numpy()
    np.testing.assert_allclose(ob.gelu_tanh(x), ref, rtol=1e-12, atol=1e-14)
    exact = 0.5 * x * (1 + erf(x / math.sqrt(2)))
    assert np.abs(ob.gelu_tanh(x) - exact).max() < 1e-3   # the tanh form approximates x*Phi(x)
    assert ob.gelu_tanh(np.array([0.0]))[0] == 0.0
    assert ob.gelu_tanh(np.array([10.0]))[0] == pytest.approx(10.0, abs=1e-12)
    assert abs(ob.gelu_tanh(np.array([-10.0]))[0]) < 1e-12
    # published 4-digit values of the tanh form
    np.testing.assert_allclose(ob.gelu_tanh(np.array([1.0, -1.0, 2.0])), [0.8412, -0.1588, 1.9546], atol=5e-5)


def test_linear_is_x_wT_plus_b():
    rng = np.random.default_rng(6)
    x, w, b = rng.normal(size=(4, 5)), rng.normal(size=(3, 5)), rng.normal(size=3)
    y = ob.linear(x, w, b)
    for i in range(4):
        for o in range(3):
            assert y[i, o] == pytest.approx(sum(x[i, c] * w[o, c] for c in range(5)) + b[o], rel=1e-12)
    np.testing.assert_array_equal(ob.linear(x, np.eye(5), None), x)
    mc = ob.MacCounter()
    ob.linear(x, w, b, mc, "t")
    assert mc.flops("t") == 2 * 4 * 3 * 5


def test_widen_is_exact_bf16():
    bits = np.array([0x3F80, 0xBF80, 0x4049, 0x0000, 0x3C00], dtype=np.uint16)
    np.testing.assert_array_equal(ob.widen(bits), [1.0, -1.0, 3.140625, 0.0, 0.0078125])


def test_rope_is_a_complex_rotation_of_consecutive_pairs():
    """The oracle's rotary embedding against complex multiplication, hand values, and the property
    that makes it a position embedding: with angles pos * omega_i the product q.k depends on the
    difference of the positions only."""
    rng = np.random.default_rng(5)
    n, H, hd = 7, 3, 8
    x = rng.normal(size=(n, H, hd))
    ang = rng.uniform(0, 2 * np.pi, size=(n, hd // 2))
    got = ob.rope(x, np.cos(ang), np.sin(ang))
    z = (x[..., 0::2] + 1j * x[..., 1::2]) * np.exp(1j * ang)[:, None, :]
    assert np.allclose(got[..., 0::2], z.real, atol=1e-14) and np.allclose(got[..., 1::2], z.imag, atol=1e-14)
    # identity at angle zero; every pair keeps its length
    assert np.array_equal(ob.rope(x, np.ones((n, hd // 2)), np.zeros((n, hd // 2))), x)
    assert np.allclose(got[..., 0::2] ** 2 + got[..., 1::2] ** 2, x[..., 0::2] ** 2 + x[..., 1::2] ** 2)
    # by hand: (1, 0) turned a quarter is (0, 1); (3, 4) turned a half is (-3, -4)
    v = np.array([[[1.0, 0.0, 3.0, 4.0]]])
    a = np.array([[np.pi / 2, np.pi]])
    assert np.allclose(ob.rope(v, np.cos(a), np.sin(a)), [[[0.0, 1.0, -3.0, -4.0]]], atol=1e-15)
    # relative positions
    omega = 100.0 ** (-np.arange(hd // 2) / (hd // 2))
    q, k = rng.normal(size=(1, 1, hd)), rng.normal(size=(1, 1, hd))
    def score(m, nn):
        am, an = (m * omega)[None], (nn * omega)[None]
        return float((ob.rope(q, np.cos(am), np.sin(am)) * ob.rope(k, np.cos(an), np.sin(an))).sum())
    assert score(5, 2) == pytest.approx(score(13, 10), rel=1e-12)
    assert abs(score(5, 2) - score(5, 3)) > 1e-3


def test_gelu_erf_against_library():
    x = np.linspace(-6, 6, 2001)
    want = F.gelu(torch.from_numpy(x)).numpy()                       # the library's exact form
    assert np.allclose(ob.gelu_erf(x), want, atol=1e-15)
    assert ob.gelu_erf(np.array([0.0]))[0] == 0.0
    # the tanh form is an approximation of this one, good to about 5e-4
    assert 1e-5 < np.abs(ob.gelu_erf(x) - ob.gelu_tanh(x)).max() < 1e-3

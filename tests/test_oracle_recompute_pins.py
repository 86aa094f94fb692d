"""Pins of the recomputation oracle (LayerNorm and the projection that follow the stored layer
input, Section 4.1): hand-worked values, closed forms, invariances and brute force."""
import math

import numpy as np
import pytest

from oracle import memo_recompute_oracle as ro


def test_layernorm_hand_example():
    # x = (1,2,3,4): mean 2.5, biased variance 1.25; gamma = (1,2,1,2), beta = (0,0,1,1), eps = 0
    y = ro.layernorm([[1.0, 2.0, 3.0, 4.0]], [1, 2, 1, 2], [0, 0, 1, 1], 0.0)
    r = 1.0 / math.sqrt(1.25)
    assert np.allclose(y, [[-1.5 * r, -0.5 * r * 2, 0.5 * r + 1, 1.5 * r * 2 + 1]], rtol=0, atol=1e-15)


def test_layernorm_constant_row_gives_beta():
    beta = np.linspace(-1, 1, 16)
    y = ro.layernorm(np.full((3, 16), 7.25), np.ones(16) * 3, beta, 1e-5)
    assert np.array_equal(y, np.tile(beta, (3, 1)))


def test_layernorm_invariances():
    rng = np.random.default_rng(0)
    x = rng.normal(size=(5, 64))
    g, b = rng.normal(size=64), rng.normal(size=64)
    base = ro.layernorm(x, g, b, 0.0)
    assert np.allclose(ro.layernorm(x + 3.5, g, b, 0.0), base, atol=1e-12)      # shift
    assert np.allclose(ro.layernorm(x * 4.0, g, b, 0.0), base, atol=1e-12)      # scale (eps = 0)
    plain = ro.layernorm(x, np.ones(64), np.zeros(64), 0.0)
    assert np.allclose(plain.mean(axis=1), 0.0, atol=1e-13)
    assert np.allclose((plain ** 2).mean(axis=1), 1.0, atol=1e-12)
    # eps enters under the root: a row of variance v is scaled by 1/sqrt(v + eps)
    v = x.var(axis=1, keepdims=True)
    assert np.allclose(ro.layernorm(x, np.ones(64), np.zeros(64), 0.5), plain * np.sqrt(v / (v + 0.5)), atol=1e-12)


def test_layernorm_rows_are_independent():
    rng = np.random.default_rng(1)
    x = rng.normal(size=(6, 32))
    g, b = rng.normal(size=32), rng.normal(size=32)
    full = ro.layernorm(x, g, b, 1e-5)
    assert np.array_equal(ro.layernorm(x[2:5], g, b, 1e-5), full[2:5])


def test_linear_brute_force_and_special_cases():
    rng = np.random.default_rng(2)
    a, w, bias = rng.normal(size=(4, 5)), rng.normal(size=(3, 5)), rng.normal(size=3)
    want = np.zeros((4, 3))
    for i in range(4):
        for n in range(3):
            acc = 0.0
            for c in range(5):
                acc += a[i, c] * w[n, c]
            want[i, n] = acc + bias[n]
    assert np.allclose(ro.linear(a, w, bias), want, atol=1e-14)
    assert np.array_equal(ro.linear(a, np.eye(5)), a)                           # identity weight
    assert np.allclose(ro.linear(a, w), ro.linear(a, w, bias) - bias, atol=1e-14)
    assert np.allclose(ro.linear(2 * a, w), 2 * ro.linear(a, w), atol=1e-14)    # linear in a
    # a one-hot row picks a column of w
    e = np.zeros((1, 5)); e[0, 3] = 1.0
    assert np.array_equal(ro.linear(e, w)[0], w[:, 3])


@pytest.mark.parametrize("k", [0, 3, 7])
def test_stitch_equals_full_tensor(k):
    rng = np.random.default_rng(3)
    x = rng.normal(size=(7, 16))
    g, b, w = rng.normal(size=16), rng.normal(size=16), rng.normal(size=(8, 16))
    full = ro.linear(ro.layernorm(x, g, b, 1e-5), w)
    swapped = full[:k].copy()
    recomputed = np.full_like(full, np.nan)
    recomputed[k:] = ro.linear(ro.layernorm(x[k:], g, b, 1e-5), w)
    assert np.array_equal(ro.stitch(swapped, recomputed, k), full)

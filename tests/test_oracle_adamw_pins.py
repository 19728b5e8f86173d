"""Pins for the AdamW oracle (CPU only): pure-Python loops, the constant-gradient closed form, degenerate cases."""
import math

import numpy as np
import pytest

from oracle import adamw_oracle as ao


def py_adamw(p, g, m, v, lr, wd, b1, b2, eps, t):
    out_p, out_m, out_v = [], [], []
    for pi, gi, mi, vi in zip(p, g, m, v):
        mn = b1 * mi + (1 - b1) * gi
        vn = b2 * vi + (1 - b2) * gi * gi
        mh = mn / (1 - b1 ** t)
        vh = vn / (1 - b2 ** t)
        out_p.append(pi - lr * (mh / (math.sqrt(vh) + eps) + wd * pi))
        out_m.append(mn)
        out_v.append(vn)
    return out_p, out_m, out_v


def test_against_python_loops_over_several_steps():
    rng = np.random.default_rng(0)
    p, m, v = rng.standard_normal(17), np.zeros(17), np.zeros(17)
    lp, lm, lv = p.tolist(), m.tolist(), v.tolist()
    for t in range(1, 6):
        g = rng.standard_normal(17)
        p, m, v = ao.adamw_step(p, g, m, v, lr=0.01, weight_decay=0.1, beta1=0.9, beta2=0.95, eps=1e-8, step=t)
        lp, lm, lv = py_adamw(lp, g.tolist(), lm, lv, 0.01, 0.1, 0.9, 0.95, 1e-8, t)
        assert np.max(np.abs(p - np.array(lp))) < 1e-15
        assert np.max(np.abs(m - np.array(lm))) < 1e-16 and np.max(np.abs(v - np.array(lv))) < 1e-16


def test_constant_gradient_closed_form():
    # with g constant and m0 = v0 = 0: m_t = (1 - b1^t) g, v_t = (1 - b2^t) g^2, so mhat = g and vhat = g^2 for
    # every t, and each step moves p by lr * (g / (|g| + eps) + wd * p)
    g = np.array([0.5, -2.0, 3.0, -1e-3])
    p = np.array([1.0, 2.0, -3.0, 4.0])
    m = np.zeros(4)
    v = np.zeros(4)
    ref = p.copy()
    for t in range(1, 8):
        p, m, v = ao.adamw_step(p, g, m, v, lr=0.1, weight_decay=0.05, beta1=0.9, beta2=0.95, eps=1e-8, step=t)
        ref = ref - 0.1 * (g / (np.abs(g) + 1e-8) + 0.05 * ref)
        assert np.max(np.abs(m - (1 - 0.9 ** t) * g)) < 1e-15
        assert np.max(np.abs(v - (1 - 0.95 ** t) * g * g)) < 1e-15
        assert np.max(np.abs(p - ref)) < 1e-13


def test_degenerate_settings():
    rng = np.random.default_rng(1)
    p, g = rng.standard_normal(9), rng.standard_normal(9)
    m, v = rng.standard_normal(9), rng.random(9)
    # lr = 0: parameters untouched, moments still advance
    pn, mn, vn = ao.adamw_step(p, g, m, v, lr=0.0, weight_decay=0.1, step=3)
    assert np.array_equal(pn, p) and not np.array_equal(mn, m) and not np.array_equal(vn, v)
    # zero gradient and zero state: pure decoupled decay, no NaN from 0 / (0 + eps)
    z = np.zeros(9)
    pn, mn, vn = ao.adamw_step(p, z, z, z, lr=0.5, weight_decay=0.1, step=1)
    assert np.allclose(pn, p * (1 - 0.05), rtol=0, atol=1e-15) and not mn.any() and not vn.any()
    # beta1 = beta2 = 0: sign-like update g / (|g| + eps)
    pn, _, _ = ao.adamw_step(p, g, m, v, lr=0.1, weight_decay=0.0, beta1=0.0, beta2=0.0, eps=1e-8, step=1)
    assert np.max(np.abs(pn - (p - 0.1 * g / (np.abs(g) + 1e-8)))) < 1e-15
    # weight decay multiplies the old parameter and is not divided by sqrt(vhat)
    a, _, _ = ao.adamw_step(p, g, m, v, lr=0.1, weight_decay=0.0, step=2)
    b, _, _ = ao.adamw_step(p, g, m, v, lr=0.1, weight_decay=0.3, step=2)
    assert np.max(np.abs((a - b) - 0.1 * 0.3 * p)) < 1e-15
    # inputs are widened, not modified
    p32 = p.astype(np.float32)
    keep = p32.copy()
    out = ao.adamw_step(p32, g, m, v, lr=0.1, weight_decay=0.1, step=1)
    assert out[0].dtype == np.float64 and np.array_equal(p32, keep)


def test_first_step_bias_correction():
    # t = 1: mhat = g, vhat = g^2 whatever the betas
    g = np.array([2.0, -0.25])
    p = np.array([1.0, 1.0])
    for b1, b2 in ((0.9, 0.999), (0.5, 0.5), (0.99, 0.95)):
        pn, _, _ = ao.adamw_step(p, g, np.zeros(2), np.zeros(2), lr=1.0, weight_decay=0.0, beta1=b1, beta2=b2, eps=0.0, step=1)
        assert np.max(np.abs(pn - (p - np.sign(g)))) < 1e-15
    with pytest.raises(ValueError):
        ao.adamw_step(p, g, np.zeros(2), np.zeros(2), lr=1.0, weight_decay=0.0, step=0)

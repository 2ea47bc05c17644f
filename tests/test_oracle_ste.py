"""Pins of the oracle's gradient through the weight / activation quantizer (clip mask on the
input, gradient of the learned clip value; Sec. 3.1 learns c end to end and prints no formula,
so the oracle's reading, the straight-through derivative of Eq. 1-4, is pinned against automatic
differentiation of Eq. 1-4 written with a straight-through rounding, against the published
step-size gradient of the learned-step-size quantizer the section cites, and against cases with
a closed form)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2407_12637_amd import synth


def _autograd(x, c, unsigned, bits, g):
    """d/dx and d/dc of sum(g * Q(x, c)) with Q = s * round_ste(clip(x, c) / s), fp64."""
    q = 2 ** bits - 1 if unsigned else 2 ** (bits - 1) - 1
    xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    ct = torch.tensor(float(c), dtype=torch.float64, requires_grad=True)
    lo = torch.zeros((), dtype=torch.float64) if unsigned else -ct
    s = ct / q
    u = torch.minimum(torch.maximum(xt, lo), ct) / s
    r = u + (torch.round(u) - u).detach()
    (torch.tensor(g, dtype=torch.float64) * (s * r)).sum().backward()
    return xt.grad.numpy(), float(ct.grad)


@pytest.mark.parametrize("unsigned", [False, True])
@pytest.mark.parametrize("bits", [2, 4, 5, 8])
def test_against_automatic_differentiation(unsigned, bits):
    r = synth.rng(0, 80, bits, int(unsigned))
    n = 4000
    x = synth.normal(r, (n,))
    g = synth.normal(r, (n,), 0.01)
    c = np.float32(1.3)
    q = 2 ** bits - 1 if unsigned else 2 ** (bits - 1) - 1
    # keep the pin away from rounding ties, where fp32 and fp64 u may round differently
    u = np.clip(x.astype(np.float64), 0.0 if unsigned else -float(c), float(c)) * q / float(c)
    keep = np.abs(u - np.floor(u) - 0.5) > 1e-4
    x, g = x[keep], g[keep]
    gx, gc, mag = oracle.ste_backward(x, c, unsigned, bits, g)
    want_gx, want_gc = _autograd(x, c, unsigned, bits, g)
    # (the chain rule multiplies by s and divides by s again: equal up to an ulp of fp64)
    assert np.array_equal(gx == 0, want_gx == 0)
    assert np.allclose(gx.astype(np.float64), want_gx, rtol=1e-14, atol=0.0)
    assert abs(gc - want_gc) <= 1e-6 * mag
    assert mag > 0 and (gx == 0).any() and (gx != 0).any()


def test_against_the_published_step_size_gradient():
    """Learned-step-size quantizer (Esser et al., cited by Sec. 3.1): dQ/ds = round(x/s) - x/s
    inside, -Q_N / +Q_P outside.  With s = c/q: dQ/dc = (dQ/ds)/q."""
    r = synth.rng(0, 81, 0, 0)
    x = synth.normal(r, (3000,))
    g = synth.normal(r, (3000,), 0.1)
    c, bits = np.float32(0.9), 4
    q = 7
    s = float(c) / q
    v = x.astype(np.float64) / s
    dqds = np.where(v <= -q, -q, np.where(v >= q, q, np.rint(v) - v))
    want = float(np.sum(g.astype(np.float64) * dqds / q))
    _, gc, mag = oracle.ste_backward(x, c, False, bits, g)
    assert abs(gc - want) <= 1e-5 * mag     # u in fp32 against v in fp64


def test_closed_forms():
    # inputs on the quantization grid: the inside term vanishes, the clipped ones count +-g
    c, bits = np.float32(3.5), 4                  # s = 0.5 exactly
    k = np.arange(-12, 13)
    x = (k * 0.5).astype(np.float32)
    g = np.linspace(0.1, 2.5, x.size).astype(np.float32)
    gx, gc, _ = oracle.ste_backward(x, c, False, bits, g)
    want_c = float(g[k >= 7].astype(np.float64).sum() - g[k <= -7].astype(np.float64).sum())
    assert gc == pytest.approx(want_c, rel=1e-15)
    assert np.array_equal(gx, np.where(np.abs(k) < 7, g, 0).astype(np.float32))
    # unsigned: values at or below zero contribute nothing to either gradient
    gx, gc, _ = oracle.ste_backward(x, np.float32(7.5), True, 4, g)    # s = 0.5, q = 15
    assert gc == 0.0 and np.array_equal(gx, np.where(k > 0, g, 0).astype(np.float32))
    gx, gc, _ = oracle.ste_backward(x, np.float32(3.0), True, 4, g)    # s = 0.2: x >= 3 clipped
    inside = (x > 0) & (x < 3.0)
    assert np.array_equal(gx, np.where(inside, g, 0).astype(np.float32))
    # a half-step offset inside: round(u) - u = -+1/2 alternately (ties to even), over q
    x = np.array([0.25, 0.75, -0.25, -0.75], np.float32)               # u = 0.5, 1.5, -0.5, -1.5
    g = np.array([1.0, 2.0, 4.0, 8.0], np.float32)
    _, gc, _ = oracle.ste_backward(x, np.float32(3.5), False, 4, g)
    assert gc == pytest.approx((1.0 * -0.5 + 2.0 * 0.5 + 4.0 * 0.5 + 8.0 * -0.5) / 7, rel=1e-15)


def test_invariance_under_power_of_two_scaling():
    r = synth.rng(0, 82, 0, 0)
    x = synth.normal(r, (5000,))
    g = synth.normal(r, (5000,))
    a = oracle.ste_backward(x, np.float32(1.1), False, 5, g)
    b = oracle.ste_backward(x * np.float32(64), np.float32(1.1) * np.float32(64), False, 5, g)
    assert np.array_equal(a[0], b[0]) and a[1] == b[1]


def test_error_bound_of_the_inside_term():
    # |round(u) - u| <= 1/2: the gradient of c is bounded by sum|g| (1/(2q) inside, 1 outside)
    r = synth.rng(0, 83, 0, 0)
    x = synth.normal(r, (5000,))
    g = np.abs(synth.normal(r, (5000,)))
    for bits in (2, 4, 8):
        c = np.float32(0.8)
        q = 2 ** (bits - 1) - 1
        _, gc, mag = oracle.ste_backward(x, c, False, bits, g)
        inside = np.abs(x) < c
        bound = g[inside].sum(dtype=np.float64) / (2 * q) + g[~inside].sum(dtype=np.float64)
        assert mag <= bound * (1 + 1e-6) and abs(gc) <= mag

"""GPU parity of the gradient through the weight / activation quantizer (clip mask on the
input, gradient of the learned clip value; Sec. 3.1) against the oracle: grad_x bit for bit
(each element is the incoming gradient or 0), grad_c within 1e-6 of the oracle's fp64 sum plus
1e-9 of the sum of magnitudes (both sides add fp64 products, in different orders)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2407_12637_amd import binding as lbt
from paper_2407_12637_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)


def _run(x, c, unsigned, bits, g, in_place=False, want_c=True, want_x=True):
    n = x.size
    xd, gd = gu.dev(x.reshape(-1)), gu.dev(g.reshape(-1))
    ws = torch.zeros(lbt.lbt_workspace_bytes_quantize(n), dtype=torch.uint8, device=gu.DEV)
    gx = gd if in_place else (torch.full((n,), float("nan"), device=gu.DEV) if want_x else None)
    gc = torch.full((1,), float("nan"), device=gu.DEV) if want_c else None
    lbt.lbt_ste_backward(xd, float(c), unsigned, bits, gd, gx, gc, ws)
    return (None if gx is None else gx.cpu().numpy().reshape(x.shape),
            None if gc is None else float(gc.item()))


def _check(x, c, unsigned, bits, g, **kw):
    want_x, want_c, mag = oracle.ste_backward(x, c, unsigned, bits, g)
    got_x, got_c = _run(x, c, unsigned, bits, g, **kw)
    if got_x is not None:
        assert np.array_equal(got_x, want_x), "grad_x differs"
    if got_c is not None:
        assert abs(got_c - want_c) <= 1e-6 * abs(want_c) + 1e-9 * mag, (got_c, want_c, mag)
    return want_c, mag


@pytest.mark.parametrize("n", [1, 3, 7, 1000, 65537, 3 * 1024 * 1024 + 5])
@pytest.mark.parametrize("unsigned", [False, True])
def test_sizes(n, unsigned):
    _say("ste", n, unsigned)
    r = synth.rng(0, 90, n % 97, int(unsigned))
    x = synth.normal(r, (n,))
    g = synth.normal(r, (n,), 0.01)
    for bits, c in ((4, 1.3), (2, 0.4), (8, 2.5)):
        if unsigned and bits == 8:
            continue
        want_c, mag = _check(x, np.float32(c), unsigned, bits, g)
        if n >= 1000:
            assert mag > 0 and want_c != 0.0


def test_in_place_and_optional_outputs():
    r = synth.rng(0, 91, 0, 0)
    x = synth.normal(r, (200003,))
    g = synth.normal(r, (200003,))
    _check(x, np.float32(0.7), False, 4, g, in_place=True)
    _check(x, np.float32(0.7), False, 4, g, want_c=False)
    _check(x, np.float32(0.7), True, 4, g, want_x=False)


def test_same_inputs_same_bits():
    r = synth.rng(0, 92, 0, 0)
    x = synth.normal(r, (1 << 22,))
    g = synth.normal(r, (1 << 22,))
    a = _run(x, np.float32(1.1), False, 4, g)
    b = _run(x, np.float32(1.1), False, 4, g)
    assert a[1] == b[1] and np.array_equal(a[0], b[0])


def test_boundaries_and_nonfinite():
    c = np.float32(3.5)
    x = np.array([3.5, -3.5, 0.0, 3.4999998, -3.4999998, 10.0, -10.0, np.inf, -np.inf, np.nan,
                  0.25, 0.75], np.float32)
    g = np.arange(1, x.size + 1).astype(np.float32)
    for unsigned in (False, True):
        want_x, want_c, _ = oracle.ste_backward(x, c, unsigned, 4, g)
        got_x, got_c = _run(x, c, unsigned, 4, g)
        assert np.array_equal(got_x, want_x)
        assert got_c == pytest.approx(want_c, rel=1e-6)
        assert got_x[0] == 0 and got_x[9] == 0        # x == c and NaN are outside the interval


def test_after_a_backward_call():
    """The use it is for: dW of the layer is dL/dQ(W); its mask and the gradient of c_w follow."""
    N, Cc, H, W, K, R, S, stride, pad = 8, 32, 14, 14, 64, 3, 3, 1, 1
    r = synth.rng(0, 93, 0, 0)
    X, Wt = synth.relu_normal(r, (N, Cc, H, W)), synth.kaiming_normal(r, (K, Cc, R, S))
    dY = synth.dense_grad(r, (N, K, H, W))
    c_x, c_w = 1.8, 0.12
    st = lbt.new_state(gamma0=0.8)
    ost = oracle.GradState(gamma=0.8)
    ref = oracle.backward_conv2d(X, Wt, dY, stride, pad, ost, c_x=c_x, c_w=c_w, seed=3, rounding=1)
    res = gu.backward_conv2d(X, Wt, dY, stride, pad, st, c_x=c_x, c_w=c_w, seed=3, rounding=1)
    assert np.array_equal(res.acc_dw, ref.acc_dw) and np.array_equal(res.acc_dx, ref.acc_dx)
    # the GPU's own dW / dX go in (equal to the oracle's within 1e-5; the masks do not depend on them)
    for x, c, unsigned, grad in ((Wt, c_w, False, res.dW), (X, c_x, True, res.dX)):
        want_x, want_c, mag = oracle.ste_backward(x, np.float32(c), unsigned, 4, grad)
        got_x, got_c = _run(x, np.float32(c), unsigned, 4, grad, in_place=True)
        assert np.array_equal(got_x, want_x)
        assert abs(got_c - want_c) <= 1e-6 * abs(want_c) + 1e-9 * mag
        assert mag > 0 and (got_x == 0).any() and (got_x != 0).any()


def test_full_size_activation_tensor():
    """The largest activation tensor of the ResNet-50 sweep (51.4 M elements) in place."""
    L = [x for x in synth.resnet50_layers(64) if x.name == "l1.1x1.256-64@56"][0]
    _say("ste full-size", L.name)
    r = synth.rng(0, 94, 0, 0)
    X = synth.relu_normal(r, L.x_shape)
    g = synth.normal(r, L.x_shape, 1e-3)
    _check(X, np.float32(2.0), True, 4, g, in_place=True)


def test_refusals():
    x = gu.dev(np.ones(64, np.float32))
    ws = torch.zeros(lbt.lbt_workspace_bytes_quantize(64), dtype=torch.uint8, device=gu.DEV)
    for c in (0.0, -1.0, float("inf"), float("nan")):
        with pytest.raises(lbt.LbtError) as e:
            lbt.lbt_ste_backward(x, c, False, 4, x, None, None, ws)
        assert e.value.code == -3
    with pytest.raises(lbt.LbtError):
        lbt.lbt_ste_backward(x, 1.0, False, 9, x, None, None, ws)

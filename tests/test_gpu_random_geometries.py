"""Seeded random convolution and linear geometries through the backward and forward calls
against the oracle: odd sizes, channel counts that are not multiples of the 16-code granule,
non-square images and filters, strides 1-3, paddings up to the filter size minus one.  Integer
sums bit for bit, fp32 outputs within 1e-5, state equal."""
import numpy as np
import pytest

import oracle
from paper_2407_12637_amd import binding as lbt
from paper_2407_12637_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu


def _geometries(n, seed):
    r = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        R, S = int(r.integers(1, 6)), int(r.integers(1, 6))
        if r.random() < 0.15:
            R = S = 7
        stride = int(r.choice([1, 1, 2, 3]))
        pad = int(r.integers(0, max(R, S)))
        H, W = int(r.integers(1, 19)), int(r.integers(1, 19))
        if H + 2 * pad < R or W + 2 * pad < S:
            continue
        N = int(r.choice([1, 2, 3, 5, 16, 17, 33]))
        C = int(r.choice([1, 3, 8, 15, 16, 17, 40, 64, 130]))
        K = int(r.choice([1, 2, 7, 16, 24, 33, 64, 150]))
        P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
        # keep the oracle's seven loops in the second range
        if N * K * P * Q * C * R * S > 6e7:
            continue
        out.append((N, C, H, W, K, R, S, stride, pad))
    return out


GEOMS = _geometries(40, 20240712)


def _check_backward(res, ref):
    assert np.array_equal(res.acc_dx, ref.acc_dx), "dX int32 accumulators differ"
    assert np.array_equal(res.acc_dw, ref.acc_dw), "dW int32 accumulators differ"
    gu.assert_outputs_close(res.dX, ref.dX)
    gu.assert_outputs_close(res.dW, ref.dW)


@pytest.mark.parametrize("idx", range(len(GEOMS)))
def test_random_conv_geometry(idx):
    N, C, H, W, K, R, S, stride, pad = GEOMS[idx]
    print("random conv", idx, GEOMS[idx], flush=True)
    r = synth.rng(0, 96, idx, 0)
    x_unsigned = bool(idx % 2)
    X = synth.relu_normal(r, (N, C, H, W)) if x_unsigned else synth.normal(r, (N, C, H, W))
    Wt = synth.kaiming_normal(r, (K, C, R, S))
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    dY = synth.dense_grad(r, (N, K, P, Q))
    rounding = idx % 2
    hs = lbt.HINDSIGHT_MAX if idx % 5 == 0 else 0
    st = lbt.new_state(gamma0=0.7)
    ost = oracle.GradState(gamma=0.7)
    for it in range(2):      # the second call matters in the single-sweep mode
        ref = oracle.backward_conv2d(X, Wt, dY, stride, pad, ost, x_unsigned=x_unsigned, seed=idx,
                                     rounding=rounding, hindsight=bool(hs))
        oracle.update_interval(ost)
        res = gu.backward_conv2d(X, Wt, dY, stride, pad, st, x_unsigned=x_unsigned, seed=idx,
                                 rounding=rounding | hs | lbt.FUSED_UPDATE)
        gu.assert_state_equal(lbt.lbt_state_read(st), ost)
        _check_backward(res, ref)
    # forward product that keeps the codes, and the backward call that reads them
    fwd_ref = oracle.forward_conv2d(X, Wt, stride, pad, x_unsigned=x_unsigned)
    fwd, saved = gu.save_conv2d(X, Wt, stride, pad, x_unsigned=x_unsigned)
    assert np.array_equal(fwd.acc, fwd_ref.acc), "forward int32 sums differ"
    gu.assert_outputs_close(fwd.Y, fwd_ref.Y)
    ref = oracle.backward_conv2d(X, Wt, dY, stride, pad, ost, x_unsigned=x_unsigned, seed=idx,
                                 rounding=rounding, hindsight=bool(hs))
    res = gu.backward_conv2d_saved(saved, X.shape, Wt.shape, dY, stride, pad, st,
                                   x_unsigned=x_unsigned, seed=idx, rounding=rounding | hs)
    gu.assert_state_equal(lbt.lbt_state_read(st), ost)
    _check_backward(res, ref)


@pytest.mark.parametrize("idx", range(0, len(GEOMS), 2))
def test_random_conv_geometry_other_bits_and_learned_clips(idx):
    """Every second geometry again at b = 5, 6 or 8 through lbt_backward_conv2d_learned (given clip
    values, masks and clip-value gradients) against the oracle's backward pass and ste_backward."""
    import torch
    N, C, H, W, K, R, S, stride, pad = GEOMS[idx]
    bits = (5, 6, 8)[(idx // 2) % 3]
    x_unsigned = bits < 8 and bool(idx % 4)
    print("random conv learned", idx, GEOMS[idx], bits, flush=True)
    r = synth.rng(0, 103, idx, 0)
    X = synth.relu_normal(r, (N, C, H, W)) if x_unsigned else synth.normal(r, (N, C, H, W))
    Wt = synth.kaiming_normal(r, (K, C, R, S))
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    dY = synth.dense_grad(r, (N, K, P, Q))
    c_x, c_w = 1.1, float(np.abs(Wt).max() * 0.7)
    st = lbt.new_state(gamma0=0.6, bits=bits)
    ost = oracle.GradState(gamma=0.6, bits=bits)
    ref = oracle.backward_conv2d(X, Wt, dY, stride, pad, ost, c_x=c_x, x_unsigned=x_unsigned, c_w=c_w,
                                 seed=idx, rounding=1)
    want_dw, want_cw, mag_w = oracle.ste_backward(Wt, np.float32(c_w), False, bits, ref.dW)
    want_dx, want_cx, mag_x = oracle.ste_backward(X, np.float32(c_x), x_unsigned, bits, ref.dX)
    ws = torch.zeros(lbt.lbt_workspace_bytes_conv2d(N, C, H, W, K, R, S, stride, pad),
                     dtype=torch.uint8, device=gu.DEV)
    dX = torch.full(X.shape, float("nan"), device=gu.DEV)
    dW = torch.full(Wt.shape, float("nan"), device=gu.DEV)
    gc = torch.full((2,), float("nan"), device=gu.DEV)
    lbt.lbt_backward_conv2d_learned(gu.dev(X), gu.dev(Wt), gu.dev(dY), N, C, H, W, K, R, S, stride,
                                    pad, c_x, x_unsigned, c_w, st, idx, 1 | lbt.BITS(bits), dX, dW, gc,
                                    ws)
    gu.assert_state_equal(lbt.lbt_state_read(st), ost)
    got_dx, got_dw, got_c = dX.cpu().numpy(), dW.cpu().numpy(), gc.cpu().numpy().astype(np.float64)
    assert np.array_equal(got_dx == 0, want_dx == 0) and np.array_equal(got_dw == 0, want_dw == 0)
    gu.assert_outputs_close(got_dx, want_dx)
    gu.assert_outputs_close(got_dw, want_dw)
    assert abs(got_c[0] - want_cw) <= 1e-5 * abs(want_cw) + 1e-6 * mag_w
    assert abs(got_c[1] - want_cx) <= 1e-5 * abs(want_cx) + 1e-6 * mag_x


def _linear_shapes(n, seed):
    r = np.random.default_rng(seed)
    return [(int(r.integers(1, 300)), int(r.integers(1, 300)), int(r.integers(1, 300)))
            for _ in range(n)]


LINEAR = _linear_shapes(16, 77)


@pytest.mark.parametrize("idx", range(len(LINEAR)))
def test_random_linear_shape(idx):
    M, K, N = LINEAR[idx]
    print("random linear", idx, LINEAR[idx], flush=True)
    r = synth.rng(0, 97, idx, 0)
    X, W = synth.normal(r, (M, K)), synth.normal(r, (K, N), 0.05)
    dY = synth.dense_grad(r, (M, N))
    st = lbt.new_state(gamma0=0.8)
    ost = oracle.GradState(gamma=0.8)
    ref = oracle.backward_linear(X, W, dY, ost, seed=idx, rounding=1)
    res = gu.backward_linear(X, W, dY, st, seed=idx, rounding=1)
    gu.assert_state_equal(lbt.lbt_state_read(st), ost)
    _check_backward(res, ref)
    fwd_ref = oracle.forward_linear(X, W)
    fwd = gu.forward_linear(X, W)
    assert np.array_equal(fwd.acc, fwd_ref.acc)
    gu.assert_outputs_close(fwd.Y, fwd_ref.Y)

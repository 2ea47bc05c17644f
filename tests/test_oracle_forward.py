"""Pins of the oracle's quantized forward pass (Sec. 3.1: Q(X), Q(W) before the product;
Eq. 4 afterwards) against things other than itself: a direct six-loop sum, torch's fp64
convolution (exact on small integers), the matrix-product special case, and the adjoint
identities that tie it to the already pinned dX / dW contractions."""
import itertools

import numpy as np
import pytest
import torch

import oracle
from paper_2407_12637_amd import synth

CASES = [
    # N, C, H, W, K, R, S, stride, pad
    (2, 3, 5, 6, 4, 3, 3, 1, 1),
    (1, 2, 7, 8, 3, 3, 3, 2, 0),
    (2, 4, 9, 7, 5, 1, 1, 2, 0),
    (2, 3, 8, 8, 2, 5, 3, 2, 2),
    (3, 5, 6, 6, 4, 1, 1, 1, 0),
]


def _codes(case, seed=0):
    N, C, H, W, K, R, S, stride, pad = case
    r = np.random.default_rng(seed)
    qX = r.integers(0, 16, (N, C, H, W)).astype(np.int32)
    qW = r.integers(-7, 8, (K, C, R, S)).astype(np.int32)
    return qX, qW


def _six_loops(qX, qW, stride, pad):
    N, C, H, W = qX.shape
    K, _, R, S = qW.shape
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    out = np.zeros((N, K, P, Q), dtype=np.int64)
    for n, k, p, q in itertools.product(range(N), range(K), range(P), range(Q)):
        t = 0
        for c, r, s in itertools.product(range(C), range(R), range(S)):
            h, w = p * stride - pad + r, q * stride - pad + s
            if 0 <= h < H and 0 <= w < W:
                t += int(qW[k, c, r, s]) * int(qX[n, c, h, w])
        out[n, k, p, q] = t
    return out


@pytest.mark.parametrize("case", CASES)
def test_conv_fwd_equals_direct_sum_and_torch(case):
    stride, pad = case[-2:]
    qX, qW = _codes(case)
    acc = oracle.conv2d_fwd(qX, qW, stride, pad)
    assert np.array_equal(acc, _six_loops(qX, qW, stride, pad))
    ref = torch.nn.functional.conv2d(torch.from_numpy(qX).double(), torch.from_numpy(qW).double(),
                                     stride=stride, padding=pad)
    assert np.array_equal(acc, ref.numpy().astype(np.int64))      # small integers: fp64 is exact
    idx = np.arange(acc.size)
    assert np.array_equal(oracle.conv2d_fwd_at(qX, qW, stride, pad, idx), acc.reshape(-1))


@pytest.mark.parametrize("case", CASES)
def test_conv_fwd_is_the_adjoint_of_dx_and_dw(case):
    # <conv(x, w), g> = <x, dX(g, w)> = <w, dW(g, x)>, exactly, in integers
    stride, pad = case[-2:]
    qX, qW = _codes(case, 1)
    acc = oracle.conv2d_fwd(qX, qW, stride, pad)
    qG = np.random.default_rng(2).integers(-7, 8, acc.shape).astype(np.int32)
    lhs = int((acc * qG).sum())
    dx = oracle.conv2d_dx(qG, qW, qX.shape, stride, pad)
    dw = oracle.conv2d_dw(qG, qX, qW.shape, stride, pad)
    assert lhs == int((dx * qX).sum()) == int((dw * qW).sum())


def test_linear_fwd_special_cases():
    r = np.random.default_rng(3)
    qX = r.integers(-7, 8, (13, 21)).astype(np.int32)
    qW = r.integers(-7, 8, (21, 9)).astype(np.int32)
    acc = oracle.linear_fwd(qX, qW)
    loops = np.array([[sum(int(qX[m, k]) * int(qW[k, n]) for k in range(21)) for n in range(9)]
                      for m in range(13)])
    assert np.array_equal(acc, loops)
    # Y = X W is the dX product with the roles of the operands exchanged
    assert np.array_equal(acc, oracle.linear_dx(qX, np.ascontiguousarray(qW.T)))
    # a 1x1 convolution on a 1x1 image is the same product
    conv = oracle.conv2d_fwd(qX[:, :, None, None], np.ascontiguousarray(qW.T)[:, :, None, None], 1, 0)
    assert np.array_equal(conv[:, :, 0, 0], acc)


def test_forward_layer_on_exactly_representable_inputs():
    # inputs that already sit on the quantizer's grid (multiples of the scale) pass through
    # Q unchanged, so the quantized layer equals the float layer on them
    r = np.random.default_rng(4)
    s_x, s_w = 2.0 ** -3, 2.0 ** -5
    X = (r.integers(0, 16, (2, 3, 6, 6)) * s_x).astype(np.float32)
    W = (r.integers(-7, 8, (4, 3, 3, 3)) * s_w).astype(np.float32)
    res = oracle.forward_conv2d(X, W, 1, 1, c_x=15 * s_x, x_unsigned=True, c_w=7 * s_w)
    assert res.status == oracle.OK and res.s_x == s_x and res.s_w == s_w
    ref = torch.nn.functional.conv2d(torch.from_numpy(X).double(), torch.from_numpy(W).double(),
                                     padding=1).numpy()
    assert np.array_equal(res.Y.astype(np.float64), ref)
    Xl = (r.integers(-7, 8, (5, 8)) * s_x).astype(np.float32)
    Wl = (r.integers(-7, 8, (8, 6)) * s_w).astype(np.float32)
    lin = oracle.forward_linear(Xl, Wl, c_x=7 * s_x, c_w=7 * s_w)
    assert np.array_equal(lin.Y.astype(np.float64), Xl.astype(np.float64) @ Wl.astype(np.float64))


def test_forward_layer_error_is_bounded_by_the_half_steps():
    # |Y - Y_float| <= sum over the window of (|x| s_w/2 + |w| s_x/2 + s_x s_w/4), inside the clips
    r = synth.rng(0, 95, 0, 0)
    X = np.clip(synth.relu_normal(r, (2, 8, 10, 10)), 0, 2.0).astype(np.float32)
    W = np.clip(synth.kaiming_normal(r, (6, 8, 3, 3)), -0.3, 0.3).astype(np.float32)
    res = oracle.forward_conv2d(X, W, 1, 1, c_x=2.0, x_unsigned=True, c_w=0.3)
    tx, tw = torch.from_numpy(X).double(), torch.from_numpy(W).double()
    ref = torch.nn.functional.conv2d(tx, tw, padding=1).numpy()
    hx, hw = res.s_x / 2, res.s_w / 2
    bound = (torch.nn.functional.conv2d(tx.abs(), torch.full_like(tw, hw), padding=1)
             + torch.nn.functional.conv2d(torch.full_like(tx, hx), tw.abs(), padding=1)
             + torch.nn.functional.conv2d(torch.full_like(tx, hx), torch.full_like(tw, hw), padding=1)).numpy()
    assert np.all(np.abs(res.Y - ref) <= bound * (1 + 1e-4) + 1e-6)
    assert np.abs(res.Y - ref).max() > 0


def test_forward_reports_nonfinite_operand():
    X = np.ones((2, 2, 3, 3), np.float32)
    W = np.ones((2, 2, 1, 1), np.float32)
    X[0, 0, 0, 0] = np.inf
    res = oracle.forward_conv2d(X, W, 1, 0)
    assert res.status == oracle.NONFINITE and res.Y is None

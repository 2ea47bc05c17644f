"""GPU parity of the single-sweep mode (LBT_HINDSIGHT_MAX): the interval of a gradient tensor
comes from the maximum of the layer's previous gradient tensor, and the tensor is read once.
An explicitly requested extra mode, not the quantizer of Sec. 3.1; the oracle's hindsight
variant is the definition.  Codes, statistics, the recorded maximum and the int32
accumulators must match bit for bit."""
import numpy as np
import pytest

import oracle
from paper_2407_12637_amd import binding as lbt
from paper_2407_12637_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu

HS = lbt.HINDSIGHT_MAX


def _say(*a):
    print(*a, flush=True)


def _check_backward(res, ref):
    if ref.acc_dx is not None:
        assert np.array_equal(res.acc_dx, ref.acc_dx), "dX int32 accumulators differ"
        gu.assert_outputs_close(res.dX, ref.dX)
    if ref.acc_dw is not None:
        assert np.array_equal(res.acc_dw, ref.acc_dw), "dW int32 accumulators differ"
        gu.assert_outputs_close(res.dW, ref.dW)


@pytest.mark.parametrize("n", [1, 9, 1000, 65537, 3 * 1024 * 1024 + 5])
@pytest.mark.parametrize("rounding", [0, 1])
def test_flat_sequence(n, rounding):
    """Fresh state (no previous maximum), then tensors of changing magnitude, with the
    interval update between the calls."""
    _say("hindsight flat", n, rounding)
    r = synth.rng(0, 30, n % 89, synth.T_DY)
    st = lbt.new_state(gamma0=0.6)
    ost = oracle.GradState(gamma=0.6)
    for it, mag in enumerate((1.0, 0.5, 3.0, 0.9)):
        g = (synth.grad_cfg4(r, (n,)) * np.float32(mag)).astype(np.float32)
        want = oracle.quantize_grad(g, ost, seed=77, rounding=rounding, hindsight=True)
        packed = gu.quantize_grad(g, st, seed=77, rounding=rounding | HS)
        h = lbt.lbt_state_read(st)
        gu.assert_state_equal(h, ost)
        assert h.sync_word == 0 and h.sync_max == 0
        if it == 0:
            assert h.status == lbt.STATUS_ZERO_GRAD and not packed.any()
        assert np.array_equal(packed, oracle.pack_nibbles(want))
        oracle.update_interval(ost)
        lbt.lbt_update_interval(st)
        assert lbt.lbt_state_read(st).gamma == ost.gamma


def test_flat_mixes_with_two_sweep_calls_and_nonfinite():
    n = 200003
    r = synth.rng(0, 31, 0, synth.T_DY)
    g1, g2, g3 = (synth.dense_grad(r, (n,)) for _ in range(3))
    st = lbt.new_state(gamma0=0.4)
    ost = oracle.GradState(gamma=0.4)
    # a two-sweep call leaves its maximum for the single-sweep call that follows
    gu.quantize_grad(g1, st, seed=5, rounding=1)
    oracle.quantize_grad(g1, ost, seed=5, rounding=1)
    want = oracle.quantize_grad(g2 * np.float32(0.25), ost, seed=5, rounding=1, hindsight=True)
    packed = gu.quantize_grad(g2 * np.float32(0.25), st, seed=5, rounding=1 | HS)
    gu.assert_state_equal(lbt.lbt_state_read(st), ost)
    assert np.array_equal(packed, oracle.pack_nibbles(want))
    # a non-finite value: reported, and the recorded maximum is kept
    kept = lbt.lbt_state_read(st).gmax
    for bad in (np.nan, -np.inf):
        gb = g3.copy()
        gb[n - 2] = bad
        oracle.quantize_grad(gb, ost, seed=5, rounding=0, hindsight=True)
        gu.quantize_grad(gb, st, seed=5, rounding=0 | HS)
        h = lbt.lbt_state_read(st)
        assert h.status == lbt.STATUS_NONFINITE == ost.status
        assert h.gmax == kept == ost.gmax and h.sync_word == 0 and h.sync_max == 0
    # the next finite tensor is quantized with the kept maximum
    want = oracle.quantize_grad(g3, ost, seed=6, rounding=0, hindsight=True)
    packed = gu.quantize_grad(g3, st, seed=6, rounding=0 | HS)
    gu.assert_state_equal(lbt.lbt_state_read(st), ost)
    assert np.array_equal(packed, oracle.pack_nibbles(want))
    # all-zero tensor: codes 0, recorded maximum 0, so the call after it reports ZERO_GRAD
    z = np.zeros(n, np.float32)
    for g in (z, g1):
        want = oracle.quantize_grad(g, ost, seed=6, rounding=0, hindsight=True)
        packed = gu.quantize_grad(g, st, seed=6, rounding=0 | HS)
        gu.assert_state_equal(lbt.lbt_state_read(st), ost)
        assert np.array_equal(packed, oracle.pack_nibbles(want))
    assert ost.status == oracle.ZERO_GRAD


CONV_CASES = [
    # N, C, H, W, K, R, S, stride, pad           tile kind of dY in the re-layout
    (16, 16, 32, 32, 16, 3, 3, 1, 1),          # windowed (P*Q = 1024)
    (8, 64, 14, 14, 160, 1, 1, 1, 0),          # whole row (P*Q = 196)
    (3, 5, 9, 7, 6, 3, 3, 2, 1),               # generic tile
    (20, 32, 12, 12, 48, 3, 3, 2, 1),          # whole row, ragged batch
    (64, 8, 1, 1, 24, 1, 1, 1, 0),             # P*Q = 1: matrix tiles
    (7, 8, 1, 1, 5, 1, 1, 1, 0),               # P*Q = 1, K % 8 != 0: generic column
]


@pytest.mark.parametrize("case", CONV_CASES)
@pytest.mark.parametrize("rounding", [0, 1])
def test_backward_conv2d_sequence(case, rounding):
    N, Cc, H, W, K, R, S, stride, pad = case
    _say("hindsight conv", case, rounding)
    r = synth.rng(0, 32, Cc * 131 + K, 0)
    X, Wt = synth.relu_normal(r, (N, Cc, H, W)), synth.kaiming_normal(r, (K, Cc, R, S))
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    st = lbt.new_state(gamma0=0.5)
    ost = oracle.GradState(gamma=0.5)
    for it, (dist, mag) in enumerate(((synth.dense_grad, 1.0), (synth.grad_cfg2, 1.0),
                                      (synth.dense_grad, 0.3))):
        dY = (dist(r, (N, K, P, Q)) * np.float32(mag)).astype(np.float32)
        ref = oracle.backward_conv2d(X, Wt, dY, stride, pad, ost, x_unsigned=True, seed=3,
                                     rounding=rounding, hindsight=True)
        res = gu.backward_conv2d(X, Wt, dY, stride, pad, st, x_unsigned=True, seed=3,
                                 rounding=rounding | HS)
        gu.assert_state_equal(lbt.lbt_state_read(st), ost)
        _check_backward(res, ref)
        if it == 0:
            assert not res.dX.any() and not res.dW.any()
        oracle.update_interval(ost)
        lbt.lbt_update_interval(st)


@pytest.mark.parametrize("shape", [(3, 5, 7), (130, 72, 200), (257, 129, 33)])
def test_backward_linear_sequence(shape):
    M, K, N = shape
    _say("hindsight linear", shape)
    r = synth.rng(0, 33, M, 0)
    X, W = synth.normal(r, (M, K)), synth.normal(r, (K, N), 0.05)
    st = lbt.new_state(gamma0=0.8)
    ost = oracle.GradState(gamma=0.8)
    for mag in (1.0, 2.0, 0.5):
        dY = (synth.dense_grad(r, (M, N)) * np.float32(mag)).astype(np.float32)
        # clip values given for X and W: no tensor is left for the maximum kernel
        ref = oracle.backward_linear(X, W, dY, ost, c_x=2.0, c_w=0.08, seed=9, rounding=1,
                                     hindsight=True)
        res = gu.backward_linear(X, W, dY, st, c_x=2.0, c_w=0.08, seed=9, rounding=1 | HS)
        gu.assert_state_equal(lbt.lbt_state_read(st), ost)
        _check_backward(res, ref)


def test_rejects_unknown_rounding_bits():
    g = gu.dev(np.ones(64, np.float32))
    st = lbt.new_state()
    import torch
    codes = torch.zeros(32, dtype=torch.uint8, device=gu.DEV)
    ws = torch.zeros(lbt.lbt_workspace_bytes_quantize(64), dtype=torch.uint8, device=gu.DEV)
    with pytest.raises(lbt.LbtError):
        lbt.lbt_quantize_grad(g, st, 0, 8, codes, ws)


def test_full_size_layer_single_sweep():
    """The largest gradient tensor of the ResNet-50 sweep (51.4 M elements): a two-sweep call records the maximum, the single-sweep call after it is checked in
    full on the statistics and on sampled outputs of both products."""
    L = [x for x in synth.resnet50_layers(64) if x.name == "l1.1x1.64-256@56"][0]
    _say("hindsight full-size", L.name)
    r = synth.rng(0, 34, 0, 0)
    X = synth.relu_normal(r, L.x_shape)
    W = synth.kaiming_normal(r, L.w_shape)
    dY1 = synth.grad_cfg4(r, L.dy_shape)
    dY2 = (synth.grad_cfg4(r, L.dy_shape) * np.float32(0.7)).astype(np.float32)
    st = lbt.new_state(gamma0=0.01)
    ost = oracle.GradState(gamma=0.01)
    gu.backward_conv2d(X, W, dY1, L.stride, L.pad, st, seed=21, rounding=1, with_acc=False)
    oracle.quantize_grad(dY1, ost, 21, 1)
    gu.assert_state_equal(lbt.lbt_state_read(st), ost)
    lbt.lbt_update_interval(st)
    oracle.update_interval(ost)
    res = gu.backward_conv2d(X, W, dY2, L.stride, L.pad, st, seed=21, rounding=1 | HS)
    qG = oracle.quantize_grad(dY2, ost, 21, 1, hindsight=True)
    gu.assert_state_equal(lbt.lbt_state_read(st), ost)
    assert ost.status == oracle.OK and ost.n_out > 0
    qX, c_x, s_x, _ = oracle.quantize_operand(X, 0.0, True)
    qW, c_w, s_w, _ = oracle.quantize_operand(W, 0.0, False)
    s_g = oracle.scale(ost.clip, 4)
    pick = np.random.default_rng(8)
    n_dx = int(np.prod(L.x_shape))
    ix = np.unique(np.concatenate([pick.integers(0, n_dx, 2000), [0, n_dx - 1]]))
    want_dx = oracle.conv2d_dx_at(qG, qW, L.x_shape, L.stride, L.pad, ix)
    assert np.array_equal(res.acc_dx.reshape(-1)[ix], want_dx), "dX accumulators differ"
    gu.assert_outputs_close(res.dX.reshape(-1)[ix], oracle.dequant(want_dx, s_g, s_w))
    n_dw = int(np.prod(L.w_shape))
    iw = np.unique(np.concatenate([pick.integers(0, n_dw, 100), [0, n_dw - 1]]))
    want_dw = oracle.conv2d_dw_at(qG, qX, L.w_shape, L.stride, L.pad, iw)
    assert np.array_equal(res.acc_dw.reshape(-1)[iw], want_dw), "dW accumulators differ"
    gu.assert_outputs_close(res.dW.reshape(-1)[iw], oracle.dequant(want_dw, s_x, s_g))
    assert np.abs(want_dx).max() > 0 and np.abs(want_dw).max() > 0

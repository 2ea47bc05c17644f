"""GPU parity at the full layer sizes the benchmark times (ResNet-50 at batch 64, plus one
ResNet-18 stem and one super-resolution layer), through the same entry points.

The oracle computes what it can in full (maximum, clip value, clip-out count, gamma
after the update: all O(n)), and the contractions on sampled output positions, one by
one, from the oracle's own codes.  Everything integer is compared bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2407_12637_amd import binding as lbt
from paper_2407_12637_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu


def _layer(name, table):
    return [L for L in table if L.name == name][0]


R50 = synth.resnet50_layers(64)
CASES = [
    # (layer, gradient recipe, gamma0, rounding)
    (_layer("l1.3x3.64-64@56", R50), "t25", 1.0, 1),
    (_layer("l1.1x1.64-256@56", R50), "t25", 0.01, 1),        # 51.4 M gradients, dense codes
    (_layer("l2.3x3s2.128-128@56", R50), "dense", 1.0, 0),     # stride 2
    (_layer("l2.ds1x1s2.256-512@56", R50), "dense", 0.5, 1),   # strided 1x1 (dX written cell-wise)
    (_layer("l3.1x1.256-1024@14", R50), "t25", 0.002, 1),      # 14x14 maps
    (_layer("l4.1x1.512-2048@7", R50), "dense", 0.5, 1),       # 7x7 maps (odd row length)
    (_layer("l4.3x3.512-512@7", R50), "t25", 0.05, 1),
    (_layer("stem.7x7s2.3-64@224", synth.resnet18_layers(64)), "laplace", 0.3, 1),
    (_layer("body.3x3.64-64", synth.sr_layers(16, 96)), "spikes", 0.1, 1),   # batch 16
]


def _grad(kind, r, shape):
    if kind == "t25":
        return synth.grad_cfg4(r, shape)
    if kind == "dense":
        return synth.dense_grad(r, shape)
    if kind == "laplace":
        return synth.grad_cfg2(r, shape, 1e-6)
    return synth.grad_cfg5(r, shape)


@pytest.mark.parametrize("idx", range(len(CASES)), ids=[c[0].name + "-" + c[1] for c in CASES])
def test_full_size_layer(idx):
    L, kind, gamma0, rounding = CASES[idx]
    print("full-size", L.name, kind, gamma0, rounding, flush=True)
    r = synth.rng(0, 40, idx, 0)
    X = synth.relu_normal(r, L.x_shape)
    W = synth.kaiming_normal(r, L.w_shape)
    dY = _grad(kind, r, L.dy_shape)
    seed = 0x5EED0000 + L.K

    # --- GPU: the call the benchmark makes, plus the raw accumulators ------------------
    st = lbt.new_state(gamma0=gamma0)
    res = gu.backward_conv2d(X, W, dY, L.stride, L.pad, st, x_unsigned=True, seed=seed,
                             rounding=rounding)
    h_before = lbt.lbt_state_read(st)
    lbt.lbt_update_interval(st)
    h_after = lbt.lbt_state_read(st)
    # the benchmark's launch configuration: the same call with the interval update inside it
    st2 = lbt.new_state(gamma0=gamma0)
    res2 = gu.backward_conv2d(X, W, dY, L.stride, L.pad, st2, x_unsigned=True, seed=seed,
                              rounding=rounding | lbt.FUSED_UPDATE, with_acc=False)
    h2 = lbt.lbt_state_read(st2)
    assert (h2.gamma, h2.step, h2.n_out, h2.status) == (h_after.gamma, h_after.step, h_after.n_out,
                                                        h_after.status)
    assert np.array_equal(res2.dX, res.dX) and np.array_equal(res2.dW, res.dW)
    # and the call that reads the operand codes a forward call kept (bench.py --saved-codes):
    # the same bits as the call checked against the oracle below
    _, saved = gu.save_conv2d(X, W, L.stride, L.pad, x_unsigned=True, product=False)
    st3 = lbt.new_state(gamma0=gamma0)
    res3 = gu.backward_conv2d_saved(saved, L.x_shape, L.w_shape, dY, L.stride, L.pad, st3,
                                    x_unsigned=True, seed=seed, rounding=rounding | lbt.FUSED_UPDATE)
    h3 = lbt.lbt_state_read(st3)
    assert (h3.gamma, h3.step, h3.n_out, h3.status) == (h2.gamma, h2.step, h2.n_out, h2.status)
    assert np.array_equal(res3.acc_dx, res.acc_dx) and np.array_equal(res3.acc_dw, res.acc_dw)
    assert np.array_equal(res3.dX, res.dX) and np.array_equal(res3.dW, res.dW)
    del saved, res3

    # --- oracle: quantizers in full ---------------------------------------------------------
    ost = oracle.GradState(gamma=gamma0)
    qG = oracle.quantize_grad(dY, ost, seed, rounding)
    gu.assert_state_equal(h_before, ost)
    oracle.update_interval(ost)
    assert h_after.gamma == ost.gamma and h_after.step == ost.step == 1
    qX, c_x, s_x, _ = oracle.quantize_operand(X, 0.0, True)
    qW, c_w, s_w, _ = oracle.quantize_operand(W, 0.0, False)
    s_g = oracle.scale(ost.clip, 4)

    # --- oracle: contractions at sampled positions ---------------------------------------------
    pick = np.random.default_rng(7)
    n_dx = int(np.prod(L.x_shape))
    ix = np.unique(np.concatenate([pick.integers(0, n_dx, 3000), [0, n_dx - 1]]))
    want_dx = oracle.conv2d_dx_at(qG, qW, L.x_shape, L.stride, L.pad, ix)
    got_dx = res.acc_dx.reshape(-1)[ix]
    assert np.array_equal(got_dx, want_dx), "dX accumulators differ"
    gu.assert_outputs_close(res.dX.reshape(-1)[ix], oracle.dequant(want_dx, s_g, s_w))
    n_dw = int(np.prod(L.w_shape))
    iw = np.unique(np.concatenate([pick.integers(0, n_dw, 150), [0, n_dw - 1]]))
    want_dw = oracle.conv2d_dw_at(qG, qX, L.w_shape, L.stride, L.pad, iw)
    got_dw = res.acc_dw.reshape(-1)[iw]
    assert np.array_equal(got_dw, want_dw), "dW accumulators differ"
    gu.assert_outputs_close(res.dW.reshape(-1)[iw], oracle.dequant(want_dw, s_x, s_g))
    # properties that hold at any size: the scale factors out exactly, nothing is NaN
    assert np.isfinite(res.dX).all() and np.isfinite(res.dW).all()
    if kind != "t25" or gamma0 < 0.1:
        assert np.abs(want_dx).max() > 0 and np.abs(want_dw).max() > 0   # the sample is not trivial


def test_full_size_flat_codes():
    # the C-ABI code format on the largest gradient tensor of the sweep (51.4 M elements)
    L = _layer("l1.1x1.64-256@56", R50)
    r = synth.rng(0, 41, 0, synth.T_DY)
    g = synth.grad_cfg4(r, L.dy_shape).reshape(-1)
    for gamma0, rounding in ((1.0, 1), (0.003, 1), (0.02, 0)):
        ost = oracle.GradState(gamma=gamma0, step=5)
        want = oracle.quantize_grad(g, ost, 99, rounding)
        st = lbt.new_state(gamma0=gamma0)
        h = lbt.lbt_state_read(st)
        h.step = 5
        lbt.lbt_state_write(st, h)
        packed = gu.quantize_grad(g, st, 99, rounding)
        gu.assert_state_equal(lbt.lbt_state_read(st), ost)
        assert np.array_equal(packed, oracle.pack_nibbles(want))


def test_full_size_linear():
    L = [x for x in R50 if isinstance(x, synth.LinearLayer)][0]
    r = synth.rng(0, 42, 0, 0)
    X, W = synth.relu_normal(r, (L.M, L.K)), synth.normal(r, (L.K, L.N), 0.02)
    dY = synth.grad_cfg4(r, (L.M, L.N))
    ost = oracle.GradState(gamma=0.1)
    st = lbt.new_state(gamma0=0.1)
    ref = oracle.backward_linear(X, W, dY, ost, x_unsigned=True, seed=3, rounding=1)
    res = gu.backward_linear(X, W, dY, st, x_unsigned=True, seed=3, rounding=1)
    gu.assert_state_equal(lbt.lbt_state_read(st), ost)
    assert np.array_equal(res.acc_dx, ref.acc_dx) and np.array_equal(res.acc_dw, ref.acc_dw)
    gu.assert_outputs_close(res.dX, ref.dX)
    gu.assert_outputs_close(res.dW, ref.dW)


def test_full_size_vit_linear():
    # the largest linear layer of a ViT-L encoder block (supplement, Table C) at batch 64:
    # 12608 token rows, 1024 -> 4096; signed activations; sampled rows of dX, columns of dW
    L = [x for x in synth.vit_l_layers(64) if x.name == "vit.fc1.1024-4096"][0]
    r = synth.rng(0, 43, 0, 0)
    X, W = synth.normal(r, (L.M, L.K), 1.0), synth.normal(r, (L.K, L.N), 0.02)
    dY = synth.grad_cfg4(r, (L.M, L.N))
    st = lbt.new_state(gamma0=0.05)
    res = gu.backward_linear(X, W, dY, st, x_unsigned=False, seed=11, rounding=1)
    ost = oracle.GradState(gamma=0.05)
    qG = oracle.quantize_grad(dY, ost, 11, 1)
    gu.assert_state_equal(lbt.lbt_state_read(st), ost)
    qX, c_x, s_x, _ = oracle.quantize_operand(X, 0.0, False)
    qW, c_w, s_w, _ = oracle.quantize_operand(W, 0.0, False)
    s_g = oracle.scale(ost.clip, 4)
    pick = np.random.default_rng(9)
    rows = np.unique(np.concatenate([pick.integers(0, L.M, 24), [0, L.M - 1]]))
    want_dx = oracle.linear_dx(qG[rows], qW)
    assert np.array_equal(res.acc_dx[rows], want_dx), "dX accumulators differ"
    gu.assert_outputs_close(res.dX[rows], oracle.dequant(want_dx, s_g, s_w))
    cols = np.unique(np.concatenate([pick.integers(0, L.N, 24), [0, L.N - 1]]))
    want_dw = oracle.linear_dw(qX, np.ascontiguousarray(qG[:, cols]))
    assert np.array_equal(res.acc_dw[:, cols], want_dw), "dW accumulators differ"
    gu.assert_outputs_close(res.dW[:, cols], oracle.dequant(want_dw, s_x, s_g))
    assert np.abs(want_dx).max() > 0 and np.abs(want_dw).max() > 0

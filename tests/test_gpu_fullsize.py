"""GPU parity at the full layer sizes of the five workload configurations (every ResNet-50
bottleneck shape at batch 64 -- the benchmark's sweep --, the ResNet-18 shapes at batch 64,
the CIFAR ResNet-20 stages at batch 128, the super-resolution head / body / tail at batch 16,
the linear layers), through the same entry points the benchmark calls.

The oracle computes what it can in full (maximum, clip value, clip-out count, gamma
after the update: all O(n)); the contractions are checked (i) on sampled output positions,
one by one, from the oracle's own codes and (ii) over the WHOLE accumulator tensors with a
Freivalds-style contraction against random +-1 vectors, again from the oracle's codes
(exact in int64; a wrong tile anywhere survives one vector with probability <= 1/2, three
vectors are used).  Everything integer is compared bit for bit."""
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
    if kind.startswith("laplace:"):
        return synth.grad_cfg2(r, shape, float(kind.split(":")[1]))
    return synth.grad_cfg5(r, shape)


N_VECTORS = 3


def _freivalds_conv(res, qG, qX, qW, L, tag):
    """Whole-tensor check of both accumulator tensors against the oracle's codes."""
    pick = np.random.default_rng(1234 + len(tag))
    for v in range(N_VECTORS):
        got, want = oracle.freivalds_conv2d_dx(res.acc_dx, qG, qW, L.stride, L.pad,
                                               oracle.signs(pick, L.C))
        assert np.array_equal(got, want), "dX accumulators fail the whole-tensor check: " + tag
        got, want = oracle.freivalds_conv2d_dw(res.acc_dw, qG, qX, L.stride, L.pad,
                                               oracle.signs(pick, L.K))
        assert np.array_equal(got, want), "dW accumulators fail the whole-tensor check: " + tag


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
    # --- oracle: both accumulator tensors as a whole ----------------------------------------------
    _freivalds_conv(res, qG, qX, qW, L, L.name)
    # properties that hold at any size: the scale factors out exactly, nothing is NaN
    assert np.isfinite(res.dX).all() and np.isfinite(res.dW).all()
    if kind != "t25" or gamma0 < 0.1:
        assert np.abs(want_dx).max() > 0 and np.abs(want_dw).max() > 0   # the sample is not trivial
    # the outputs are the accumulators times one fp32 scale, everywhere
    scale_x = np.float32(s_g * s_w)
    assert np.array_equal(res.dX, res.acc_dx.astype(np.float32) * scale_x)


# Every remaining layer shape of the five configurations at its named batch size, through the
# benchmark's call: quantizer state in full, sampled sums, whole-tensor check.
R18 = synth.resnet18_layers(64)
CIFAR = synth.cifar_layers(128)
SR = synth.sr_layers(16, 96)
_done = {c[0].name for c in CASES if c[0] in R50}
MORE = (
    # (layer, gradient recipe, gamma0, rounding, activations unsigned)
    [(L, "t25" if i % 3 else "dense", (0.02, 0.5, 1.0)[i % 3], 1, True)
     for i, L in enumerate(R50) if isinstance(L, synth.ConvLayer) and L.name not in _done]
    # ResNet-18 (Laplace gradients with sparse outliers, per-layer scale 1e-3 .. 1e-6)
    + [(_layer(n, R18), "laplace:%g" % sc, g0, 1, True) for n, sc, g0 in (
        ("l2.3x3s2.64-128@56", 1e-5, 0.05), ("l2.ds1x1s2.64-128@56", 1e-5, 0.3),
        ("l3.ds1x1s2.128-256@28", 1e-4, 0.1), ("l4.ds1x1s2.256-512@14", 3e-4, 0.05),
        ("l3.3x3s2.128-256@28", 1e-4, 1.0), ("l4.3x3s2.256-512@14", 3e-4, 0.2))]
    # CIFAR ResNet-20 stages at batch 128
    + [(L, "laplace:1e-4", g0, 1, True) for L, g0 in zip(CIFAR, (0.05, 0.3, 1.0))]
    # super-resolution head (zero-centred input image: signed activations) and x4 tail
    + [(_layer("head.3x3.3-64", SR), "spikes", 0.1, 1, False),
       (_layer("tail.3x3.64-256", SR), "spikes", 0.05, 1, True),
       (_layer("body.3x3.64-64", SR), "spikes", 0.3, 0, False)]   # post-add input: signed
)


@pytest.mark.parametrize("idx", range(len(MORE)),
                         ids=["%s-%s-b%d" % (c[0].name, c[1], c[0].N) for c in MORE])
def test_full_size_layer_of_every_configuration(idx):
    L, kind, gamma0, rounding, x_unsigned = MORE[idx]
    print("full-size", L.name, "batch", L.N, kind, gamma0, rounding, x_unsigned, flush=True)
    r = synth.rng(0, 44, idx, 0)
    X = synth.relu_normal(r, L.x_shape) if x_unsigned else synth.normal(r, L.x_shape)
    W = synth.kaiming_normal(r, L.w_shape)
    dY = _grad(kind, r, L.dy_shape)
    seed = 0xC0FFEE00 + idx
    st = lbt.new_state(gamma0=gamma0)
    res = gu.backward_conv2d(X, W, dY, L.stride, L.pad, st, x_unsigned=x_unsigned, seed=seed,
                             rounding=rounding | lbt.FUSED_UPDATE)
    h = lbt.lbt_state_read(st)
    ost = oracle.GradState(gamma=gamma0)
    qG = oracle.quantize_grad(dY, ost, seed, rounding)
    oracle.update_interval(ost)
    gu.assert_state_equal(h, ost)
    qX, c_x, s_x, _ = oracle.quantize_operand(X, 0.0, x_unsigned)
    qW, c_w, s_w, _ = oracle.quantize_operand(W, 0.0, False)
    s_g = oracle.scale(ost.clip, 4)
    pick = np.random.default_rng(70 + idx)
    n_dx, n_dw = int(np.prod(L.x_shape)), int(np.prod(L.w_shape))
    ix = np.unique(np.concatenate([pick.integers(0, n_dx, 1000), [0, n_dx - 1]]))
    want_dx = oracle.conv2d_dx_at(qG, qW, L.x_shape, L.stride, L.pad, ix)
    assert np.array_equal(res.acc_dx.reshape(-1)[ix], want_dx), "dX accumulators differ"
    gu.assert_outputs_close(res.dX.reshape(-1)[ix], oracle.dequant(want_dx, s_g, s_w))
    iw = np.unique(np.concatenate([pick.integers(0, n_dw, 60), [0, n_dw - 1]]))
    want_dw = oracle.conv2d_dw_at(qG, qX, L.w_shape, L.stride, L.pad, iw)
    assert np.array_equal(res.acc_dw.reshape(-1)[iw], want_dw), "dW accumulators differ"
    gu.assert_outputs_close(res.dW.reshape(-1)[iw], oracle.dequant(want_dw, s_x, s_g))
    _freivalds_conv(res, qG, qX, qW, L, L.name)
    assert np.isfinite(res.dX).all() and np.isfinite(res.dW).all()
    assert np.abs(res.acc_dw).max() > 0
    assert np.array_equal(res.dX, res.acc_dx.astype(np.float32) * np.float32(s_g * s_w))


# The protocol of the ResNet-50 configuration on two of its layers: 100 iterations, a fresh
# seeded gradient draw each, {quantize + count, dX, dW, update} per iteration.  The state is
# compared with the oracle's bit for bit after every update, the whole accumulator tensors
# after every iteration (one vector each), sampled sums on the first and last iteration.
@pytest.mark.parametrize("name", ["l3.3x3.256-256@14", "l4.1x1.512-2048@7"])
def test_hundred_iterations_of_the_resnet50_protocol(name):
    L = _layer(name, R50)
    li = [x.name for x in R50].index(name)
    r = synth.rng(0, 4, li, 0)
    X = synth.relu_normal(r, L.x_shape)
    W = synth.kaiming_normal(r, L.w_shape)
    Xd, Wd = gu.dev(X), gu.dev(W)
    qX, c_x, s_x, _ = oracle.quantize_operand(X, 0.0, True)
    qW, c_w, s_w, _ = oracle.quantize_operand(W, 0.0, False)
    # gamma0 = 1 is the configuration's start; the second layer starts where the gradient
    # tail makes the sign of the update change during the run
    st = lbt.new_state(gamma0=1.0 if li % 2 else 0.012)
    ost = oracle.GradState(gamma=1.0 if li % 2 else 0.012)
    ws = torch.zeros(lbt.lbt_workspace_bytes_conv2d(L.N, L.C, L.H, L.W, L.K, L.R, L.S, L.stride, L.pad),
                     dtype=torch.uint8, device=gu.DEV)
    dX = torch.empty(L.x_shape, dtype=torch.float32, device=gu.DEV)
    dW = torch.empty(L.w_shape, dtype=torch.float32, device=gu.DEV)
    aX = torch.empty(L.x_shape, dtype=torch.int32, device=gu.DEV)
    aW = torch.empty(L.w_shape, dtype=torch.int32, device=gu.DEV)
    pick = np.random.default_rng(5)
    signs_seen = set()
    for it in range(100):
        if it % 10 == 0:
            print("protocol", name, "iteration", it, "gamma", ost.gamma, flush=True)
        dY = synth.grad_cfg4(synth.rng(0, 4, li, synth.T_DY, it), L.dy_shape)
        lbt.lbt_backward_conv2d_acc(Xd, Wd, gu.dev(dY), L.N, L.C, L.H, L.W, L.K, L.R, L.S, L.stride,
                                    L.pad, 0.0, True, 0.0, st, 1000 + it, lbt.ROUND_STOCHASTIC,
                                    dX, dW, aX, aW, ws)
        h = lbt.lbt_state_read(st)
        qG = oracle.quantize_grad(dY, ost, 1000 + it, oracle.STOCHASTIC)
        gu.assert_state_equal(h, ost)
        lbt.lbt_update_interval(st)
        signs_seen.add(oracle.update_interval(ost))
        h = lbt.lbt_state_read(st)
        assert h.gamma == ost.gamma and h.step == ost.step == it + 1
        res = gu.Result()
        res.acc_dx, res.acc_dw = aX.cpu().numpy(), aW.cpu().numpy()
        got, want = oracle.freivalds_conv2d_dx(res.acc_dx, qG, qW, L.stride, L.pad, oracle.signs(pick, L.C))
        assert np.array_equal(got, want), "dX accumulators, iteration %d" % it
        got, want = oracle.freivalds_conv2d_dw(res.acc_dw, qG, qX, L.stride, L.pad, oracle.signs(pick, L.K))
        assert np.array_equal(got, want), "dW accumulators, iteration %d" % it
        if it in (0, 99):
            s_g = oracle.scale(ost.clip, 4)
            ix = pick.integers(0, int(np.prod(L.x_shape)), 500)
            want_dx = oracle.conv2d_dx_at(qG, qW, L.x_shape, L.stride, L.pad, ix)
            assert np.array_equal(res.acc_dx.reshape(-1)[ix], want_dx)
            gu.assert_outputs_close(dX.cpu().numpy().reshape(-1)[ix], oracle.dequant(want_dx, s_g, s_w))
            iw = pick.integers(0, int(np.prod(L.w_shape)), 40)
            want_dw = oracle.conv2d_dw_at(qG, qX, L.w_shape, L.stride, L.pad, iw)
            assert np.array_equal(res.acc_dw.reshape(-1)[iw], want_dw)
            gu.assert_outputs_close(dW.cpu().numpy().reshape(-1)[iw], oracle.dequant(want_dw, s_x, s_g))
    if li % 2 == 0:
        assert signs_seen >= {1, -1}, signs_seen     # the interval moved both ways


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


def test_full_size_linear_resnet18_classifier():
    L = [x for x in R18 if isinstance(x, synth.LinearLayer)][0]        # 512 -> 1000 at batch 64
    r = synth.rng(0, 45, 0, 0)
    X, W = synth.relu_normal(r, (L.M, L.K)), synth.normal(r, (L.K, L.N), 0.03)
    dY = synth.grad_cfg2(r, (L.M, L.N), 1e-3)
    for rounding in (0, 1):
        ost = oracle.GradState(gamma=0.2)
        st = lbt.new_state(gamma0=0.2)
        ref = oracle.backward_linear(X, W, dY, ost, x_unsigned=True, seed=8, rounding=rounding)
        res = gu.backward_linear(X, W, dY, st, x_unsigned=True, seed=8, rounding=rounding)
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
    # both accumulator matrices as a whole
    for v in range(N_VECTORS):
        (g1, w1), (g2, w2) = oracle.freivalds_linear(res.acc_dx, res.acc_dw, qG, qX, qW,
                                                     oracle.signs(pick, L.K), oracle.signs(pick, L.N))
        assert np.array_equal(g1, w1), "dX accumulators fail the whole-matrix check"
        assert np.array_equal(g2, w2), "dW accumulators fail the whole-matrix check"

"""The backward call under HIP graph capture: the call only enqueues kernels (no allocation,
no memset node, no host synchronisation), so a captured call can be replayed.  Every replay is
checked against the oracle, with new gradient values copied into the captured buffers and eager
work and synchronisations of the program's own between the replays; the state (gamma, step)
advances across replays exactly as across eager calls."""
import numpy as np
import pytest
import torch

import oracle
from paper_2407_12637_amd import binding as lbt
from paper_2407_12637_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu


def test_captured_backward_call_replays_like_eager_calls():
    N, C, H, W, K, R, S, stride, pad = 8, 32, 14, 14, 64, 3, 3, 1, 1
    geom = (N, C, H, W, K, R, S, stride, pad)
    print("graph capture", geom, flush=True)
    r = synth.rng(0, 102, 0, 0)
    X, Wt = synth.relu_normal(r, (N, C, H, W)), synth.kaiming_normal(r, (K, C, R, S))
    grads = [synth.dense_grad(r, (N, K, H, W)), synth.grad_cfg2(r, (N, K, H, W)),
             synth.dense_grad(r, (N, K, H, W)) * np.float32(3.0), synth.grad_cfg4(r, (N, K, H, W))]
    Xd, Wd = gu.dev(X), gu.dev(Wt)
    dY = torch.zeros((N, K, H, W), device=gu.DEV)
    dX = torch.zeros((N, C, H, W), device=gu.DEV)
    dW = torch.zeros((K, C, R, S), device=gu.DEV)
    aX = torch.zeros((N, C, H, W), dtype=torch.int32, device=gu.DEV)
    aW = torch.zeros((K, C, R, S), dtype=torch.int32, device=gu.DEV)
    ws = torch.zeros(lbt.lbt_workspace_bytes_conv2d(*geom), dtype=torch.uint8, device=gu.DEV)
    st = lbt.new_state(gamma0=0.6)
    ost = oracle.GradState(gamma=0.6)
    flags = lbt.ROUND_STOCHASTIC | lbt.FUSED_UPDATE

    def call():
        lbt.lbt_backward_conv2d_acc(Xd, Wd, dY, *geom, 0.0, True, 0.0, st, 77, flags, dX, dW, aX, aW, ws)

    def check(g):
        ref = oracle.backward_conv2d(X, Wt, g, stride, pad, ost, seed=77, rounding=1)
        oracle.update_interval(ost)
        torch.cuda.synchronize()
        gu.assert_state_equal(lbt.lbt_state_read(st), ost)
        assert np.array_equal(aX.cpu().numpy(), ref.acc_dx) and np.array_equal(aW.cpu().numpy(), ref.acc_dw)
        gu.assert_outputs_close(dX.cpu().numpy(), ref.dX)
        gu.assert_outputs_close(dW.cpu().numpy(), ref.dW)

    # one eager call first (also loads the kernels before the capture)
    dY.copy_(gu.dev(grads[0]))
    call()
    check(grads[0])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        dY.copy_(gu.dev(grads[1]))
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            call()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    # the capture itself ran nothing: the state is where the eager call left it
    assert lbt.lbt_state_read(st).step == 1
    for it, g in enumerate(grads[1:] + grads[:2]):
        dY.copy_(gu.dev(g))
        for out in (dX, dW):
            out.fill_(float("nan"))
        scratch = torch.randn(1 << 20, device=gu.DEV).sum()     # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        check(g)
        assert torch.isfinite(scratch)
    assert lbt.lbt_state_read(st).step == 6

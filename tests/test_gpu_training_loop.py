"""The calls compose into a training loop: a two-layer perceptron on a synthetic regression
task, every product of the forward and the backward pass on the integer path (forward calls
that keep the operand codes, backward calls that read them, the interval update inside the
backward call).  Not a parity test (those compare every call with the oracle): it checks that
the pieces fit together as Sec. 3.1 / Alg. 1 use them - the loss goes down, the clipping
factors of both layers move and stay inside (0, 1], no call reports a fault."""
import numpy as np
import pytest
import torch

from paper_2407_12637_amd import binding as lbt
from paper_2407_12637_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu


class Linear:
    def __init__(self, r, k_in, n_out, bits):
        self.K, self.N, self.bits = k_in, n_out, bits
        self.W = gu.dev(synth.normal(r, (k_in, n_out), (1.0 / k_in) ** 0.5))
        self.state = lbt.new_state(gamma0=1.0, bits=bits)
        self.saved = self.M = None

    def forward(self, X, x_unsigned):
        M = X.shape[0]
        self.M, self.x_unsigned = M, x_unsigned
        self.saved = torch.zeros(lbt.lbt_saved_bytes_linear(M, self.K, self.N), dtype=torch.uint8,
                                 device=gu.DEV)
        ws = torch.zeros(lbt.lbt_workspace_bytes_forward_linear(M, self.K, self.N),
                         dtype=torch.uint8, device=gu.DEV)
        Y = torch.empty((M, self.N), device=gu.DEV)
        status = torch.zeros(1, dtype=torch.int32, device=gu.DEV)
        lbt.lbt_forward_linear_save(X, self.W, M, self.K, self.N, 0.0, x_unsigned, 0.0,
                                    lbt.BITS(self.bits), Y, None, status, self.saved, ws)
        assert int(status.item()) == lbt.STATUS_OK
        return Y

    def backward(self, dY, step, want_dx=True):
        ws = torch.zeros(lbt.lbt_workspace_bytes_linear(self.M, self.K, self.N), dtype=torch.uint8,
                         device=gu.DEV)
        dX = torch.empty((self.M, self.K), device=gu.DEV) if want_dx else None
        dW = torch.empty((self.K, self.N), device=gu.DEV)
        lbt.lbt_backward_linear_saved(self.saved, dY.contiguous(), self.M, self.K, self.N,
                                      self.x_unsigned, self.state, 1234,
                                      lbt.ROUND_STOCHASTIC | lbt.FUSED_UPDATE | lbt.BITS(self.bits),
                                      dX, dW, None, None, ws)
        return dX, dW


@pytest.mark.parametrize("bits", [4, 8])
def test_two_layer_perceptron_learns(bits):
    print("training loop", bits, flush=True)
    r = synth.rng(0, 95, bits, 0)
    M, D, Hd, O = 512, 64, 128, 16
    X = gu.dev(synth.normal(r, (M, D)))
    teacher = gu.dev(synth.normal(r, (D, O), (1.0 / D) ** 0.5))
    target = torch.tanh(X @ teacher)
    l1, l2 = Linear(r, D, Hd, bits), Linear(r, Hd, O, bits)
    lr, losses, lowest = 0.5, [], {}
    for step in range(120):
        h_pre = l1.forward(X, x_unsigned=False)
        h = torch.relu(h_pre)
        y = l2.forward(h, x_unsigned=bits < 8)
        err = y - target
        losses.append(float((err * err).mean().item()))
        d_y = err * (2.0 / err.numel())
        d_h, d_w2 = l2.backward(d_y, step)
        d_hpre = d_h * (h_pre > 0)
        _, d_w1 = l1.backward(d_hpre, step, want_dx=False)
        l1.W -= lr * d_w1
        l2.W -= lr * d_w2
        for L in (l1, l2):
            st = lbt.lbt_state_read(L.state)
            assert st.status == lbt.STATUS_OK and st.step == step + 1 and 0.0 < st.gamma <= 1.0
            lowest[L.K] = min(lowest.get(L.K, 1.0), st.gamma)
    assert np.isfinite(losses).all()
    assert np.mean(losses[-10:]) < 0.6 * np.mean(losses[:5]), (losses[:5], losses[-10:])
    # Alg. 1 has moved both clipping factors (on tensors this small it settles just below 1: one
    # clipped element out of 8192 already exceeds alpha / (2^b - 1))
    assert all(g < 1.0 for g in lowest.values()) and len(lowest) == 2

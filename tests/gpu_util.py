"""Helpers for the GPU parity tests: move numpy inputs to the device, call the C ABI
through the binding, bring results back.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

from paper_2407_12637_amd import binding as lbt

DEV = "cuda"


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def unpack_nibbles(packed: np.ndarray, n: int, signed: bool) -> np.ndarray:
    """Decode the ABI's flat code format (test-side decoder, independent of both paths)."""
    lo = (packed & 0xF).astype(np.int32)
    hi = (packed >> 4).astype(np.int32)
    out = np.stack([lo, hi], 1).reshape(-1)[:n]
    return np.where(out >= 8, out - 16, out) if signed else out


def flat_codes(code: np.ndarray, bits: int) -> np.ndarray:
    """Integer codes -> the ABI's flat byte format (test-side encoder, independent of both
    paths): nibbles for b <= 4, one byte per code above."""
    c = np.asarray(code).reshape(-1).astype(np.int64)
    if bits > 4:
        return (c & 0xFF).astype(np.uint8)
    c = c & 0xF
    if c.size % 2:
        c = np.concatenate([c, [0]])
    return (c[0::2] | (c[1::2] << 4)).astype(np.uint8)


def quantize_grad(g: np.ndarray, st, seed=0, rounding=0):
    n = g.size
    bits = ((rounding >> 8) & 15) or 4
    codes = torch.full((n if bits > 4 else (n + 1) // 2,), 0xEE, dtype=torch.uint8, device=DEV)
    ws = torch.zeros(lbt.lbt_workspace_bytes_quantize(n), dtype=torch.uint8, device=DEV)
    lbt.lbt_quantize_grad(dev(g.reshape(-1)), st, seed, rounding, codes, ws)
    return codes.cpu().numpy()


def quantize_operand(x: np.ndarray, c: float, unsigned: bool, bits: int = 4):
    n = x.size
    codes = torch.full((n if bits > 4 else (n + 1) // 2,), 0xEE, dtype=torch.uint8, device=DEV)
    cs = torch.zeros(2, dtype=torch.float32, device=DEV)
    ws = torch.zeros(lbt.lbt_workspace_bytes_quantize(n), dtype=torch.uint8, device=DEV)
    lbt.lbt_quantize_operand(dev(x.reshape(-1)), c, unsigned, bits, codes, cs, ws)
    return codes.cpu().numpy(), cs.cpu().numpy()


class Result:
    pass


def backward_linear(X, W, dY, st, c_x=0.0, x_unsigned=False, c_w=0.0, seed=0, rounding=0,
                    want_dx=True, want_dw=True):
    M, K = X.shape
    N = W.shape[1]
    ws = torch.zeros(lbt.lbt_workspace_bytes_linear(M, K, N), dtype=torch.uint8, device=DEV)
    r = Result()
    dX = torch.full((M, K), float("nan"), device=DEV) if want_dx else None
    dW = torch.full((K, N), float("nan"), device=DEV) if want_dw else None
    aX = torch.full((M, K), -1, dtype=torch.int32, device=DEV) if want_dx else None
    aW = torch.full((K, N), -1, dtype=torch.int32, device=DEV) if want_dw else None
    lbt.lbt_backward_linear_acc(dev(X), dev(W), dev(dY), M, K, N, c_x, x_unsigned, c_w, st, seed,
                                rounding, dX, dW, aX, aW, ws)
    r.dX, r.dW, r.acc_dx, r.acc_dw = [None if t is None else t.cpu().numpy()
                                      for t in (dX, dW, aX, aW)]
    return r


def backward_conv2d(X, W, dY, stride, pad, st, c_x=0.0, x_unsigned=True, c_w=0.0, seed=0,
                    rounding=0, want_dx=True, want_dw=True, with_acc=True):
    N, Cc, H, Wd = X.shape
    K, _, R, S = W.shape
    ws = torch.zeros(lbt.lbt_workspace_bytes_conv2d(N, Cc, H, Wd, K, R, S, stride, pad),
                     dtype=torch.uint8, device=DEV)
    r = Result()
    dX = torch.full(X.shape, float("nan"), device=DEV) if want_dx else None
    dW = torch.full(W.shape, float("nan"), device=DEV) if want_dw else None
    aX = torch.full(X.shape, -1, dtype=torch.int32, device=DEV) if want_dx and with_acc else None
    aW = torch.full(W.shape, -1, dtype=torch.int32, device=DEV) if want_dw and with_acc else None
    lbt.lbt_backward_conv2d_acc(dev(X), dev(W), dev(dY), N, Cc, H, Wd, K, R, S, stride, pad, c_x,
                                x_unsigned, c_w, st, seed, rounding, dX, dW, aX, aW, ws)
    r.dX, r.dW, r.acc_dx, r.acc_dw = [None if t is None else t.cpu().numpy()
                                      for t in (dX, dW, aX, aW)]
    return r


def forward_linear(X, W, c_x=0.0, x_unsigned=False, c_w=0.0, flags=0, with_acc=True):
    M, K = X.shape
    N = W.shape[1]
    ws = torch.zeros(lbt.lbt_workspace_bytes_forward_linear(M, K, N), dtype=torch.uint8, device=DEV)
    Y = torch.full((M, N), float("nan"), device=DEV)
    acc = torch.full((M, N), -1, dtype=torch.int32, device=DEV) if with_acc else None
    status = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    lbt.lbt_forward_linear(dev(X), dev(W), M, K, N, c_x, x_unsigned, c_w, flags, Y, acc, status, ws)
    r = Result()
    r.Y, r.acc, r.status = Y.cpu().numpy(), None if acc is None else acc.cpu().numpy(), int(status.item())
    return r


def forward_conv2d(X, W, stride, pad, c_x=0.0, x_unsigned=True, c_w=0.0, flags=0, with_acc=True):
    N, Cc, H, Wd = X.shape
    K, _, R, S = W.shape
    P, Q = (H + 2 * pad - R) // stride + 1, (Wd + 2 * pad - S) // stride + 1
    ws = torch.zeros(lbt.lbt_workspace_bytes_forward_conv2d(N, Cc, H, Wd, K, R, S, stride, pad),
                     dtype=torch.uint8, device=DEV)
    Y = torch.full((N, K, P, Q), float("nan"), device=DEV)
    acc = torch.full((N, K, P, Q), -1, dtype=torch.int32, device=DEV) if with_acc else None
    status = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    lbt.lbt_forward_conv2d(dev(X), dev(W), N, Cc, H, Wd, K, R, S, stride, pad, c_x, x_unsigned, c_w,
                           flags, Y, acc, status, ws)
    r = Result()
    r.Y, r.acc, r.status = Y.cpu().numpy(), None if acc is None else acc.cpu().numpy(), int(status.item())
    return r


def assert_state_equal(h, o):
    """Device state (binding.GradState) vs oracle.GradState, bit for bit."""
    assert h.status == o.status, (h.status, o.status)
    assert h.n_total == o.n_total and h.bits == o.bits
    if o.status == 1:
        return
    assert h.n_out == o.n_out, (h.n_out, o.n_out)
    assert h.gamma == o.gamma and h.step == o.step
    assert np.float32(h.gmax) == o.gmax, (h.gmax, o.gmax)
    assert np.float32(h.clip) == o.clip and np.float32(h.scale) == o.scale


def assert_outputs_close(got, want):
    """fp32 outputs: 1e-5 relative (the accumulators themselves are compared exactly)."""
    np.testing.assert_allclose(got, want, rtol=1e-5, atol=0)


def save_conv2d(X, W, stride, pad, c_x=0.0, x_unsigned=True, c_w=0.0, flags=0, product=True):
    """lbt_forward_conv2d_save: the forward result (when product) and the saved-codes buffer."""
    N, Cc, H, Wd = X.shape
    K, _, R, S = W.shape
    P, Q = (H + 2 * pad - R) // stride + 1, (Wd + 2 * pad - S) // stride + 1
    saved = torch.full((lbt.lbt_saved_bytes_conv2d(N, Cc, H, Wd, K, R, S, stride, pad),), 0xEE,
                       dtype=torch.uint8, device=DEV)
    r = Result()
    if product:
        ws = torch.zeros(lbt.lbt_workspace_bytes_forward_conv2d(N, Cc, H, Wd, K, R, S, stride, pad),
                         dtype=torch.uint8, device=DEV)
        Y = torch.full((N, K, P, Q), float("nan"), device=DEV)
        acc = torch.full((N, K, P, Q), -1, dtype=torch.int32, device=DEV)
        status = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    else:
        ws = Y = acc = status = None
    lbt.lbt_forward_conv2d_save(dev(X), dev(W), N, Cc, H, Wd, K, R, S, stride, pad, c_x, x_unsigned,
                                c_w, flags, Y, acc, status, saved, ws)
    if product:
        r.Y, r.acc, r.status = Y.cpu().numpy(), acc.cpu().numpy(), int(status.item())
    return r, saved


def save_linear(X, W, c_x=0.0, x_unsigned=False, c_w=0.0, flags=0, product=True):
    M, K = X.shape
    N = W.shape[1]
    saved = torch.full((lbt.lbt_saved_bytes_linear(M, K, N),), 0xEE, dtype=torch.uint8, device=DEV)
    r = Result()
    if product:
        ws = torch.zeros(lbt.lbt_workspace_bytes_forward_linear(M, K, N), dtype=torch.uint8, device=DEV)
        Y = torch.full((M, N), float("nan"), device=DEV)
        acc = torch.full((M, N), -1, dtype=torch.int32, device=DEV)
        status = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    else:
        ws = Y = acc = status = None
    lbt.lbt_forward_linear_save(dev(X), dev(W), M, K, N, c_x, x_unsigned, c_w, flags, Y, acc, status,
                                saved, ws)
    if product:
        r.Y, r.acc, r.status = Y.cpu().numpy(), acc.cpu().numpy(), int(status.item())
    return r, saved


def backward_conv2d_saved(saved, x_shape, w_shape, dY, stride, pad, st, x_unsigned=True, seed=0,
                          rounding=0, want_dx=True, want_dw=True):
    N, Cc, H, Wd = x_shape
    K, _, R, S = w_shape
    ws = torch.zeros(lbt.lbt_workspace_bytes_conv2d(N, Cc, H, Wd, K, R, S, stride, pad),
                     dtype=torch.uint8, device=DEV)
    r = Result()
    dX = torch.full(x_shape, float("nan"), device=DEV) if want_dx else None
    dW = torch.full(w_shape, float("nan"), device=DEV) if want_dw else None
    aX = torch.full(x_shape, -1, dtype=torch.int32, device=DEV) if want_dx else None
    aW = torch.full(w_shape, -1, dtype=torch.int32, device=DEV) if want_dw else None
    lbt.lbt_backward_conv2d_saved(saved, dev(dY), N, Cc, H, Wd, K, R, S, stride, pad, x_unsigned, st,
                                  seed, rounding, dX, dW, aX, aW, ws)
    r.dX, r.dW, r.acc_dx, r.acc_dw = [None if t is None else t.cpu().numpy()
                                      for t in (dX, dW, aX, aW)]
    return r


def backward_linear_saved(saved, M, K, N, dY, st, x_unsigned=False, seed=0, rounding=0,
                          want_dx=True, want_dw=True):
    ws = torch.zeros(lbt.lbt_workspace_bytes_linear(M, K, N), dtype=torch.uint8, device=DEV)
    r = Result()
    dX = torch.full((M, K), float("nan"), device=DEV) if want_dx else None
    dW = torch.full((K, N), float("nan"), device=DEV) if want_dw else None
    aX = torch.full((M, K), -1, dtype=torch.int32, device=DEV) if want_dx else None
    aW = torch.full((K, N), -1, dtype=torch.int32, device=DEV) if want_dw else None
    lbt.lbt_backward_linear_saved(saved, dev(dY), M, K, N, x_unsigned, st, seed, rounding, dX, dW,
                                  aX, aW, ws)
    r.dX, r.dW, r.acc_dx, r.acc_dw = [None if t is None else t.cpu().numpy()
                                      for t in (dX, dW, aX, aW)]
    return r

"""CPU oracle for the INT4 fixed-point backward pass -- TEST INFRASTRUCTURE ONLY.

A plain double / int64 implementation of what the GPU library computes, written
from the paper (Kim et al., "Toward INT4 Fixed-Point Training via Exploring
Quantization Error for Gradients"): the uniform quantizer of Eq. (1)-(4), the
gradient clip value c_g = gamma * g_max of Sec. 3.1, the clip-out count and the
clipping-factor update of Eq. (15)-(16) / Alg. 1, and the two integer
contractions of the backward pass with the denormalisation of Eq. (4); also the
quantized forward product Y = Q(X) . Q(W) of the same layers (numpy int64).

Only tests, the smoke entry and the benchmark's cpu_baseline leg may import
this package.  It shares nothing with the HIP path and imports nothing from it.
The arithmetic lives in ``lbt_oracle.c`` (compiled with gcc on first use);
this file marshals numpy arrays and strings the steps together in the paper's
order.  ``diagnostics.py`` holds the error measures E(G), E(G_L), the bound
U(G_L) and its derivative, used to pin the oracle against the paper's closed
forms.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lbt_oracle.c")
_LIB = os.path.join(_HERE, "liblbt_oracle.so")

OK, NONFINITE, ZERO_GRAD = 0, 1, 2
NEAREST, STOCHASTIC = 0, 1


def build(force: bool = False) -> str:
    """Compile lbt_oracle.c with gcc (no fused multiply-add, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
             "-fno-fast-math", "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _L():
    global _lib
    if _lib is None:
        lib = C.CDLL(build())
        i64, u64, f32, f64, i32 = C.c_int64, C.c_uint64, C.c_float, C.c_double, C.c_int
        p = C.c_void_p
        lib.orc_num_threads.restype = i32
        lib.orc_philox4x32_10.argtypes = [p, p, p]
        lib.orc_r16.argtypes = [u64, u64, u64]
        lib.orc_r16.restype = C.c_uint32
        lib.orc_max.argtypes = [p, i64, i32, p]
        lib.orc_max.restype = i32
        lib.orc_clip_value.argtypes = [f64, f32]
        lib.orc_clip_value.restype = f32
        lib.orc_levels.argtypes = [i32, i32]
        lib.orc_levels.restype = i32
        lib.orc_interval_usable.argtypes = [f32, i32, i32]
        lib.orc_interval_usable.restype = i32
        lib.orc_scale.argtypes = [f32, i32, i32]
        lib.orc_scale.restype = f64
        lib.orc_quantize.argtypes = [p, i64, f32, i32, i32, i32, u64, u64, p, p]
        lib.orc_pack_nibbles.argtypes = [p, i64, p]
        lib.orc_update_interval.argtypes = [p, f64, f64, f64, f64, i32, u64, u64]
        lib.orc_update_interval.restype = i32
        lib.orc_linear_dx.argtypes = [p, p, i64, i64, i64, p]
        lib.orc_linear_dw.argtypes = [p, p, i64, i64, i64, p]
        conv = [p, p] + [i64] * 9
        lib.orc_conv2d_dx.argtypes = conv + [p]
        lib.orc_conv2d_dw.argtypes = conv + [p]
        lib.orc_conv2d_dx_at.argtypes = conv + [p, i64, p]
        lib.orc_conv2d_dw_at.argtypes = conv + [p, i64, p]
        lib.orc_dequant.argtypes = [p, i64, f64, f64, p]
        _lib = lib
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _f32(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.float32, "oracle inputs are the same fp32 bits the GPU sees"
    return a


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def num_threads() -> int:
    return int(_L().orc_num_threads())


# ----------------------------------------------------------------------------
# primitives
# ----------------------------------------------------------------------------
def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    out = np.zeros(4, dtype=np.uint32)
    _L().orc_philox4x32_10(_ptr(c), _ptr(k), _ptr(out))
    return out


def r16(e: int, seed: int, step: int) -> int:
    return int(_L().orc_r16(e, seed, step))


def tensor_max(x, use_abs: bool = True):
    """(max |x| or max x as fp32, status)."""
    x = _f32(x)
    out = C.c_float(0.0)
    st = _L().orc_max(_ptr(x), x.size, int(use_abs), C.byref(out))
    return np.float32(out.value), int(st)


def clip_value(gamma: float, gmax) -> np.float32:
    return np.float32(_L().orc_clip_value(float(gamma), float(gmax)))


def levels(bits: int, is_unsigned: bool = False) -> int:
    return int(_L().orc_levels(bits, int(is_unsigned)))


def interval_usable(c, bits: int, is_unsigned: bool = False) -> bool:
    """False for c <= 0 and for c so small that q / c is not a finite fp32 number."""
    return bool(_L().orc_interval_usable(float(c), bits, int(is_unsigned)))


def scale(c, bits: int, is_unsigned: bool = False) -> float:
    return float(_L().orc_scale(float(c), bits, int(is_unsigned)))


def quantize(x, c, bits: int = 4, is_unsigned: bool = False, rounding: int = NEAREST,
             seed: int = 0, step: int = 0):
    """Eq. (1)-(4) with clip value c: (int32 codes shaped like x, clip-out count)."""
    x = _f32(x)
    code = np.empty(x.shape, dtype=np.int32)
    n_out = C.c_uint64(0)
    _L().orc_quantize(_ptr(x), x.size, float(c), bits, int(is_unsigned), rounding,
                      seed, step, _ptr(code), C.byref(n_out))
    return code, int(n_out.value)


def pack_nibbles(code) -> np.ndarray:
    code = _i32(code).reshape(-1)
    out = np.zeros((code.size + 1) // 2, dtype=np.uint8)
    _L().orc_pack_nibbles(_ptr(code), code.size, _ptr(out))
    return out


# ----------------------------------------------------------------------------
# per-layer gradient-quantizer state (the scalars of Alg. 1)
# ----------------------------------------------------------------------------
@dataclass
class GradState:
    gamma: float = 1.0
    alpha: float = 1e-3
    beta: float = 1e-3
    gamma_min: float = 1e-3
    gamma_max: float = 1.0
    bits: int = 4
    status: int = OK
    step: int = 0
    n_total: int = 0
    n_out: int = 0
    gmax: np.float32 = field(default_factory=lambda: np.float32(0))
    clip: np.float32 = field(default_factory=lambda: np.float32(0))
    scale: np.float32 = field(default_factory=lambda: np.float32(0))


def quantize_grad(g, st: GradState, seed: int = 0, rounding: int = NEAREST,
                  hindsight: bool = False):
    """Gradient quantizer of one layer: g_max, c_g = gamma*g_max, codes, N(G_out).

    Writes gmax, clip, scale, n_total, n_out, status into ``st``; gamma and step
    are left alone (the update is a separate call, as in Alg. 1 whose input is
    the clip-out set of the quantization just done).  Returns int32 codes.

    hindsight=True is NOT the paper's quantizer (Sec. 3.1 takes the maximum of the tensor
    being quantized): the interval comes from the maximum of the PREVIOUS tensor of this
    layer, st.gmax, so that one sweep over the tensor suffices; this tensor's maximum is
    recorded in st.gmax for the next call.  A separate, explicitly requested mode.
    """
    g = _f32(g)
    if hindsight:
        return _quantize_grad_hindsight(g, st, seed, rounding)
    gmax, status = tensor_max(g, use_abs=True)
    st.status = status
    st.n_total = int(g.size)
    if status == NONFINITE:
        return None
    c = clip_value(st.gamma, gmax) if status == OK else np.float32(0)
    if status == ZERO_GRAD or not interval_usable(c, st.bits):
        # all-zero tensor, or gradients of subnormal scale whose interval cannot be divided by
        st.status = ZERO_GRAD
        st.gmax = gmax
        st.clip = np.float32(0)
        st.scale = np.float32(0)
        st.n_out = 0
        return np.zeros(g.shape, dtype=np.int32)
    code, n_out = quantize(g, c, st.bits, False, rounding, seed, st.step)
    st.gmax, st.clip, st.n_out = gmax, c, n_out
    st.scale = np.float32(scale(c, st.bits, False))
    return code


def _quantize_grad_hindsight(g, st: GradState, seed: int, rounding: int):
    gmax_now, status_now = tensor_max(g, use_abs=True)
    st.n_total = int(g.size)
    prev = np.float32(st.gmax)
    if np.isfinite(prev) and prev > 0 and interval_usable(clip_value(st.gamma, prev), st.bits):
        c = clip_value(st.gamma, prev)
        code, n_out = quantize(g, c, st.bits, False, rounding, seed, st.step)
        status = OK
    else:                       # no usable previous maximum: everything is clipped to 0
        c, n_out, status = np.float32(0), 0, ZERO_GRAD
        code = np.zeros(g.shape, dtype=np.int32)
    if status_now == NONFINITE:
        status = NONFINITE      # and the recorded maximum stays what it was
    else:
        st.gmax = np.float32(gmax_now)
    st.clip, st.n_out, st.status = np.float32(c), int(n_out), status
    st.scale = np.float32(scale(c, st.bits, False)) if c > 0 else np.float32(0)
    return code


def update_interval(st: GradState) -> int:
    """Alg. 1 on the counts of the last quantize_grad; returns the sign used."""
    if st.status != OK:
        return 0
    g = C.c_double(st.gamma)
    sg = _L().orc_update_interval(C.byref(g), st.alpha, st.beta, st.gamma_min, st.gamma_max,
                                  st.bits, st.n_out, st.n_total)
    st.gamma = float(g.value)
    st.step += 1
    return int(sg)


def quantize_operand(x, c: float, is_unsigned: bool, bits: int = 4):
    """Weights / activations: Eq. (2) or (3), nearest rounding.

    c <= 0 selects the per-tensor maximum (max |x| signed, max x unsigned).
    Returns (codes, clip value fp32, scale double, status).
    """
    x = _f32(x)
    status = OK
    if not (c > 0):
        m, status = tensor_max(x, use_abs=not is_unsigned)
        if status == NONFINITE:
            return None, np.float32(0), 0.0, status
        c = m
        status = OK  # an all-zero operand is legal: codes 0, scale 0
    c = np.float32(c)
    code, _ = quantize(x, c, bits, is_unsigned, NEAREST)
    return code, c, scale(c, bits, is_unsigned), status


# ----------------------------------------------------------------------------
# integer contractions
# ----------------------------------------------------------------------------
def linear_dx(qG, qW):
    qG, qW = _i32(qG), _i32(qW)
    M, N = qG.shape
    K, N2 = qW.shape
    assert N == N2
    acc = np.empty((M, K), dtype=np.int64)
    _L().orc_linear_dx(_ptr(qG), _ptr(qW), M, K, N, _ptr(acc))
    return acc


def linear_dw(qX, qG):
    qX, qG = _i32(qX), _i32(qG)
    M, K = qX.shape
    M2, N = qG.shape
    assert M == M2
    acc = np.empty((K, N), dtype=np.int64)
    _L().orc_linear_dw(_ptr(qX), _ptr(qG), M, K, N, _ptr(acc))
    return acc


def _conv_dims(x_shape, w_shape, stride, pad):
    N, Cc, H, W = x_shape
    K, C2, R, S = w_shape
    assert Cc == C2
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    return N, Cc, H, W, K, R, S, P, Q


def conv2d_dx(qG, qW, x_shape, stride: int, pad: int):
    qG, qW = _i32(qG), _i32(qW)
    N, Cc, H, W, K, R, S, P, Q = _conv_dims(x_shape, qW.shape, stride, pad)
    assert qG.shape == (N, K, P, Q)
    acc = np.empty((N, Cc, H, W), dtype=np.int64)
    _L().orc_conv2d_dx(_ptr(qG), _ptr(qW), N, Cc, H, W, K, R, S, stride, pad, _ptr(acc))
    return acc


def conv2d_dw(qG, qX, w_shape, stride: int, pad: int):
    qG, qX = _i32(qG), _i32(qX)
    N, Cc, H, W, K, R, S, P, Q = _conv_dims(qX.shape, w_shape, stride, pad)
    assert qG.shape == (N, K, P, Q)
    acc = np.empty((K, Cc, R, S), dtype=np.int64)
    _L().orc_conv2d_dw(_ptr(qG), _ptr(qX), N, Cc, H, W, K, R, S, stride, pad, _ptr(acc))
    return acc


def conv2d_dx_at(qG, qW, x_shape, stride: int, pad: int, flat_idx):
    qG, qW = _i32(qG), _i32(qW)
    N, Cc, H, W, K, R, S, P, Q = _conv_dims(x_shape, qW.shape, stride, pad)
    idx = np.ascontiguousarray(flat_idx, dtype=np.int64)
    acc = np.empty(idx.size, dtype=np.int64)
    _L().orc_conv2d_dx_at(_ptr(qG), _ptr(qW), N, Cc, H, W, K, R, S, stride, pad,
                          _ptr(idx), idx.size, _ptr(acc))
    return acc


def conv2d_dw_at(qG, qX, w_shape, stride: int, pad: int, flat_idx):
    qG, qX = _i32(qG), _i32(qX)
    N, Cc, H, W, K, R, S, P, Q = _conv_dims(qX.shape, w_shape, stride, pad)
    idx = np.ascontiguousarray(flat_idx, dtype=np.int64)
    acc = np.empty(idx.size, dtype=np.int64)
    _L().orc_conv2d_dw_at(_ptr(qG), _ptr(qX), N, Cc, H, W, K, R, S, stride, pad,
                          _ptr(idx), idx.size, _ptr(acc))
    return acc


# ----------------------------------------------------------------------------
# Freivalds-style check of a WHOLE accumulator tensor handed in from elsewhere: the claimed
# result is contracted with a random +-1 vector along one axis, and the same contraction is
# pushed through the definition (the products are linear in each operand), which costs one
# product with that axis collapsed to length 1.  Integer arithmetic in int64: equality is
# exact.  A claimed tensor that is wrong at some position of the kept axes passes one
# vector with probability <= 1/2.
# ----------------------------------------------------------------------------
def signs(rng: np.random.Generator, n: int) -> np.ndarray:
    return (2 * rng.integers(0, 2, n, dtype=np.int64) - 1).astype(np.int64)


def freivalds_conv2d_dx(acc_dx, qG, qW, stride: int, pad: int, r_c):
    """sum_c r[c] acc_dX[n,c,h,w]  vs  dX of the one-channel filter  sum_c r[c] qW[k,c,r,s]
    (dX is linear in W).  Returns the two [N,H,W] arrays; the caller asserts equality."""
    acc = np.asarray(acc_dx)
    N, Cc, H, W = acc.shape
    r_c = np.asarray(r_c, dtype=np.int64)
    assert r_c.shape == (Cc,)
    got = np.tensordot(acc.astype(np.int64), r_c, axes=([1], [0]))
    w1 = np.tensordot(np.asarray(qW, dtype=np.int64), r_c, axes=([1], [0]))[:, None, :, :]
    want = conv2d_dx(qG, w1, (N, 1, H, W), stride, pad)[:, 0]
    return got, want


def freivalds_conv2d_dw(acc_dw, qG, qX, stride: int, pad: int, r_k):
    """sum_k r[k] acc_dW[k,c,r,s]  vs  dW of the one-channel gradient  sum_k r[k] qG[n,k,p,q]
    (dW is linear in dY).  Returns the two [C,R,S] arrays."""
    acc = np.asarray(acc_dw)
    K, Cc, R, S = acc.shape
    r_k = np.asarray(r_k, dtype=np.int64)
    assert r_k.shape == (K,)
    got = np.tensordot(r_k, acc.astype(np.int64), axes=([0], [0]))
    g1 = np.tensordot(np.asarray(qG, dtype=np.int64), r_k, axes=([1], [0]))[:, None, :, :]
    want = conv2d_dw(g1, qX, (1, Cc, R, S), stride, pad)[0]
    return got, want


def freivalds_linear(acc_dx, acc_dw, qG, qX, qW, r_k, r_n):
    """Linear layer: acc_dX[M,K] r_k  vs  qG (qW^T r_k);  acc_dW[K,N] r_n  vs  qX^T (qG r_n).
    Returns ((got, want) for dX or None, (got, want) for dW or None)."""
    qG, qW = np.asarray(qG, dtype=np.int64), np.asarray(qW, dtype=np.int64)
    out_dx = out_dw = None
    if acc_dx is not None:
        r_k = np.asarray(r_k, dtype=np.int64)
        out_dx = (np.asarray(acc_dx).astype(np.int64) @ r_k, qG @ (qW.T @ r_k))
    if acc_dw is not None:
        r_n = np.asarray(r_n, dtype=np.int64)
        qX = np.asarray(qX, dtype=np.int64)
        out_dw = (np.asarray(acc_dw).astype(np.int64) @ r_n, qX.T @ (qG @ r_n))
    return out_dx, out_dw


def dequant(acc, s_a: float, s_b: float) -> np.ndarray:
    acc = np.ascontiguousarray(acc, dtype=np.int64)
    out = np.empty(acc.shape, dtype=np.float32)
    _L().orc_dequant(_ptr(acc), acc.size, float(s_a), float(s_b), _ptr(out))
    return out


# ----------------------------------------------------------------------------
# whole-layer backward, in the order of the method
# ----------------------------------------------------------------------------
@dataclass
class BackwardResult:
    qG: np.ndarray
    qX: np.ndarray
    qW: np.ndarray
    s_g: float
    s_x: float
    s_w: float
    acc_dx: np.ndarray | None
    acc_dw: np.ndarray | None
    dX: np.ndarray | None
    dW: np.ndarray | None


def _operands(X, W, dY, c_x, x_unsigned, c_w, st, seed, rounding, hindsight=False):
    qG = quantize_grad(dY, st, seed, rounding, hindsight)
    if st.status == NONFINITE:
        return None
    s_g = scale(st.clip, st.bits, False)
    qX, _, s_x, sx_status = quantize_operand(X, c_x, bool(x_unsigned), st.bits)
    qW, _, s_w, sw_status = quantize_operand(W, c_w, False, st.bits)
    if sx_status == NONFINITE or sw_status == NONFINITE:
        st.status = NONFINITE
        return None
    return qG, qX, qW, s_g, s_x, s_w


def backward_linear(X, W, dY, st: GradState, c_x: float = 0.0, x_unsigned: bool = False,
                    c_w: float = 0.0, seed: int = 0, rounding: int = NEAREST,
                    want_dx: bool = True, want_dw: bool = True, hindsight: bool = False):
    """X[M,K], W[K,N], dY[M,N]: dX = Q(dY).Q(W)^T, dW = Q(X)^T.Q(dY)."""
    ops = _operands(X, W, dY, c_x, x_unsigned, c_w, st, seed, rounding, hindsight)
    if ops is None:
        return None
    qG, qX, qW, s_g, s_x, s_w = ops
    acc_dx = linear_dx(qG, qW) if want_dx else None
    acc_dw = linear_dw(qX, qG) if want_dw else None
    for a in (acc_dx, acc_dw):
        assert a is None or np.abs(a).max(initial=0) < 2 ** 31
    return BackwardResult(qG, qX, qW, s_g, s_x, s_w, acc_dx, acc_dw,
                          dequant(acc_dx, s_g, s_w) if want_dx else None,
                          dequant(acc_dw, s_x, s_g) if want_dw else None)


def backward_conv2d(X, W, dY, stride: int, pad: int, st: GradState, c_x: float = 0.0,
                    x_unsigned: bool = True, c_w: float = 0.0, seed: int = 0,
                    rounding: int = NEAREST, want_dx: bool = True, want_dw: bool = True,
                    hindsight: bool = False):
    """X[N,C,H,W], W[K,C,R,S], dY[N,K,P,Q]: both gradients of the convolution."""
    ops = _operands(X, W, dY, c_x, x_unsigned, c_w, st, seed, rounding, hindsight)
    if ops is None:
        return None
    qG, qX, qW, s_g, s_x, s_w = ops
    acc_dx = conv2d_dx(qG, qW, X.shape, stride, pad) if want_dx else None
    acc_dw = conv2d_dw(qG, qX, W.shape, stride, pad) if want_dw else None
    for a in (acc_dx, acc_dw):
        assert a is None or np.abs(a).max(initial=0) < 2 ** 31
    return BackwardResult(qG, qX, qW, s_g, s_x, s_w, acc_dx, acc_dw,
                          dequant(acc_dx, s_g, s_w) if want_dx else None,
                          dequant(acc_dw, s_x, s_g) if want_dw else None)


# ----------------------------------------------------------------------------
# quantized forward pass (Sec. 3.1: weights and activations quantized with Eq. 2 / 3 before
# the layer's product; Eq. 4 denormalises the integer result).  Written out as the plain
# definition in numpy int64: Y = s_x s_w * sum qX qW.
# ----------------------------------------------------------------------------
def linear_fwd(qX, qW):
    """acc[m, n] = sum_k qX[m, k] * qW[k, n]."""
    qX, qW = np.asarray(qX, dtype=np.int64), np.asarray(qW, dtype=np.int64)
    assert qX.shape[1] == qW.shape[0]
    return qX @ qW


def conv2d_fwd(qX, qW, stride: int, pad: int):
    """Cross-correlation with zero padding:
    acc[n, k, p, q] = sum_{c, r, s} qW[k, c, r, s] * qX[n, c, p*stride - pad + r, q*stride - pad + s]."""
    qX, qW = np.asarray(qX, dtype=np.int64), np.asarray(qW, dtype=np.int64)
    N, Cc, H, W, K, R, S, P, Q = _conv_dims(qX.shape, qW.shape, stride, pad)
    xp = np.zeros((N, Cc, H + 2 * pad, W + 2 * pad), dtype=np.int64)
    xp[:, :, pad:pad + H, pad:pad + W] = qX
    acc = np.zeros((N, K, P, Q), dtype=np.int64)
    for r in range(R):
        for s in range(S):
            window = xp[:, :, r:r + stride * (P - 1) + 1:stride, s:s + stride * (Q - 1) + 1:stride]
            acc += np.einsum("ncpq,kc->nkpq", window, qW[:, :, r, s])
    return acc


def conv2d_fwd_at(qX, qW, stride: int, pad: int, flat_idx):
    """The same sum for single output positions (flat indices into [N, K, P, Q]), one by one."""
    qX, qW = np.asarray(qX), np.asarray(qW)
    N, Cc, H, W, K, R, S, P, Q = _conv_dims(qX.shape, qW.shape, stride, pad)
    out = np.empty(len(flat_idx), dtype=np.int64)
    for i, f in enumerate(np.asarray(flat_idx, dtype=np.int64)):
        n, k, p, q = np.unravel_index(int(f), (N, K, P, Q))
        total = 0
        for r in range(R):
            h = p * stride - pad + r
            if h < 0 or h >= H:
                continue
            for s in range(S):
                w = q * stride - pad + s
                if w < 0 or w >= W:
                    continue
                total += int(np.dot(qW[k, :, r, s].astype(np.int64), qX[n, :, h, w].astype(np.int64)))
        out[i] = total
    return out


@dataclass
class ForwardResult:
    qX: np.ndarray
    qW: np.ndarray
    s_x: float
    s_w: float
    status: int
    acc: np.ndarray | None
    Y: np.ndarray | None


def _forward_operands(X, W, c_x, x_unsigned, c_w, bits):
    qX, _, s_x, sx_status = quantize_operand(X, c_x, bool(x_unsigned), bits)
    qW, _, s_w, sw_status = quantize_operand(W, c_w, False, bits)
    status = NONFINITE if NONFINITE in (sx_status, sw_status) else OK
    return qX, qW, s_x, s_w, status


def forward_linear(X, W, c_x: float = 0.0, x_unsigned: bool = False, c_w: float = 0.0,
                   bits: int = 4):
    """X[M,K], W[K,N]: Y = Q(X) . Q(W), denormalised."""
    qX, qW, s_x, s_w, status = _forward_operands(X, W, c_x, x_unsigned, c_w, bits)
    if status != OK:
        return ForwardResult(qX, qW, s_x, s_w, status, None, None)
    acc = linear_fwd(qX, qW)
    return ForwardResult(qX, qW, s_x, s_w, status, acc, dequant(acc, s_x, s_w))


def forward_conv2d(X, W, stride: int, pad: int, c_x: float = 0.0, x_unsigned: bool = True,
                   c_w: float = 0.0, bits: int = 4):
    """X[N,C,H,W], W[K,C,R,S]: Y[N,K,P,Q] = conv(Q(X), Q(W)), denormalised."""
    qX, qW, s_x, s_w, status = _forward_operands(X, W, c_x, x_unsigned, c_w, bits)
    if status != OK:
        return ForwardResult(qX, qW, s_x, s_w, status, None, None)
    acc = conv2d_fwd(qX, qW, stride, pad)
    return ForwardResult(qX, qW, s_x, s_w, status, acc, dequant(acc, s_x, s_w))


# ----------------------------------------------------------------------------
# learned clip values of the weight / activation quantizers (Sec. 3.1)
# ----------------------------------------------------------------------------
def ste_backward(x, c, is_unsigned: bool, bits: int, grad_q):
    """Gradient of a loss through the quantizer of Eq. (1)-(4), w.r.t. the input x and w.r.t.
    the clip value c, given grad_q = dL/dQ(x).

    Sec. 3.1 learns c for weights and activations end to end, following the learned-step-size
    and clipping-activation quantizers it cites, and prints no formula of its own.  The reading
    taken here is the derivative of Eq. (1)-(4) with the rounding passed straight through
    (d round(u)/du = 1), Q = s round(u), u = clip(x, c)/s, s = c/q:
        dQ/dx = 1 for lo < x < c, else 0                        (lo = -c signed, 0 unsigned)
        dQ/dc = (round(u) - u)/q inside;  +1 for x >= c;  -1 for x <= -c (signed);
                0 for x <= 0 (unsigned)
    which is the step-size gradient of the learned-step-size quantizer divided by q.
    round(u) is taken as the operand quantizer takes it (u as one fp32 multiply by q/c);
    everything after that decision is fp64.  Returns (grad_x fp32 shaped like x, grad_c as a
    Python float, sum of |grad_q * dQ/dc| as a Python float: the scale of grad_c's error)."""
    x = _f32(x)
    g = _f32(grad_q)
    assert x.shape == g.shape
    c = np.float32(c)
    assert interval_usable(c, bits, is_unsigned)
    q = levels(bits, is_unsigned)
    inv_s = np.float32(np.float64(q) / np.float64(c))
    lo = np.float32(0.0) if is_unsigned else np.float32(-c)
    inside = (x > lo) & (x < c)
    with np.errstate(invalid="ignore"):
        xc = np.minimum(np.maximum(x, lo), c)
        u = (xc * inv_s).astype(np.float32)
        r = np.rint(u)
    below = np.float64(0.0 if is_unsigned else -1.0)
    d_c = np.where(inside, (r.astype(np.float64) - u.astype(np.float64)) / np.float64(q),
                   np.where(x >= c, 1.0, np.where(x <= lo, below, 0.0)))
    prod = g.astype(np.float64) * d_c
    grad_x = np.where(inside, g, np.float32(0.0)).astype(np.float32)
    return grad_x, float(np.sum(prod)), float(np.sum(np.abs(prod)))

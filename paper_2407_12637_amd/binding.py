"""ctypes binding of liblbt.so: argument marshalling only.

Every function here has the name of the C entry point it calls (see
include/lbt.h); tensors are torch CUDA tensors used as device-memory handles,
the stream is torch's current stream.  Nothing is computed in Python, and
there is no fallback: a missing library raises at import of the symbol table.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblbt.so")

OK = 0
ROUND_NEAREST, ROUND_STOCHASTIC = 0, 1
HINDSIGHT_MAX = 2  # may be OR-ed into `rounding`: interval from the previous tensor's maximum
FUSED_UPDATE = 4   # may be OR-ed into `rounding`: the call also applies the interval update (Alg. 1)


def BITS(b: int) -> int:
    """LBT_BITS(b): the bit-width field of the `rounding` flag word (absent = 4)."""
    return (b & 15) << 8


STATUS_OK, STATUS_NONFINITE, STATUS_ZERO_GRAD = 0, 1, 2


class LbtError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s failed: %s (%d)" % (where, strerror(code), code))


class GradState(C.Structure):
    """Mirror of lbt_grad_state (96 bytes)."""
    _fields_ = [
        ("gamma", C.c_double), ("alpha", C.c_double), ("beta", C.c_double),
        ("gamma_min", C.c_double), ("gamma_max", C.c_double),
        ("bits", C.c_int32), ("status", C.c_int32),
        ("step", C.c_uint64), ("n_total", C.c_uint64), ("n_out", C.c_uint64),
        ("sync_word", C.c_uint64),
        ("gmax", C.c_float), ("clip", C.c_float), ("scale", C.c_float),
        ("sync_max", C.c_uint32),
    ]


_lib = None

_i64, _u64, _f32, _f64, _int, _p, _sz = (C.c_int64, C.c_uint64, C.c_float, C.c_double, C.c_int,
                                         C.c_void_p, C.c_size_t)

SIGNATURES = {
    "lbt_version": (C.c_char_p, []),
    "lbt_strerror": (C.c_char_p, [_int]),
    "lbt_state_sizeof": (_sz, []),
    "lbt_state_init": (_int, [_p, _f64, _f64, _f64, _f64, _f64, _int, _p]),
    "lbt_state_read": (_int, [_p, _p, _p]),
    "lbt_state_write": (_int, [_p, _p, _p]),
    "lbt_update_interval": (_int, [_p, _p]),
    "lbt_quantize_grad": (_int, [_p, _i64, _p, _u64, _int, _p, _p, _sz, _p]),
    "lbt_workspace_bytes_quantize": (_sz, [_i64]),
    "lbt_quantize_grad_static": (_int, [_p, _i64, _p, _u64, _int, _p, _p]),
    "lbt_quantize_operand": (_int, [_p, _i64, _f32, _int, _int, _p, _p, _p, _sz, _p]),
    "lbt_backward_linear_learned": (_int, [_p, _p, _p, _i64, _i64, _i64, _f32, _int, _f32, _p, _u64,
                                           _int, _p, _p, _p, _p, _sz, _p]),
    "lbt_backward_conv2d_learned": (_int, [_p, _p, _p] + [_i64] * 9 + [_f32, _int, _f32, _p, _u64,
                                                                       _int, _p, _p, _p, _p, _sz, _p]),
    "lbt_ste_backward": (_int, [_p, _i64, _f32, _int, _int, _p, _p, _p, _p, _sz, _p]),
    "lbt_backward_linear": (_int, [_p, _p, _p, _i64, _i64, _i64, _f32, _int, _f32, _p, _u64, _int,
                                   _p, _p, _p, _sz, _p]),
    "lbt_workspace_bytes_linear": (_sz, [_i64, _i64, _i64]),
    "lbt_backward_conv2d": (_int, [_p, _p, _p] + [_i64] * 9 + [_f32, _int, _f32, _p, _u64, _int,
                                                               _p, _p, _p, _sz, _p]),
    "lbt_workspace_bytes_conv2d": (_sz, [_i64] * 9),
    "lbt_backward_linear_acc": (_int, [_p, _p, _p, _i64, _i64, _i64, _f32, _int, _f32, _p, _u64,
                                       _int, _p, _p, _p, _p, _p, _sz, _p]),
    "lbt_backward_conv2d_acc": (_int, [_p, _p, _p] + [_i64] * 9 + [_f32, _int, _f32, _p, _u64, _int,
                                                                   _p, _p, _p, _p, _p, _sz, _p]),
    "lbt_forward_linear": (_int, [_p, _p, _i64, _i64, _i64, _f32, _int, _f32, _int, _p, _p, _p, _p,
                                  _sz, _p]),
    "lbt_workspace_bytes_forward_linear": (_sz, [_i64, _i64, _i64]),
    "lbt_forward_conv2d": (_int, [_p, _p] + [_i64] * 9 + [_f32, _int, _f32, _int, _p, _p, _p, _p,
                                                          _sz, _p]),
    "lbt_workspace_bytes_forward_conv2d": (_sz, [_i64] * 9),
    "lbt_saved_bytes_linear": (_sz, [_i64, _i64, _i64]),
    "lbt_saved_bytes_conv2d": (_sz, [_i64] * 9),
    "lbt_forward_linear_save": (_int, [_p, _p, _i64, _i64, _i64, _f32, _int, _f32, _int, _p, _p, _p,
                                       _p, _sz, _p, _sz, _p]),
    "lbt_forward_conv2d_save": (_int, [_p, _p] + [_i64] * 9 + [_f32, _int, _f32, _int, _p, _p, _p,
                                                               _p, _sz, _p, _sz, _p]),
    "lbt_backward_linear_saved": (_int, [_p, _sz, _p, _i64, _i64, _i64, _int, _p, _u64, _int,
                                         _p, _p, _p, _p, _p, _sz, _p]),
    "lbt_backward_conv2d_saved": (_int, [_p, _sz, _p] + [_i64] * 9 + [_int, _p, _u64, _int,
                                                                      _p, _p, _p, _p, _p, _sz, _p]),
    "lbt_profile_enable": (_int, [_int]),
    "lbt_profile_skeleton": (_int, [_int]),
    "lbt_profile_kernel_count": (_int, []),
    "lbt_profile_kernel_name": (C.c_char_p, [_int]),
    "lbt_profile_read": (_int, [_p, _p, _p, _int]),
}


def load():
    """Load liblbt.so and declare every exported symbol.  Raises if it is not built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                "liblbt.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def strerror(code: int) -> str:
    return load().lbt_strerror(code).decode()


def _check(code: int, where: str):
    if code != OK:
        raise LbtError(code, where)


def _dp(t):
    """Device pointer of a tensor (None -> NULL)."""
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous()
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def lbt_version() -> str:
    return load().lbt_version().decode()


def lbt_state_sizeof() -> int:
    return int(load().lbt_state_sizeof())


def new_state(gamma0=1.0, alpha=1e-3, beta=1e-3, gamma_min=None, gamma_max=1.0, bits=4,
              device="cuda"):
    """Allocate a device state and initialise it with lbt_state_init."""
    st = torch.empty(lbt_state_sizeof(), dtype=torch.uint8, device=device)
    lbt_state_init(st, gamma0, alpha, beta, beta if gamma_min is None else gamma_min, gamma_max,
                   bits)
    return st


def lbt_state_init(st, gamma0, alpha, beta, gamma_min, gamma_max, bits):
    _check(load().lbt_state_init(_dp(st), gamma0, alpha, beta, gamma_min, gamma_max, bits,
                                 _stream()), "lbt_state_init")


def lbt_state_read(st) -> GradState:
    host = GradState()
    _check(load().lbt_state_read(_dp(st), C.addressof(host), _stream()), "lbt_state_read")
    return host


def lbt_state_write(st, host: GradState):
    _check(load().lbt_state_write(_dp(st), C.addressof(host), _stream()), "lbt_state_write")


def lbt_update_interval(st):
    _check(load().lbt_update_interval(_dp(st), _stream()), "lbt_update_interval")


def lbt_workspace_bytes_quantize(n: int) -> int:
    return int(load().lbt_workspace_bytes_quantize(n))


def lbt_workspace_bytes_linear(M, K_in, N_out) -> int:
    return int(load().lbt_workspace_bytes_linear(M, K_in, N_out))


def lbt_workspace_bytes_conv2d(N, Cc, H, W, K, R, S, stride, pad) -> int:
    return int(load().lbt_workspace_bytes_conv2d(N, Cc, H, W, K, R, S, stride, pad))


def _ws_args(ws):
    return _dp(ws), (ws.numel() * ws.element_size() if ws is not None else 0)


def lbt_quantize_grad(g, st, seed, rounding, codes, ws):
    wp, wb = _ws_args(ws)
    _check(load().lbt_quantize_grad(_dp(g), g.numel(), _dp(st), seed, rounding, _dp(codes), wp, wb,
                                    _stream()), "lbt_quantize_grad")


def lbt_quantize_grad_static(g, st, seed, rounding, codes):
    _check(load().lbt_quantize_grad_static(_dp(g), g.numel(), _dp(st), seed, rounding, _dp(codes),
                                           _stream()), "lbt_quantize_grad_static")


def lbt_quantize_operand(x, c, is_unsigned, bits, codes, clip_scale_out, ws):
    wp, wb = _ws_args(ws)
    _check(load().lbt_quantize_operand(_dp(x), x.numel(), c, int(is_unsigned), bits, _dp(codes),
                                       _dp(clip_scale_out), wp, wb, _stream()),
           "lbt_quantize_operand")


def lbt_backward_linear(X, W, dY, M, K_in, N_out, c_x, x_unsigned, c_w, st, seed, rounding, dX, dW,
                        ws):
    wp, wb = _ws_args(ws)
    _check(load().lbt_backward_linear(_dp(X), _dp(W), _dp(dY), M, K_in, N_out, c_x, int(x_unsigned),
                                      c_w, _dp(st), seed, rounding, _dp(dX), _dp(dW), wp, wb,
                                      _stream()), "lbt_backward_linear")


def lbt_backward_conv2d(X, W, dY, N, Cc, H, Wd, K, R, S, stride, pad, c_x, x_unsigned, c_w, st,
                        seed, rounding, dX, dW, ws):
    wp, wb = _ws_args(ws)
    _check(load().lbt_backward_conv2d(_dp(X), _dp(W), _dp(dY), N, Cc, H, Wd, K, R, S, stride, pad,
                                      c_x, int(x_unsigned), c_w, _dp(st), seed, rounding, _dp(dX),
                                      _dp(dW), wp, wb, _stream()), "lbt_backward_conv2d")


def lbt_backward_linear_acc(X, W, dY, M, K_in, N_out, c_x, x_unsigned, c_w, st, seed, rounding, dX,
                            dW, acc_dX, acc_dW, ws):
    wp, wb = _ws_args(ws)
    _check(load().lbt_backward_linear_acc(_dp(X), _dp(W), _dp(dY), M, K_in, N_out, c_x,
                                          int(x_unsigned), c_w, _dp(st), seed, rounding, _dp(dX),
                                          _dp(dW), _dp(acc_dX), _dp(acc_dW), wp, wb, _stream()),
           "lbt_backward_linear_acc")


def lbt_backward_conv2d_acc(X, W, dY, N, Cc, H, Wd, K, R, S, stride, pad, c_x, x_unsigned, c_w, st,
                            seed, rounding, dX, dW, acc_dX, acc_dW, ws):
    wp, wb = _ws_args(ws)
    _check(load().lbt_backward_conv2d_acc(_dp(X), _dp(W), _dp(dY), N, Cc, H, Wd, K, R, S, stride,
                                          pad, c_x, int(x_unsigned), c_w, _dp(st), seed, rounding,
                                          _dp(dX), _dp(dW), _dp(acc_dX), _dp(acc_dW), wp, wb,
                                          _stream()), "lbt_backward_conv2d_acc")


def lbt_workspace_bytes_forward_linear(M, K_in, N_out) -> int:
    return load().lbt_workspace_bytes_forward_linear(M, K_in, N_out)


def lbt_workspace_bytes_forward_conv2d(N, Cc, H, W, K, R, S, stride, pad) -> int:
    return load().lbt_workspace_bytes_forward_conv2d(N, Cc, H, W, K, R, S, stride, pad)


def lbt_forward_linear(X, W, M, K_in, N_out, c_x, x_unsigned, c_w, flags, Y, acc_Y, status, ws):
    wp, wb = _ws_args(ws)
    _check(load().lbt_forward_linear(_dp(X), _dp(W), M, K_in, N_out, c_x, int(x_unsigned), c_w,
                                     flags, _dp(Y), _dp(acc_Y), _dp(status), wp, wb, _stream()),
           "lbt_forward_linear")


def lbt_forward_conv2d(X, W, N, Cc, H, Wd, K, R, S, stride, pad, c_x, x_unsigned, c_w, flags, Y,
                       acc_Y, status, ws):
    wp, wb = _ws_args(ws)
    _check(load().lbt_forward_conv2d(_dp(X), _dp(W), N, Cc, H, Wd, K, R, S, stride, pad, c_x,
                                     int(x_unsigned), c_w, flags, _dp(Y), _dp(acc_Y), _dp(status),
                                     wp, wb, _stream()), "lbt_forward_conv2d")


def lbt_ste_backward(x, c, is_unsigned, bits, grad_q, grad_x, grad_c, ws):
    wp, wb = _ws_args(ws)
    _check(load().lbt_ste_backward(_dp(x), x.numel(), c, int(is_unsigned), bits, _dp(grad_q),
                                   _dp(grad_x), _dp(grad_c), wp, wb, _stream()), "lbt_ste_backward")


def lbt_backward_linear_learned(X, W, dY, M, K_in, N_out, c_x, x_unsigned, c_w, st, seed, rounding,
                                dX, dW, grad_c, ws):
    wp, wb = _ws_args(ws)
    _check(load().lbt_backward_linear_learned(_dp(X), _dp(W), _dp(dY), M, K_in, N_out, c_x,
                                              int(x_unsigned), c_w, _dp(st), seed, rounding,
                                              _dp(dX), _dp(dW), _dp(grad_c), wp, wb, _stream()),
           "lbt_backward_linear_learned")


def lbt_backward_conv2d_learned(X, W, dY, N, Cc, H, Wd, K, R, S, stride, pad, c_x, x_unsigned, c_w,
                                st, seed, rounding, dX, dW, grad_c, ws):
    wp, wb = _ws_args(ws)
    _check(load().lbt_backward_conv2d_learned(_dp(X), _dp(W), _dp(dY), N, Cc, H, Wd, K, R, S,
                                              stride, pad, c_x, int(x_unsigned), c_w, _dp(st), seed,
                                              rounding, _dp(dX), _dp(dW), _dp(grad_c), wp, wb,
                                              _stream()), "lbt_backward_conv2d_learned")


def lbt_saved_bytes_linear(M, K_in, N_out) -> int:
    return load().lbt_saved_bytes_linear(M, K_in, N_out)


def lbt_saved_bytes_conv2d(N, Cc, H, W, K, R, S, stride, pad) -> int:
    return load().lbt_saved_bytes_conv2d(N, Cc, H, W, K, R, S, stride, pad)


def lbt_forward_linear_save(X, W, M, K_in, N_out, c_x, x_unsigned, c_w, flags, Y, acc_Y, status,
                            saved, ws):
    """Y (and ws) may be None: only the codes for the backward call are produced."""
    wp, wb = _ws_args(ws) if ws is not None else (None, 0)
    sp, sb = _ws_args(saved)
    _check(load().lbt_forward_linear_save(_dp(X), _dp(W), M, K_in, N_out, c_x, int(x_unsigned), c_w,
                                          flags, _dp(Y), _dp(acc_Y), _dp(status), sp, sb, wp, wb,
                                          _stream()), "lbt_forward_linear_save")


def lbt_forward_conv2d_save(X, W, N, Cc, H, Wd, K, R, S, stride, pad, c_x, x_unsigned, c_w, flags,
                            Y, acc_Y, status, saved, ws):
    wp, wb = _ws_args(ws) if ws is not None else (None, 0)
    sp, sb = _ws_args(saved)
    _check(load().lbt_forward_conv2d_save(_dp(X), _dp(W), N, Cc, H, Wd, K, R, S, stride, pad, c_x,
                                          int(x_unsigned), c_w, flags, _dp(Y), _dp(acc_Y),
                                          _dp(status), sp, sb, wp, wb, _stream()),
           "lbt_forward_conv2d_save")


def lbt_backward_linear_saved(saved, dY, M, K_in, N_out, x_unsigned, st, seed, rounding, dX, dW,
                              acc_dX, acc_dW, ws):
    wp, wb = _ws_args(ws)
    sp, sb = _ws_args(saved)
    _check(load().lbt_backward_linear_saved(sp, sb, _dp(dY), M, K_in, N_out, int(x_unsigned),
                                            _dp(st), seed, rounding, _dp(dX), _dp(dW), _dp(acc_dX),
                                            _dp(acc_dW), wp, wb, _stream()),
           "lbt_backward_linear_saved")


def lbt_backward_conv2d_saved(saved, dY, N, Cc, H, Wd, K, R, S, stride, pad, x_unsigned, st, seed,
                              rounding, dX, dW, acc_dX, acc_dW, ws):
    wp, wb = _ws_args(ws)
    sp, sb = _ws_args(saved)
    _check(load().lbt_backward_conv2d_saved(sp, sb, _dp(dY), N, Cc, H, Wd, K, R, S, stride, pad,
                                            int(x_unsigned), _dp(st), seed, rounding, _dp(dX),
                                            _dp(dW), _dp(acc_dX), _dp(acc_dW), wp, wb, _stream()),
           "lbt_backward_conv2d_saved")


def lbt_profile_enable(on: bool):
    _check(load().lbt_profile_enable(int(on)), "lbt_profile_enable")


def lbt_profile_skeleton(on: bool):
    _check(load().lbt_profile_skeleton(int(on)), "lbt_profile_skeleton")


def lbt_profile_read():
    """{kernel class name: (launches, total ms, total algorithmic work)} since the last read."""
    lib = load()
    n = lib.lbt_profile_kernel_count()
    launches = (C.c_int64 * n)()
    ms = (C.c_double * n)()
    work = (C.c_double * n)()
    _check(lib.lbt_profile_read(launches, ms, work, n), "lbt_profile_read")
    return {lib.lbt_profile_kernel_name(i).decode(): (int(launches[i]), float(ms[i]), float(work[i]))
            for i in range(n)}

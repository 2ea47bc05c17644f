"""lbt_quantize_grad_static (the entry point that allocates nothing: scratch in a static
device array) against lbt_quantize_grad (scratch in the caller's workspace) through the C ABI:
codes and every field of the state must be equal bit for bit, on two calls in a row, the
second on a smaller tensor (the array keeps the first call's contents), then on further
sizes, roundings and modes; the call must not change the amount of allocated device memory."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2407_12637_amd import binding as lbt
from paper_2407_12637_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)


def _state_bytes(st):
    return bytes(lbt.lbt_state_read(st))


_warm = [False]   # the first static call on the device looks up the array's address


def _both(g, gamma, seed, rounding, step=0):
    """(codes, state) of the workspace call and of the static call on the same input."""
    n = g.size
    bits = ((rounding >> 8) & 15) or 4
    out = []
    gd = gu.dev(g.reshape(-1))
    for static in (False, True):
        st = lbt.new_state(gamma0=gamma)
        if step:
            h = lbt.lbt_state_read(st)
            h.step = step
            lbt.lbt_state_write(st, h)
        codes = torch.full((n if bits > 4 else (n + 1) // 2,), 0xEE, dtype=torch.uint8, device=gu.DEV)
        if static:
            torch.cuda.synchronize()
            before = torch.cuda.mem_get_info()[0]       # free device memory, as the driver sees it
            lbt.lbt_quantize_grad_static(gd, st, seed, rounding, codes)
            torch.cuda.synchronize()
            if _warm[0]:
                assert torch.cuda.mem_get_info()[0] == before
            _warm[0] = True
        else:
            ws = torch.zeros(lbt.lbt_workspace_bytes_quantize(n), dtype=torch.uint8, device=gu.DEV)
            lbt.lbt_quantize_grad(gd, st, seed, rounding, codes, ws)
        out.append((codes.cpu().numpy(), _state_bytes(st)))
    return out


def test_static_scratch_matches_workspace_call_twice_in_a_row():
    r = synth.rng(0, 77, 0, synth.T_DY)
    first = True
    # a large tensor (many partial maxima, every arrival counter used), then a smaller one
    for n, gamma, rounding in (((1 << 22) + 5, 0.05, 1), (70001, 0.3, 1), (9, 1.0, 0),
                               (1 << 20, 0.02, 0), (333, 0.5, 1 | lbt.BITS(8)),
                               (65536, 0.1, 1 | lbt.FUSED_UPDATE)):
        _say("static scratch", n, gamma, rounding)
        g = synth.grad_cfg4(r, (n,))
        (cw, sw), (cs, ss) = _both(g, gamma, 0x1234ABCD, rounding, step=2)
        assert np.array_equal(cw, cs), "codes differ"
        assert sw == ss, "state differs"
        if first:
            assert lbt.GradState.from_buffer_copy(ss).n_out > 0   # a real quantization happened
            first = False


def test_static_scratch_single_sweep_mode_and_degenerate_inputs():
    r = synth.rng(0, 77, 1, synth.T_DY)
    st_w, st_s = lbt.new_state(gamma0=0.2), lbt.new_state(gamma0=0.2)
    for it, n in enumerate((50000, 1 << 21, 4097)):
        _say("static scratch, single sweep", n)
        g = gu.dev(synth.grad_cfg4(r, (n,)))
        cw = torch.zeros((n + 1) // 2, dtype=torch.uint8, device=gu.DEV)
        cs = torch.zeros_like(cw)
        ws = torch.zeros(lbt.lbt_workspace_bytes_quantize(n), dtype=torch.uint8, device=gu.DEV)
        flags = lbt.ROUND_STOCHASTIC | lbt.HINDSIGHT_MAX | lbt.FUSED_UPDATE
        lbt.lbt_quantize_grad(g, st_w, 5, flags, cw, ws)
        lbt.lbt_quantize_grad_static(g, st_s, 5, flags, cs)
        assert torch.equal(cw, cs) and _state_bytes(st_w) == _state_bytes(st_s)
    for bad in (0.0, float("nan")):
        g = torch.full((1000,), bad, device=gu.DEV)
        codes = torch.full((500,), 0xEE, dtype=torch.uint8, device=gu.DEV)
        st = lbt.new_state(gamma0=0.5)
        lbt.lbt_quantize_grad_static(g, st, 0, 0, codes)
        h = lbt.lbt_state_read(st)
        assert h.status == (lbt.STATUS_ZERO_GRAD if bad == 0.0 else lbt.STATUS_NONFINITE)


def test_static_scratch_rejects_sizes_beyond_its_limit():
    lib = lbt.load()
    p = C.c_void_p(4096)
    too_many = (1 << 30) + 1
    assert lib.lbt_quantize_grad_static(p, too_many, p, 0, 0, p, None) == -8
    assert b"static scratch" in lib.lbt_strerror(-8)
    assert lib.lbt_quantize_grad_static(p, 0, p, 0, 0, p, None) == -2
    assert lib.lbt_quantize_grad_static(None, 8, p, 0, 0, p, None) == -1

"""CPU-side checks of the boundary: the library loads and exports every symbol the
header declares, the binding's struct mirrors the C struct, and host-side
validation rejects bad arguments without touching a GPU."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "lbt.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2407_12637_amd import binding, build
    if not os.path.exists(build.LIB):
        build.build(force=True)
    return binding.load()


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lbt_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_exported(lib):
    names = _declared_functions()
    assert {"lbt_update_interval", "lbt_quantize_grad", "lbt_backward_linear",
            "lbt_backward_conv2d"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name


def test_binding_declares_every_symbol():
    from paper_2407_12637_amd import binding
    assert sorted(binding.SIGNATURES) == _declared_functions()


def test_state_struct_size(lib):
    from paper_2407_12637_amd import binding
    assert lib.lbt_state_sizeof() == C.sizeof(binding.GradState) == 96
    assert binding.GradState.gmax.offset == 80 and binding.GradState.step.offset == 48


def test_strerror_and_version(lib):
    assert lib.lbt_strerror(0) == b"ok"
    assert b"workspace" in lib.lbt_strerror(-4)
    assert lib.lbt_version().startswith(b"lbt-gfx950")


def test_host_validation_rejects_without_gpu(lib):
    # these return before any HIP call
    assert lib.lbt_update_interval(None, None) == -1
    assert lib.lbt_quantize_grad(None, 8, None, 0, 0, None, None, 0, None) == -1
    assert lib.lbt_state_init(C.c_void_p(256), 1.0, 1e-3, 1e-3, 1e-3, 1.0, 9, None) == -3
    assert lib.lbt_state_init(C.c_void_p(256), 1.0, 1e-3, 1e-3, 1e-3, 1.0, 1, None) == -3
    assert lib.lbt_state_init(C.c_void_p(256), 2.0, 1e-3, 1e-3, 1e-3, 1.0, 4, None) == -2
    p = C.c_void_p(4096)
    big = 1 << 20
    assert lib.lbt_quantize_grad(p, 0, p, 0, 0, p, p, big, None) == -2          # n <= 0
    assert lib.lbt_quantize_grad(p, 8, p, 0, 8, p, p, big, None) == -3          # rounding bits
    assert lib.lbt_quantize_grad(C.c_void_p(4100), 8, p, 0, 0, p, p, big, None) == -7
    assert lib.lbt_quantize_grad(p, 8, p, 0, 0, p, p, 16, None) == -4           # workspace
    assert lib.lbt_workspace_bytes_quantize(8) == 256 + 2048 * 16
    # conv shape checks
    assert lib.lbt_workspace_bytes_conv2d(1, 1, 2, 2, 1, 3, 3, 1, 0) == 0       # kernel > image
    need = lib.lbt_workspace_bytes_conv2d(4, 16, 12, 12, 32, 3, 3, 1, 1)
    assert need > 0 and need % 256 == 0
    rc = lib.lbt_backward_conv2d(p, p, p, 4, 16, 12, 12, 32, 3, 3, 1, 1, 0.0, 1, 0.0, p, 0, 0,
                                 p, p, p, need - 1, None)
    assert rc == -4
    rc = lib.lbt_backward_conv2d(p, p, p, 4, 16, 12, 12, 32, 3, 3, 0, 1, 0.0, 1, 0.0, p, 0, 0,
                                 p, p, p, need, None)
    assert rc == -2
    assert lib.lbt_workspace_bytes_linear(256, 512, 512) > 0
    # bit-width field of the flag word: 2..8, and no unsigned 8-bit activations for dW
    for flags, want in ((9 << 8, -3), (1 << 8, -3), (8 << 8, -3), (1 << 12, -3)):
        rc = lib.lbt_backward_conv2d(p, p, p, 4, 16, 12, 12, 32, 3, 3, 1, 1, 0.0, 1, 0.0, p, 0,
                                     flags, p, p, p, need, None)
        assert rc == want, (flags, rc)


def test_workspace_formula(lib):
    # header + four code tensors + split-K partial tiles, each padded to 256 bytes
    N, Cc, H, W, K, R, S, st, pad = 64, 256, 14, 14, 256, 3, 3, 1, 1
    P = Q = 14
    pad256 = lambda b: (b + 255) // 256 * 256
    want = 256 + 2048 * 16 + pad256(N * P * Q * K) + pad256(K * P * Q * N) \
        + pad256(Cc * H * W * N) + pad256(Cc * R * S * K)
    got = lib.lbt_workspace_bytes_conv2d(N, Cc, H, W, K, R, S, st, pad)
    partial = got - want
    # dW is [256][2304] int32; the contraction is cut into at most 512/36 slices
    assert partial % (K * Cc * R * S * 4) == 0 and 2 <= partial // (K * Cc * R * S * 4) <= 14


def test_sizes_beyond_the_documented_limits_are_refused(lib):
    # tensors of 2^31 elements or more: refused by the geometry check, before any HIP call
    assert lib.lbt_workspace_bytes_conv2d(1 << 16, 1 << 10, 8, 8, 8, 1, 1, 1, 0) == 0
    assert lib.lbt_workspace_bytes_linear(1 << 20, 1 << 12, 8) == 0
    p = C.c_void_p(4096)
    rc = lib.lbt_backward_conv2d(p, p, p, 1 << 16, 1 << 10, 8, 8, 8, 1, 1, 1, 0, 0.0, 1, 0.0, p, 0, 0,
                                 p, p, p, 1 << 40, None)
    assert rc == -3
    # non-positive sizes, kernel larger than the padded image, zero stride
    for shape in ((0, 1, 4, 4, 1, 1, 1, 1, 0), (1, 1, 4, 4, 1, 7, 7, 1, 1), (1, 1, 4, 4, 1, 1, 1, 0, 0)):
        rc = lib.lbt_backward_conv2d(p, p, p, *shape, 0.0, 1, 0.0, p, 0, 0, p, p, p, 1 << 40, None)
        assert rc == -2, shape
    assert lib.lbt_forward_conv2d(p, p, 0, 1, 4, 4, 1, 1, 1, 1, 0, 0.0, 1, 0.0, 0, p, None, None, p,
                                  1 << 40, None) == -2
    assert lib.lbt_forward_linear(p, p, 4, 4, 4, 0.0, 1, 0.0, 1, p, None, None, p, 1 << 40, None) == -3


def test_saved_codes_calls_check_their_arguments(lib):
    """Host-side checks of the forward call that keeps the operand codes and of the backward
    call that reads them (no kernel is launched by any of these)."""
    N, Cc, H, W, K, R, S, st, pad = 4, 16, 12, 12, 32, 3, 3, 1, 1
    pad256 = lambda b: (b + 255) // 256 * 256
    need = lib.lbt_saved_bytes_conv2d(N, Cc, H, W, K, R, S, st, pad)
    # header, X as [C][N/16][H*W][16], W as [C][R*S][K/16][16]
    assert need == 256 + 2048 * 16 + pad256(Cc * H * W * 16) + pad256(Cc * R * S * K)
    assert lib.lbt_saved_bytes_linear(256, 512, 512) == 256 + 2048 * 16 + 512 * 256 + 512 * 512
    assert lib.lbt_saved_bytes_conv2d(0, 1, 4, 4, 1, 1, 1, 1, 0) == 0
    p = C.c_void_p(4096)
    geom = (N, Cc, H, W, K, R, S, st, pad)
    big = 1 << 40
    # no saved buffer / too small / misaligned
    assert lib.lbt_forward_conv2d_save(p, p, *geom, 0.0, 1, 0.0, 0, None, None, None, None, 0, None, 0,
                                       None) == -1
    assert lib.lbt_forward_conv2d_save(p, p, *geom, 0.0, 1, 0.0, 0, None, None, None, p, need - 1,
                                       None, 0, None) == -4
    assert lib.lbt_forward_conv2d_save(p, p, *geom, 0.0, 1, 0.0, 0, None, None, None,
                                       C.c_void_p(4100), need, None, 0, None) == -7
    # a product needs a workspace; no product, no status
    assert lib.lbt_forward_conv2d_save(p, p, *geom, 0.0, 1, 0.0, 0, p, None, None, p, need, None, 0,
                                       None) == -1
    assert lib.lbt_forward_conv2d_save(p, p, *geom, 0.0, 1, 0.0, 0, None, None, p, p, need, None, 0,
                                       None) == -1
    assert lib.lbt_forward_linear_save(p, p, 4, 4, 4, 0.0, 1, 0.0, 8 << 8, None, None, None, p, big,
                                       None, 0, None) == -3          # unsigned 8-bit activations
    ws = lib.lbt_workspace_bytes_conv2d(*geom)
    assert lib.lbt_backward_conv2d_saved(None, need, p, *geom, 1, p, 0, 0, p, p, None, None, p, ws,
                                         None) == -1
    assert lib.lbt_backward_conv2d_saved(p, need - 1, p, *geom, 1, p, 0, 0, p, p, None, None, p, ws,
                                         None) == -4
    assert lib.lbt_backward_conv2d_saved(p, need, p, *geom, 1, p, 0, 0, p, p, None, None, p, ws - 1,
                                         None) == -4
    assert lib.lbt_backward_linear_saved(p, big, p, 4, 4, 4, 0, p, 0, 8, p, p, None, None, p, big,
                                         None) == -3                 # unknown rounding bit

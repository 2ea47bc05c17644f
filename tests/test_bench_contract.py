"""Host-side checks of the benchmark's contract and of the synthetic workload tables (no GPU)."""
import json
import os
import subprocess
import sys

import numpy as np

from paper_2407_12637_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert p.returncode != 0
    assert "one GPU" in p.stderr and not p.stdout.strip()


def test_resnet50_sweep_table():
    """53 layer occurrences at batch 64; operation counts 2*N*P*Q*K*C*R*S per product; the
    gradient tensors of one pass hold 660 M elements."""
    table = synth.resnet50_layers(64)
    assert sum(L.count for L in table) == 53
    ops = grads = 0
    for L in table:
        if isinstance(L, synth.LinearLayer):
            want = 2 * L.M * L.K * L.N
            n_dy = L.M * L.N
        else:
            want = 2 * L.N * L.P * L.Q * L.K * L.C * L.R * L.S
            n_dy = int(np.prod(L.dy_shape))
            assert L.dy_shape == (L.N, L.K, L.P, L.Q) and L.x_shape == (L.N, L.C, L.H, L.W)
            assert L.w_shape == (L.K, L.C, L.R, L.S)
            # bottleneck convolutions keep the map size unless strided
            assert L.P == (L.H + 2 * L.pad - L.R) // L.stride + 1
        assert L.gemm_ops == want, L.name
        ops += 2 * want * L.count          # dX and dW
        grads += n_dy * L.count
    assert round(ops / 1e9, 1) == 1016.6
    assert grads == 659978752
    # the shapes named in the per-layer tables
    by = {L.name: L for L in table}
    assert by["l3.3x3.256-256@14"].gemm_ops == 2 * 64 * 14 * 14 * 256 * 256 * 9
    assert by["l2.ds1x1s2.256-512@56"].P == 28 and by["l2.ds1x1s2.256-512@56"].stride == 2


def test_vit_l_table():
    table = synth.vit_l_layers(64)
    assert all(isinstance(L, synth.LinearLayer) for L in table)
    assert all(L.M == 64 * 197 for L in table)
    shapes = sorted((L.K, L.N) for L in table)
    assert shapes == [(1024, 1024), (1024, 3072), (1024, 4096), (4096, 1024)]


def test_committed_traffic_summary_is_readable():
    sys.path.insert(0, ROOT)
    import bench
    t, source = bench.measured_traffic(("k_absmax3", "k_quantize_layer"))
    assert t is not None and 1e8 < t < 6e8       # one layer's pass: both sweeps plus the codes
    assert source and "commit=" in source          # the summary says what it was measured at
    one, _ = bench.measured_traffic(("k_quantize_layer",))
    assert one is not None and one < t
    assert bench.measured_traffic(("no_such_kernel",))[0] is None


def test_seeded_generators_are_reproducible():
    a = synth.grad_cfg4(synth.rng(0, 1, 2, synth.T_DY), (1000,))
    b = synth.grad_cfg4(synth.rng(0, 1, 2, synth.T_DY), (1000,))
    c = synth.grad_cfg4(synth.rng(1, 1, 2, synth.T_DY), (1000,))
    assert a.dtype == np.float32 and np.array_equal(a, b) and not np.array_equal(a, c)
    x = synth.relu_normal(synth.rng(0, 1, 2, 0), (1000,))
    assert (x >= 0).all() and (x == 0).mean() > 0.3

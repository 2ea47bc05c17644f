#!/usr/bin/env python3
"""Benchmark of the INT4 quantized backward pass on one MI355X.

A "step" is one pass of the whole hot path over the ResNet-50 bottleneck sweep at
batch 64 (every bottleneck convolution of the network plus the classifier, 53
layers): per layer the gradient quantizer (max, clip value gamma*g_max, stochastic
rounding, clip-out count, pack), the operand quantizers for X and W, the integer dX
and dW contractions with dequantisation, and the clipping-factor update.  Inputs
are seeded synthetic tensors already resident in HBM: ReLU'd normal activations,
Kaiming-normal weights, Student-t(2.5) gradients scaled by 1e-3.

Prints ONE JSON line: whole-job TOPS of the two contractions over the full step
time, the roofline position of the dominant kernel (from HIP-event timings taken by
the library around each of its launches) and the CPU oracle timed on a bounded
sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "INT4 backward TOPS (dX+dW) + quantize GB/s, ResNet-50 layers, % roofline"
PEAK_HBM_GBPS = 8000.0          # MI355X HBM3E
PEAK_INT8_TOPS = 5000.0         # MI355X dense int8 MFMA
BYTES_PER_GRAD_ELEMENT = 4.5    # algorithmic: 4 B fp32 read + 0.5 B code written
# The library's event brackets add a fixed marker overhead to every kernel.  It is
# measured live on launches of the one-thread clipping-factor update kernel and removed:
#   kernel time = bracket(kernel) - (bracket(update kernel) - UPDATE_KERNEL_US)
# with the constant for which the corrected averages of all kernel classes agree with
# rocprofv3's durations (profiles/bench_resnet50_b64_kernel_stats.txt).
UPDATE_KERNEL_US = 4.1


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--rounding", choices=["stochastic", "nearest"], default="stochastic")
    ap.add_argument("--gamma0", type=float, default=1.0)
    ap.add_argument("--bits", type=int, default=4, choices=[2, 3, 4, 5, 6, 7, 8],
                    help="bit-width of weights, activations and gradients (the headline is 4; "
                         "at 8 the activations are quantized as signed values)")
    ap.add_argument("--separate-update", action="store_true",
                    help="apply the interval update with lbt_update_interval after every layer "
                         "instead of inside the backward call (LBT_FUSED_UPDATE)")
    ap.add_argument("--streams", type=int, default=1,
                    help="layers are issued round-robin on this many HIP streams, each with a "
                         "workspace of its own (the sweep's layers are independent of each other); "
                         "1 = everything on one stream, the headline configuration")
    ap.add_argument("--no-overlap-probe", action="store_true",
                    help="skip the extra measurement of the same steps on three streams")
    ap.add_argument("--given-clips", action="store_true",
                    help="pass clip values for X and W (learned parameters in the paper, Sec. 3.1: "
                         "3 standard deviations here) instead of letting the call take the tensors' "
                         "maxima; a separate measurement, the default sweep uses the maxima")
    ap.add_argument("--forward", action="store_true",
                    help="time the quantized forward pass Y = Q(X).Q(W) of the same layers instead "
                         "of the backward pass (a separate measurement, never the headline)")
    ap.add_argument("--single-sweep", action="store_true",
                    help="extra mode, not the paper's quantizer: the gradient interval comes "
                         "from the previous step's maximum, so dY is read once (needs "
                         "--warmup >= 1; reported separately, never the headline)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true")
    ap.add_argument("--layer", default=None, help="run only layers whose name contains this")
    ap.add_argument("--workload", choices=["resnet50", "vit-l"], default="resnet50",
                    help="resnet50: the headline sweep (default); vit-l: the linear layers of one "
                         "ViT-L encoder block at batch 64 x 197 tokens (signed activations)")
    ap.add_argument("--learned-clips", action="store_true",
                    help="clip values of X and W given and learned: lbt_backward_*_learned (the "
                         "backward pass, dW and dX masked with the quantizers' intervals, the "
                         "gradients of c_w and c_x)")
    ap.add_argument("--unfused-ste", action="store_true",
                    help="with --learned-clips: lbt_backward_* followed by two lbt_ste_backward "
                         "calls instead of the one call lbt_backward_*_learned (same kernels)")
    ap.add_argument("--saved-codes", action="store_true",
                    help="the backward calls read the operand codes a forward call kept "
                         "(lbt_forward_*_save before the timed region, lbt_backward_*_saved in it): "
                         "X and W are not quantized again")
    ap.add_argument("--dense-codes", action="store_true",
                    help="control: gradients uniform over the interval, so that all 15 codes "
                         "occur (the heavy-tailed default leaves almost every code at 0)")
    ap.add_argument("--per-layer", action="store_true",
                    help="print a table: every layer shape of the sweep run on its own, "
                         "kernel times against the layer's own rooflines; then exit")
    ap.add_argument("--with-oracle", action="store_true",
                    help="with --per-layer: also time the CPU oracle's full backward of every layer "
                         "shape (one repetition, all host cores)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="only run three plain 256 MiB device copies (calibrates the HBM byte "
                         "counters of a rocprofv3 --pmc run) and exit")
    ap.add_argument("--grad-sets", type=int, default=3,
                    help="distinct output-gradient tensors per layer; step i quantizes set i mod N, "
                         "so consecutive steps see fresh draws and gamma follows data that changes")
    ap.add_argument("--repeats", type=int, default=5,
                    help="the timed region of K steps is run this many times in all; the headline "
                         "is the first (the contract's), the median of all is reported beside it")
    ap.add_argument("--skeleton", action="store_true",
                    help="with --per-layer: also time every product with its contraction loop "
                         "skipped (launch + set-up + writing the result)")
    ap.add_argument("--peaks", action="store_true",
                    help="only run the stand-alone probe of the chip's ceilings (HBM read / write / "
                         "copy, LDS reads, back-to-back int8 MFMA) and exit")
    return ap.parse_args()


class LayerRun:
    """Device tensors and state of one layer occurrence."""

    def __init__(self, spec, idx, torch, lbt, gen, is_linear, x_unsigned=True, dense=False,
                 grad_sets=1):
        dev = "cuda"
        self.spec, self.is_linear, self.x_unsigned = spec, is_linear, x_unsigned
        f32 = torch.float32
        if is_linear:
            xs, ws, gs = (spec.M, spec.K), (spec.K, spec.N), (spec.M, spec.N)
            fan_in = spec.K
        else:
            xs, ws, gs = spec.x_shape, spec.w_shape, spec.dy_shape
            fan_in = spec.C * spec.R * spec.S
        self.X = torch.randn(xs, generator=gen, device=dev, dtype=f32)
        if x_unsigned:
            self.X.clamp_(min=0)        # post-ReLU activations, quantized with Eq. 3
        self.W = torch.randn(ws, generator=gen, device=dev, dtype=f32).mul_((2.0 / fan_in) ** 0.5)
        self.dYs = []
        for _ in range(max(1, grad_sets)):
            if dense:
                # control: uniform over (-1e-3, 1e-3), every code equally likely
                g = torch.rand(gs, generator=gen, device=dev, dtype=f32).mul_(2e-3).sub_(1e-3)
            else:
                # Student-t(nu) = Z / sqrt(chi2_nu / nu), chi2_nu = 2 * Gamma(nu / 2)
                nu = 2.5
                z = torch.randn(gs, generator=gen, device=dev, dtype=f32)
                chi2 = torch._standard_gamma(torch.full(gs, nu / 2, device=dev, dtype=f32), generator=gen) * 2
                g = (z / (chi2 / nu).sqrt_()).mul_(1e-3)
                del z, chi2
            self.dYs.append(g)
        self.dY = self.dYs[0]
        self.dX = torch.empty(xs, device=dev, dtype=f32)
        self.dW = torch.empty(ws, device=dev, dtype=f32)
        self.state = None
        self.seed = 1000 + idx
        self.c_x = self.c_w = 0.0            # <= 0: the call takes the tensor's maximum
        self.fan_in = fan_in
        self.saved = None
        self.grad_c = None                   # gradients of (c_w, c_x) when the clips are learned
        self.unfused_ste = False

    def use_grad_set(self, i):
        self.dY = self.dYs[i % len(self.dYs)]

    def keep_codes(self, torch, lbt, flags):
        """What the forward pass of the layer leaves behind: the codes of X and W in the layouts
        the backward products read (no forward product here: Y = NULL)."""
        s = self.spec
        if self.is_linear:
            self.saved = torch.zeros(lbt.lbt_saved_bytes_linear(s.M, s.K, s.N), dtype=torch.uint8,
                                     device="cuda")
            lbt.lbt_forward_linear_save(self.X, self.W, s.M, s.K, s.N, self.c_x, self.x_unsigned,
                                        self.c_w, flags, None, None, None, self.saved, None)
        else:
            self.saved = torch.zeros(lbt.lbt_saved_bytes_conv2d(s.N, s.C, s.H, s.W, s.K, s.R, s.S,
                                                                s.stride, s.pad),
                                     dtype=torch.uint8, device="cuda")
            lbt.lbt_forward_conv2d_save(self.X, self.W, s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.stride,
                                        s.pad, self.c_x, self.x_unsigned, self.c_w, flags, None,
                                        None, None, self.saved, None)

    def use_given_clips(self):
        self.c_x, self.c_w = 3.0, 3.0 * (2.0 / self.fan_in) ** 0.5

    def ws_bytes(self, lbt, forward=False):
        s = self.spec
        if forward:
            if self.is_linear:
                return lbt.lbt_workspace_bytes_forward_linear(s.M, s.K, s.N)
            return lbt.lbt_workspace_bytes_forward_conv2d(s.N, s.C, s.H, s.W, s.K, s.R, s.S,
                                                          s.stride, s.pad)
        if self.is_linear:
            return lbt.lbt_workspace_bytes_linear(s.M, s.K, s.N)
        return lbt.lbt_workspace_bytes_conv2d(s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.stride, s.pad)

    def run_forward(self, lbt, ws, flags):
        s = self.spec
        if self.saved is not None:      # the forward product that also keeps the codes
            if self.is_linear:
                lbt.lbt_forward_linear_save(self.X, self.W, s.M, s.K, s.N, self.c_x, self.x_unsigned,
                                            self.c_w, flags, self.Y, None, None, self.saved, ws)
            else:
                lbt.lbt_forward_conv2d_save(self.X, self.W, s.N, s.C, s.H, s.W, s.K, s.R, s.S,
                                            s.stride, s.pad, self.c_x, self.x_unsigned, self.c_w,
                                            flags, self.Y, None, None, self.saved, ws)
        elif self.is_linear:
            lbt.lbt_forward_linear(self.X, self.W, s.M, s.K, s.N, self.c_x, self.x_unsigned,
                                   self.c_w, flags, self.Y, None, None, ws)
        else:
            lbt.lbt_forward_conv2d(self.X, self.W, s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.stride,
                                   s.pad, self.c_x, self.x_unsigned, self.c_w, flags, self.Y, None,
                                   None, ws)

    def run(self, lbt, ws, rounding):
        """One layer's backward and its interval update (inside the call when `rounding`
        carries LBT_FUSED_UPDATE, else as a call of its own)."""
        s = self.spec
        if self.saved is not None:
            if self.is_linear:
                lbt.lbt_backward_linear_saved(self.saved, self.dY, s.M, s.K, s.N, self.x_unsigned,
                                              self.state, self.seed, rounding, self.dX, self.dW,
                                              None, None, ws)
            else:
                lbt.lbt_backward_conv2d_saved(self.saved, self.dY, s.N, s.C, s.H, s.W, s.K, s.R, s.S,
                                              s.stride, s.pad, self.x_unsigned, self.state,
                                              self.seed, rounding, self.dX, self.dW, None, None, ws)
        elif self.grad_c is not None and self.unfused_ste:
            # the same result from separate calls: the backward pass, then the gradient through
            # each operand quantizer as a pass of its own
            bits = ((rounding >> 8) & 15) or 4
            if self.is_linear:
                lbt.lbt_backward_linear(self.X, self.W, self.dY, s.M, s.K, s.N, self.c_x,
                                        self.x_unsigned, self.c_w, self.state, self.seed, rounding,
                                        self.dX, self.dW, ws)
            else:
                lbt.lbt_backward_conv2d(self.X, self.W, self.dY, s.N, s.C, s.H, s.W, s.K, s.R, s.S,
                                        s.stride, s.pad, self.c_x, self.x_unsigned, self.c_w,
                                        self.state, self.seed, rounding, self.dX, self.dW, ws)
            lbt.lbt_ste_backward(self.W, self.c_w, False, bits, self.dW, self.dW, self.grad_c[0:1], ws)
            lbt.lbt_ste_backward(self.X, self.c_x, self.x_unsigned, bits, self.dX, self.dX,
                                 self.grad_c[1:2], ws)
        elif self.grad_c is not None:
            if self.is_linear:
                lbt.lbt_backward_linear_learned(self.X, self.W, self.dY, s.M, s.K, s.N, self.c_x,
                                                self.x_unsigned, self.c_w, self.state, self.seed,
                                                rounding, self.dX, self.dW, self.grad_c, ws)
            else:
                lbt.lbt_backward_conv2d_learned(self.X, self.W, self.dY, s.N, s.C, s.H, s.W, s.K,
                                                s.R, s.S, s.stride, s.pad, self.c_x, self.x_unsigned,
                                                self.c_w, self.state, self.seed, rounding, self.dX,
                                                self.dW, self.grad_c, ws)
        elif self.is_linear:
            lbt.lbt_backward_linear(self.X, self.W, self.dY, s.M, s.K, s.N, self.c_x, self.x_unsigned,
                                    self.c_w, self.state, self.seed, rounding, self.dX, self.dW, ws)
        else:
            lbt.lbt_backward_conv2d(self.X, self.W, self.dY, s.N, s.C, s.H, s.W, s.K, s.R, s.S,
                                    s.stride, s.pad, self.c_x, self.x_unsigned, self.c_w, self.state,
                                    self.seed, rounding, self.dX, self.dW, ws)
        if not rounding & lbt.FUSED_UPDATE:
            lbt.lbt_update_interval(self.state)


def cpu_baseline(layers, rounding, bits=4):
    """Time the CPU oracle (as it stands) on a few layers of the same sweep."""
    import numpy as np

    import oracle
    # a bounded sample (10-15 s of host time on the GPU machine) that spans the sweep's stages
    pick = ["l1.3x3.64-64@56", "l1.1x1.64-256@56", "l2.1x1.128-512@28", "l2.3x3.128-128@28",
            "l2.3x3s2.128-128@56", "l3.1x1.256-1024@14", "l3.3x3.256-256@14", "l3.1x1.1024-256@14",
            "l4.1x1.512-2048@7", "l4.3x3.512-512@7", "l4.1x1.2048-512@7", "l3.3x3s2.256-256@28",
            "l1.1x1.256-64@56", "l2.1x1.256-128@56", "l2.ds1x1s2.256-512@56", "l2.1x1.512-128@28",
            "l3.1x1.512-256@28", "l3.ds1x1s2.512-1024@28", "l4.1x1.1024-512@14"]
    chosen = [L for L in layers if not L.is_linear and L.spec.name in pick]
    if not chosen:      # a sweep of linear layers: its smallest layer
        chosen = [min(layers, key=lambda L: L.spec.gemm_ops)]
    seen, sample = set(), []
    for L in chosen:
        if L.spec.name not in seen:
            seen.add(L.spec.name)
            sample.append(L)
    ops, n_grad, t_total, t_quant = 0.0, 0, 0.0, 0.0
    for L in sample:
        s = L.spec
        X, W, dY = (t.cpu().numpy() for t in (L.X, L.W, L.dY))
        st = oracle.GradState(gamma=1.0, bits=bits)
        t0 = time.perf_counter()
        oracle.quantize_grad(dY, st, L.seed, rounding)
        t1 = time.perf_counter()
        st = oracle.GradState(gamma=1.0, bits=bits)
        if L.is_linear:
            oracle.backward_linear(X, W, dY, st, x_unsigned=L.x_unsigned, seed=L.seed,
                                   rounding=rounding)
        else:
            oracle.backward_conv2d(X, W, dY, s.stride, s.pad, st, x_unsigned=L.x_unsigned,
                                   seed=L.seed, rounding=rounding)
        oracle.update_interval(st)
        t2 = time.perf_counter()
        ops += 2.0 * s.gemm_ops
        n_grad += dY.size
        t_quant += t1 - t0
        t_total += t2 - t1
    return {
        "value": ops / t_total / 1e12, "unit": "TOPS", "cores": oracle.num_threads(),
        "kind": "oracle",
        "sample": "full backward (quantize dY/X/W + dX + dW + update) of %d layers of the sweep: %s; %.1f s"
                  % (len(sample), ", ".join(L.spec.name for L in sample), t_total),
        "quantize_GBps": n_grad * BYTES_PER_GRAD_ELEMENT / t_quant / 1e9,
    }


def per_layer_report(args, torch, lbt, synth, rounding, gen, vit):
    """Every layer shape of the sweep on its own: the call is repeated over enough instances of
    the layer (distinct tensors, > 600 MB together) that no cache serves the next call's reads,
    with the library's event brackets on.  Times are per call; the products are rated against
    the int8 peak and against the layer's own roofline max(ops / peak, algorithmic bytes / HBM
    peak); the quantize pass (maximum + quantize launches over dY, X and W) at 4.5 B/element."""
    table = synth.vit_l_layers(64) if vit else synth.resnet50_layers(64)
    reps = 12
    # marker overhead, as in the main run
    lbt.lbt_profile_enable(True)
    spare = lbt.new_state()
    for _ in range(64):
        lbt.lbt_update_interval(spare)
    torch.cuda.synchronize()
    cal = lbt.lbt_profile_read()["k_update_interval"]
    lbt.lbt_profile_enable(False)
    ov = max(cal[1] / cal[0] * 1e3 - UPDATE_KERNEL_US, 0.0)
    head = ("%-24s %2s %7s | %7s %6s %5s | %7s %6s %5s %5s %1s | %7s %6s %5s %5s %1s"
            % ("layer", "x", "n_dY(M)", "quant", "GB/s", "%HBM", "dX us", "TOPS", "%MFMA", "%roof",
               "b", "dW us", "TOPS", "%MFMA", "%roof", "b"))
    if args.skeleton:
        head += " | %7s %7s" % ("dX skel", "dW skel")
    if args.with_oracle:
        import oracle
        head += " | %9s" % "oracle ms"
    print(head)
    print("-" * len(head))
    tot = {"q_t": 0.0, "q_b": 0.0, "c_ops": 0.0, "c_t": 0.0, "all_ops": 0.0, "all_t": 0.0,
           "roof_t": 0.0}
    for spec in table:
        if args.layer and args.layer not in spec.name:
            continue
        is_lin = isinstance(spec, synth.LinearLayer)
        probe = LayerRun(spec, 0, torch, lbt, gen, is_lin, x_unsigned=not vit and args.bits < 8,
                         dense=args.dense_codes)
        per_inst = 4 * (2 * probe.X.numel() + 2 * probe.W.numel() + probe.dY.numel())
        n_inst = min(max(2, -(-600_000_000 // per_inst)), 8)
        Ls = [probe] + [LayerRun(spec, i, torch, lbt, gen, is_lin,
                                 x_unsigned=not vit and args.bits < 8, dense=args.dense_codes)
                        for i in range(1, n_inst)]
        for L in Ls:
            L.state = lbt.new_state(gamma0=args.gamma0, bits=args.bits)
            if args.given_clips:
                L.use_given_clips()
            if args.saved_codes:
                L.keep_codes(torch, lbt, lbt.BITS(args.bits))
        ws = torch.zeros(probe.ws_bytes(lbt), dtype=torch.uint8, device="cuda")
        for L in Ls:
            L.run(lbt, ws, rounding)
        torch.cuda.synchronize()
        lbt.lbt_profile_enable(True)
        lbt.lbt_profile_read()
        for r in range(reps):
            Ls[r % n_inst].run(lbt, ws, rounding)
        torch.cuda.synchronize()
        prof = lbt.lbt_profile_read()
        lbt.lbt_profile_enable(False)
        us = {k: max((v[1] * 1e3 - ov * v[0]) / reps, 0.0) for k, v in prof.items()}
        skel = None
        if args.skeleton:
            # the same calls with the products' contraction loops skipped
            lbt.lbt_profile_skeleton(True)
            lbt.lbt_profile_enable(True)
            lbt.lbt_profile_read()
            for r in range(reps):
                Ls[r % n_inst].run(lbt, ws, rounding)
            torch.cuda.synchronize()
            prof2 = lbt.lbt_profile_read()
            lbt.lbt_profile_enable(False)
            lbt.lbt_profile_skeleton(False)
            us2 = {k: max((v[1] * 1e3 - ov * v[0]) / reps, 0.0) for k, v in prof2.items()}
            skel = (us2.get("k_implicit_gemm(dX)", 0.0),
                    us2.get("k_implicit_gemm(dW)", 0.0) + us2.get("k_splitk_reduce", 0.0))
        ng, nx, nw = probe.dY.numel(), probe.X.numel(), probe.W.numel()
        ops = spec.gemm_ops
        t_q = us.get("k_absmax3", 0.0) + us.get("k_quantize_layer", 0.0)
        q_bytes = BYTES_PER_GRAD_ELEMENT * (ng if args.saved_codes else ng + nx + nw)
        t_dx = us.get("k_implicit_gemm(dX)", 0.0)
        t_dw = us.get("k_implicit_gemm(dW)", 0.0) + us.get("k_splitk_reduce", 0.0)
        cols = []
        for t_us, byts in ((t_dx, 0.5 * ng + 0.5 * nw + 4.0 * nx), (t_dw, 0.5 * nx + 0.5 * ng + 4.0 * nw)):
            t_c, t_m = ops / (PEAK_INT8_TOPS * 1e12), byts / (PEAK_HBM_GBPS * 1e9)
            roof_us = max(t_c, t_m) * 1e6
            tops = ops / (t_us * 1e-6) / 1e12
            cols += [t_us, tops, 100 * tops / PEAK_INT8_TOPS, 100 * roof_us / t_us, "C" if t_c > t_m else "M"]
            tot["all_ops"] += ops * spec.count
            tot["all_t"] += t_us * spec.count
            tot["roof_t"] += roof_us * spec.count
            if t_c > t_m:
                tot["c_ops"] += ops * spec.count
                tot["c_t"] += t_us * spec.count
        tot["q_t"] += t_q * spec.count
        tot["q_b"] += q_bytes * spec.count
        gbps = q_bytes / (t_q * 1e-6) / 1e9
        line = ("%-24s %2d %7.2f | %7.1f %6.0f %5.1f | %7.1f %6.0f %5.1f %5.1f %1s | %7.1f %6.0f %5.1f %5.1f %1s"
                % (spec.name, spec.count, ng / 1e6, t_q, gbps, 100 * gbps / PEAK_HBM_GBPS, *cols))
        if skel:
            line += " | %7.1f %7.1f" % skel
            tot["skel_dx"] = tot.get("skel_dx", 0.0) + skel[0] * spec.count
            tot["skel_dw"] = tot.get("skel_dw", 0.0) + skel[1] * spec.count
            tot["full_dx"] = tot.get("full_dx", 0.0) + t_dx * spec.count
            tot["full_dw"] = tot.get("full_dw", 0.0) + t_dw * spec.count
        if args.with_oracle:
            X, W, dY = (t.cpu().numpy() for t in (probe.X, probe.W, probe.dY))
            ost = oracle.GradState(gamma=args.gamma0, bits=args.bits)
            t0 = time.perf_counter()
            if is_lin:
                oracle.backward_linear(X, W, dY, ost, x_unsigned=probe.x_unsigned, seed=probe.seed,
                                       rounding=rounding & lbt.ROUND_STOCHASTIC)
            else:
                oracle.backward_conv2d(X, W, dY, spec.stride, spec.pad, ost, x_unsigned=probe.x_unsigned,
                                       seed=probe.seed, rounding=rounding & lbt.ROUND_STOCHASTIC)
            oracle.update_interval(ost)
            line += " | %9.0f" % ((time.perf_counter() - t0) * 1e3)
            del X, W, dY
        print(line, flush=True)
        del Ls, probe, ws
        torch.cuda.empty_cache()
    print("-" * len(head))
    print("x = occurrences in the network; quant = maximum + quantize launches of dY, X and W, rated at "
          "4.5 B per element; %%roof = the layer's own roofline time max(ops / 5.0 POP/s, algorithmic "
          "bytes / 8 TB/s) over the measured time; b = which of the two binds (C compute, M memory); "
          "dX includes the sum of dW's split contraction (carried by the dX launch).  Event-bracket overhead removed per launch: %.2f us." % ov
          + ("  oracle ms = the CPU oracle's whole backward of the layer (quantizers, both products, "
             "update), one repetition on %d threads." % oracle.num_threads() if args.with_oracle else ""))
    summary = {
        "quantize_pass_GBps": tot["q_b"] / (tot["q_t"] * 1e-6) / 1e9,
        "products_TOPS": tot["all_ops"] / (tot["all_t"] * 1e-6) / 1e12,
        "products_frac_of_layer_rooflines": tot["roof_t"] / tot["all_t"],
        "compute_bound_products_TOPS": (tot["c_ops"] / (tot["c_t"] * 1e-6) / 1e12) if tot["c_t"] else None,
        "compute_bound_products_frac_of_int8_peak":
            (tot["c_ops"] / (tot["c_t"] * 1e-6) / 1e12 / PEAK_INT8_TOPS) if tot["c_t"] else None,
    }
    if args.skeleton:
        summary["skeleton_us_per_step"] = {k: tot[k] for k in ("full_dx", "skel_dx", "full_dw", "skel_dw")}
        print("dX skel / dW skel = the same launches with the contraction loop skipped: launch, set-up "
              "(tap tables, addresses), and the epilogue that writes the (all-zero) result; for dW the "
              "partial tiles and their sum as well.")
    print("occurrence-weighted over the sweep:", json.dumps(summary))


def measured_traffic(kernel_classes):
    """HBM bytes per launch (fetched + written), summed over the given kernel classes, from the
    committed summary of the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this benchmark, and
    that summary's own statement of the commit it was measured at: (bytes or None, source)."""
    rel = os.path.join("profiles", "bench_resnet50_b64_hbm_traffic.txt")
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), rel)
    found, source = {}, None
    try:
        for line in open(path):
            f = line.split()
            if len(f) == 4 and f[0] == "TRAFFIC":
                found[f[1]] = float(f[2].split("=")[1]) + float(f[3].split("=")[1])
            elif len(f) >= 2 and f[0] == "SOURCE":
                source = "%s (%s)" % (rel, " ".join(f[1:]))
    except OSError:
        return None, None
    if source is None or any(k not in found for k in kernel_classes):
        return None, source
    return sum(found[k] for k in kernel_classes), source


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives are part of it); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.peaks:
        # a child process of its own: this one has not touched the GPU yet
        import subprocess
        from paper_2407_12637_amd import build as lbt_build
        if not os.path.exists(lbt_build.PEAKS):
            print("bench.py: the peak probe is not built (python -c 'import __graft_entry__ as g; "
                  "g.build()')", file=sys.stderr)
            sys.exit(2)
        sys.exit(subprocess.call([lbt_build.PEAKS]))
    import torch

    from paper_2407_12637_amd import binding as lbt
    from paper_2407_12637_amd import synth

    lbt.load()
    torch.cuda.set_device(0)
    if args.copy_probe:
        n = 256 << 20
        src = torch.full((n,), 7, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes_each_way": n, "copies": 3}))
        return
    rounding = lbt.ROUND_STOCHASTIC if args.rounding == "stochastic" else lbt.ROUND_NEAREST
    if not args.separate_update:
        rounding |= lbt.FUSED_UPDATE
    if args.single_sweep:
        if args.warmup < 1:
            print("bench.py: --single-sweep needs --warmup >= 1 (the first step has no previous "
                  "maximum and quantizes everything to 0)", file=sys.stderr)
            sys.exit(2)
        rounding |= lbt.HINDSIGHT_MAX
    gen = torch.Generator(device="cuda")
    gen.manual_seed(0)

    rounding |= lbt.BITS(args.bits)
    vit = args.workload == "vit-l"
    if args.per_layer:
        if args.forward:
            print("bench.py: --per-layer covers the backward calls", file=sys.stderr)
            sys.exit(2)
        per_layer_report(args, torch, lbt, synth, rounding, gen, vit)
        return
    table = synth.vit_l_layers(64) if vit else synth.resnet50_layers(64)
    layers = []
    for spec in table:
        if args.layer and args.layer not in spec.name:
            continue
        for _ in range(spec.count):
            layers.append(LayerRun(spec, len(layers), torch, lbt, gen,
                                   isinstance(spec, synth.LinearLayer),
                                   x_unsigned=not vit and args.bits < 8, dense=args.dense_codes,
                                   grad_sets=1 if args.forward else args.grad_sets))
    for L in layers:
        L.state = lbt.new_state(gamma0=args.gamma0, bits=args.bits)
        if args.given_clips or args.learned_clips:
            L.use_given_clips()
        if args.learned_clips:
            L.grad_c = torch.zeros(2, device="cuda")
            L.unfused_ste = args.unfused_ste
        if args.saved_codes:
            L.keep_codes(torch, lbt, lbt.BITS(args.bits))
    ws = torch.zeros(max(L.ws_bytes(lbt, args.forward) for L in layers), dtype=torch.uint8,
                     device="cuda")
    gemm_ops = sum(2.0 * L.spec.gemm_ops for L in layers)       # dX and dW
    if args.forward:
        gemm_ops /= 2.0                                          # one product per layer
        for L in layers:
            L.Y = torch.empty_like(L.dY)
            L.dX = L.dW = None
    n_grad = sum(L.dY.numel() for L in layers)

    n_streams = max(1, args.streams)

    def run_layer(L, space):
        if args.forward:
            L.run_forward(lbt, space, lbt.BITS(args.bits))
        else:
            L.run(lbt, space, rounding)

    counter = [0]     # steps issued so far: step i takes every layer's gradient set i mod N

    def make_step(n):
        """One pass over the sweep, layers issued round-robin on n streams (each stream has a
        workspace of its own; n = 1: everything on the current stream)."""
        if n == 1:
            def one_stream():
                for L in layers:
                    L.use_grad_set(counter[0])
                    run_layer(L, ws)
                counter[0] += 1
            return one_stream
        streams = [torch.cuda.Stream() for _ in range(n)]
        spaces = [ws] + [torch.zeros_like(ws) for _ in range(n - 1)]

        def many_streams():
            main = torch.cuda.current_stream()
            for st in streams:
                st.wait_stream(main)
            for i, L in enumerate(layers):
                L.use_grad_set(counter[0])
                with torch.cuda.stream(streams[i % n]):
                    run_layer(L, spaces[i % n])
            for st in streams:
                main.wait_stream(st)
            counter[0] += 1
        return many_streams

    step = make_step(n_streams)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    # the same region again (args.repeats in all): run-to-run spread and the median
    region_ms = [ms_per_step]
    for _ in range(max(0, args.repeats - 1)):
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        region_ms.append((time.perf_counter() - t1) / args.steps * 1e3)

    out = {
        "metric": METRIC, "value": gemm_ops / (dt / args.steps) / 1e12, "unit": "TOPS",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": "%s, batch 64, %d layers, INT%d W/A/G, %s rounding, gamma0=%g"
                               % ("ViT-L encoder block linear layers (197 tokens)" if vit
                                  else "ResNet-50 bottleneck sweep", len(layers), args.bits,
                                  args.rounding, args.gamma0),
                   "gemm_GOP_per_step": gemm_ops / 1e9, "grad_elements_per_step": n_grad,
                   "grad_sets": 1 if args.forward else args.grad_sets},
        "repeats": {"regions": len(region_ms), "ms_per_step_median": sorted(region_ms)[len(region_ms) // 2],
                    "ms_per_step_min": min(region_ms), "ms_per_step_max": max(region_ms)},
    }
    if n_streams > 1:
        out["config"]["workload"] += ", layers round-robin on %d streams" % n_streams
    elif not args.no_overlap_probe:
        # the same K steps once more with the (independent) layers of the sweep issued on three
        # streams: kernels bound by HBM overlap with kernels bound by latency.  Reported beside
        # the headline, which stays the one-stream figure the per-kernel numbers refer to.
        overlapped = make_step(3)
        overlapped()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            overlapped()
        torch.cuda.synchronize()
        dt3 = (time.perf_counter() - t0) / args.steps
        out["multi_stream"] = {"streams": 3, "ms_per_step": dt3 * 1e3,
                               "value": gemm_ops / dt3 / 1e12, "unit": "TOPS"}
        del overlapped
        step = make_step(1)
    if args.learned_clips:
        out["config"]["workload"] += (", clip values of X and W given, gradient through both "
                                      "operand quantizers after every layer")
    if args.saved_codes:
        out["config"]["workload"] += (", X and W codes kept by the forward pass (not quantized "
                                      "again in the backward calls)")
    if args.dense_codes:
        out["config"]["workload"] += ", CONTROL: gradients uniform over the interval (dense codes)"
    if args.given_clips:
        out["config"]["workload"] += ", clip values of X and W given (no maximum taken)"
    if args.forward:
        out["config"]["workload"] += ", FORWARD pass Y = Q(X).Q(W) only"
    if args.single_sweep:
        out["config"]["workload"] += ", single-sweep mode (interval from the previous step's maximum)"

    if not args.no_kernel_timing:
        # same steps again with the library's event timing on: per-kernel durations
        lbt.lbt_profile_enable(True)
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        out["ms_per_step_with_kernel_timing"] = (time.perf_counter() - t0) / args.steps * 1e3
        prof = lbt.lbt_profile_read()
        # marker overhead: brackets around the one-thread update kernel on a spare state
        # (after the steps; with the update inside the backward calls the steps have none)
        spare = lbt.new_state()
        for _ in range(64):
            lbt.lbt_update_interval(spare)
        torch.cuda.synchronize()
        cal = lbt.lbt_profile_read()["k_update_interval"]
        lbt.lbt_profile_enable(False)
        overhead_us = max(cal[1] / cal[0] * 1e3 - UPDATE_KERNEL_US, 0.0)
        out["event_bracket_overhead_us"] = overhead_us
        kernels = {}
        for name, (launches, ms_raw, work) in prof.items():
            if not launches or name == "k_state_set":
                continue
            ms = max(ms_raw - launches * overhead_us * 1e-3, 1e-9)
            k = {"launches_per_step": launches / args.steps, "ms_per_step": ms / args.steps,
                 "avg_us": ms / launches * 1e3, "avg_us_with_markers": ms_raw / launches * 1e3}
            if "gemm" in name:
                k["TOPS"] = work / (ms * 1e-3) / 1e12
            elif "ste" in name:
                k["GBps"] = work * 12.0 / (ms * 1e-3) / 1e9     # x and grad read, grad written
            elif "quantize" in name or "absmax" in name:
                # the quantizer's algorithmic 4.5 B/element covers both sweeps of the tensor
                # (maximum, then quantize); the maximum pass alone is rated at 4 B/element
                per = BYTES_PER_GRAD_ELEMENT if "quantize" in name else 4.0
                k["GBps"] = work * per / (ms * 1e-3) / 1e9
            kernels[name] = k
        out["kernels"] = kernels
        # The dominant kernel of the step.  The quantize pass (the maximum sweep and the quantize
        # sweep over the same tensors: two launches, one kernel in the sense of the scope table)
        # counts as one; it is rated at the algorithmic 4.5 B per quantized element over the
        # time of both launches.
        q, am = kernels.get("k_quantize_layer"), kernels.get("k_absmax3")
        groups = {n: kernels[n]["ms_per_step"] for n in kernels if n not in ("k_quantize_layer", "k_absmax3")}
        if q and am:
            groups["quantize pass (k_absmax3 + k_quantize_layer)"] = q["ms_per_step"] + am["ms_per_step"]
        dom = max(groups, key=lambda n: groups[n])
        pass_dom = dom.startswith("quantize pass")
        traffic, traffic_source = (None, None) if vit else measured_traffic(
            ("k_absmax3", "k_quantize_layer") if pass_dom else (dom,))   # counters: default sweep only
        if "gemm" in dom:
            # A product class is rated against whichever of its two rooflines binds over the
            # sweep: the int8 matrix cores (its operations) or HBM (its algorithmic bytes: 4-bit
            # codes of the two operands read once, the fp32 result written once).
            def product_bytes(L):
                nx, nw, ng = L.X.numel(), L.W.numel(), L.dY.numel()
                if "dX" in dom:
                    return 0.5 * ng + 0.5 * nw + 4.0 * nx
                if "dW" in dom:
                    return 0.5 * nx + 0.5 * ng + 4.0 * nw
                return 0.5 * nx + 0.5 * nw + 4.0 * ng       # forward: Y has dY's shape
            ops = sum(L.spec.gemm_ops for L in layers)
            byts = sum(product_bytes(L) for L in layers)
            t_s = kernels[dom]["ms_per_step"] * 1e-3
            rates = {"TOPS": ops / t_s / 1e12, "GBps_algorithmic": byts / t_s / 1e9,
                     "frac_of_int8_peak": ops / t_s / 1e12 / PEAK_INT8_TOPS,
                     "frac_of_hbm_peak": byts / t_s / 1e9 / PEAK_HBM_GBPS}
            if byts / (PEAK_HBM_GBPS * 1e9) > ops / (PEAK_INT8_TOPS * 1e12):
                out["roofline"] = {"kernel": dom, "bound": "hbm", "achieved": rates["GBps_algorithmic"],
                                   "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                                   "frac": rates["frac_of_hbm_peak"], "traffic": traffic}
            else:
                out["roofline"] = {"kernel": dom, "bound": "mfma", "achieved": rates["TOPS"],
                                   "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                                   "frac": rates["frac_of_int8_peak"], "traffic": traffic}
            out["roofline"]["both_rates"] = rates
        elif pass_dom:
            n_all = (0 if args.forward else n_grad) + (0 if args.saved_codes else
                                                       sum(L.X.numel() + L.W.numel() for L in layers))
            launches = q["launches_per_step"]
            per_launch_bytes = n_all * BYTES_PER_GRAD_ELEMENT / launches
            per_launch_s = (q["avg_us"] + am["avg_us"]) * 1e-6
            ach = per_launch_bytes / per_launch_s / 1e9
            out["roofline"] = {"kernel": dom, "bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBPS,
                               "unit": "GB/s", "frac": ach / PEAK_HBM_GBPS, "traffic": traffic,
                               "algorithmic_bytes_per_launch": per_launch_bytes,
                               "avg_launch_us": {"k_absmax3": am["avg_us"], "k_quantize_layer": q["avg_us"]}}
        else:
            ach = kernels[dom].get("GBps", 0.0)
            out["roofline"] = {"kernel": dom, "bound": "hbm", "achieved": ach,
                               "peak": PEAK_HBM_GBPS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBPS,
                               "traffic": traffic}
        out["roofline"]["traffic_source"] = traffic_source
        # the quantize pass = the maximum kernel + the quantize kernel (gradient, activations
        # and weights of a layer share both launches), rated at the algorithmic 4.5 B per
        # quantized element
        if q and am:
            n_all = (0 if args.forward else n_grad) + (0 if args.saved_codes else
                                                       sum(L.X.numel() + L.W.numel() for L in layers))
            t_ms = q["ms_per_step"] + am["ms_per_step"]
            gbps = n_all * BYTES_PER_GRAD_ELEMENT / (t_ms * 1e-3) / 1e9
            out["quantize_pass"] = {"GBps": gbps, "frac_of_hbm_peak": gbps / PEAK_HBM_GBPS,
                                    "ms_per_step": t_ms, "bytes_per_element": BYTES_PER_GRAD_ELEMENT,
                                    "elements_per_step": n_all}
        # the two contractions against the int8 MFMA peak and against each layer's own
        # roofline min(compute, memory) with the algorithmic bytes of the packed operands
        g = [kernels[n] for n in kernels if "gemm" in n or "splitk" in n]
        if g:
            t_ms = sum(k["ms_per_step"] for k in g)
            tops = gemm_ops / (t_ms * 1e-3) / 1e12
            t_roof = 0.0
            for L in layers:
                ops = L.spec.gemm_ops
                nx, nw, ng = L.X.numel(), L.W.numel(), L.dY.numel()
                products = ((0.5 * nx + 0.5 * nw + 4.0 * ng,) if args.forward else
                            (0.5 * ng + 0.5 * nw + 4.0 * nx, 0.5 * nx + 0.5 * ng + 4.0 * nw))
                for byts in products:
                    t_roof += max(ops / (PEAK_INT8_TOPS * 1e12), byts / (PEAK_HBM_GBPS * 1e9))
            out["contractions"] = {"TOPS": tops, "frac_of_int8_peak": tops / PEAK_INT8_TOPS,
                                   "ms_per_step": t_ms, "roofline_ms_per_step": t_roof * 1e3,
                                   "frac_of_layer_rooflines": t_roof * 1e3 / t_ms}

    if not (args.no_cpu_baseline or args.single_sweep or args.forward or args.given_clips or args.saved_codes or args.learned_clips):   # the oracle is timed on the paper's mode
        out["cpu_baseline"] = cpu_baseline(layers, rounding & lbt.ROUND_STOCHASTIC, args.bits)

    print(json.dumps(out))


if __name__ == "__main__":
    main()

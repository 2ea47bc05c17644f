"""Pins for the error bound and the clipping-factor update (Sec. 3.3, Alg. 1)."""
import math

import numpy as np
import pytest

import oracle
from oracle import diagnostics as dg
from paper_2407_12637_amd import synth


def _tensors(n=30000):
    r = synth.rng(1, 91, 0, synth.T_DY)
    return {
        "t3": synth.grad_cfg1(r, (n,)),
        "laplace": synth.grad_cfg2(r, (n,)),
        "t2.5": synth.grad_cfg4(r, (n,)),
        "spikes": synth.grad_cfg5(r, (n,)),
    }


# -- E(G_L) <= U(G_L), Eq. (7), (8), supplement (i)-(iii) ------------------------
@pytest.mark.parametrize("bits", [3, 4, 8])
def test_error_of_large_gradients_below_ulg(bits):
    alpha = 1e-3                                   # alpha * N = 30: integral
    for name, g in _tensors().items():
        gmax = float(oracle.tensor_max(g)[0])
        for gamma in (1.0, 0.8, 0.5, 0.2, 0.05, 0.01):
            c = oracle.clip_value(gamma, np.float32(gmax))
            s = oracle.scale(c, bits)
            code, _ = oracle.quantize(g, c, bits)
            gam = float(c) / gmax                   # the gamma actually realised in fp32
            i_in, i_out = dg.split_large(g, alpha, gam)
            e6 = dg.error_large(g, code, s, alpha)
            e7 = dg.error_large_split(g, code, s, alpha, gam)
            assert e6 == pytest.approx(e7, rel=1e-12)
            n = g.size
            r_in, r_out = i_in.size / n, i_out.size / n
            assert r_in + r_out == pytest.approx(alpha, rel=1e-12)        # Eq. (10)
            u_i = dg.ulg_counts(i_in.size, i_out.size, gam, bits, gmax)
            u_8 = dg.ulg_ratios(r_in, r_out, gam, bits, alpha)
            assert u_i == pytest.approx(u_8, rel=1e-12)                   # (i) == (8)
            assert e6 <= u_8 * (1 + 1e-9), (name, gamma, bits)
            assert dg.error_all(g, code, s) >= 0


def test_optimal_ratios_values():
    # Eq. (14) for the bit-widths the paper uses
    for bits, (a, b) in {4: (14 / 15, 1 / 15), 3: (6 / 7, 1 / 7), 8: (254 / 255, 1 / 255)}.items():
        r_in, r_out = dg.optimal_ratios(bits, 1.0)
        assert r_in == pytest.approx(a) and r_out == pytest.approx(b)
        # they satisfy Eq. (10) and the optimality condition Eq. (13)
        assert r_in + r_out == pytest.approx(1.0)
        assert dg.dulg_dgamma_approx(r_in, r_out, bits, 1.0) == pytest.approx(0.0, abs=1e-15)


# -- update rule truth table (Eq. 15, 16; Alg. 1) -------------------------------
def _step(gamma, n_out, n_total, alpha=1e-3, beta=1e-3, bits=4, gmin=1e-3, gmax=1.0):
    st = oracle.GradState(gamma=gamma, alpha=alpha, beta=beta, bits=bits,
                          gamma_min=gmin, gamma_max=gmax)
    st.n_out, st.n_total = n_out, n_total
    sg = oracle.update_interval(st)
    return sg, st


def test_update_truth_table():
    # R_out > alpha/15 raises gamma by beta, < lowers it, == leaves it
    sg, st = _step(0.5, 7, 100000)            # 7e-5 > 6.67e-5
    assert sg == 1 and st.gamma == 0.5 + 1e-3 and st.step == 1
    sg, st = _step(0.5, 6, 100000)            # 6e-5 < 6.67e-5
    assert sg == -1 and st.gamma == 0.5 - 1e-3
    sg, st = _step(0.5, 2, 30000)             # 15*2 == 1e-3*30000 exactly
    assert sg == 0 and st.gamma == 0.5
    sg, st = _step(0.5, 2, 30000, bits=8)     # 255*2 > 30
    assert sg == 1
    sg, st = _step(0.5, 0, 1000)
    assert sg == -1
    # clamps: gamma stays in [gamma_min, gamma_max]
    sg, st = _step(1.0, 10 ** 6, 10 ** 6)
    assert sg == 1 and st.gamma == 1.0
    sg, st = _step(1e-3, 0, 1000)
    assert sg == -1 and st.gamma == 1e-3
    # beta = 0 is the fixed-gamma baseline
    sg, st = _step(0.8, 0, 1000, beta=0.0)
    assert st.gamma == 0.8 and st.step == 1


def test_gamma_one_always_steps_down():
    for g in _tensors().values():
        st = oracle.GradState(gamma=1.0)
        oracle.quantize_grad(g, st)
        assert st.n_out == 0
        assert oracle.update_interval(st) == -1 and st.gamma == pytest.approx(0.999)


def test_update_is_sign_descent_on_ulg():
    # Eq. (12) with R_in = alpha - R_out has the opposite sign of T in Eq. (16);
    # and counting clip-outs over all of G gives the same direction as counting
    # them inside G_L (the paper's definition) whenever G_L is non-empty.
    alpha = 1e-3
    for g in _tensors().values():
        gmax = oracle.tensor_max(g)[0]
        for gamma in np.linspace(0.01, 1.0, 34):
            st = oracle.GradState(gamma=float(gamma), alpha=alpha)
            oracle.quantize_grad(g, st)
            gam = float(st.clip) / float(gmax)
            i_in, i_out = dg.split_large(g, alpha, gam)
            r_in, r_out = i_in.size / g.size, i_out.size / g.size
            slope = dg.dulg_dgamma_approx(r_in, r_out, 4, alpha)
            sg = oracle.update_interval(st)
            assert sg == -int(np.sign(slope)) or abs(slope) < 1e-12
            t_paper = r_out - alpha / 15
            assert sg == int(np.sign(t_paper)) or abs(t_paper) < 1e-15


@pytest.mark.parametrize("bits", [4, 8])
def test_converges_to_order_statistic(bits):
    # gamma rises while #{|g| > c} > alpha N/(2^b-1) and falls otherwise, so it
    # settles within beta of a_(k)/g_max, a_(k) the k-th largest magnitude,
    # k = floor(alpha N/(2^b-1)) + 1.
    alpha, beta = 1e-3, 1e-3
    finals = {}
    for name, g in _tensors(n=31000).items():      # alpha N/15 not integral: no plateau
        n = g.size
        a = np.sort(np.abs(g.astype(np.float64)))[::-1]
        k = math.floor(alpha * n / (2 ** bits - 1)) + 1
        target = a[k - 1] / a[0]
        st = oracle.GradState(gamma=1.0, alpha=alpha, beta=beta, bits=bits)
        trace = []
        for it in range(1400):
            oracle.quantize_grad(g, st)
            oracle.update_interval(st)
            trace.append(st.gamma)
        assert abs(st.gamma - max(target, st.gamma_min)) <= beta * 1.5, (name, target, st.gamma)
        assert abs(trace[-1] - trace[-3]) < 1e-12         # a two-cycle
        if target > 2 * beta:
            # at convergence the clip-out ratio brackets alpha/(2^b-1) (Eq. 14)
            lo = oracle.GradState(gamma=st.gamma - beta, alpha=alpha, bits=bits)
            hi = oracle.GradState(gamma=st.gamma + beta, alpha=alpha, bits=bits)
            oracle.quantize_grad(g, lo)
            oracle.quantize_grad(g, hi)
            assert hi.n_out / n <= alpha / (2 ** bits - 1) <= lo.n_out / n + 1.0 / n
        finals[name] = st.gamma
    assert len(finals) == 4


def test_exact_ratio_is_a_fixed_point():
    # alpha N/(2^b-1) integral: once N(G_out) equals it, sign(0) = 0 holds gamma
    g = _tensors(n=30000)["laplace"]
    st = oracle.GradState(gamma=1.0)
    for _ in range(300):
        oracle.quantize_grad(g, st)
        oracle.update_interval(st)
    before = st.gamma
    oracle.quantize_grad(g, st)
    assert st.n_out == 2 and oracle.update_interval(st) == 0 and st.gamma == before


def test_lower_bitwidth_gives_lower_gamma():
    # Supplement S3: the clipping factor settles lower at 4 bits than at 8 bits
    alpha = 1e-3
    for g in _tensors(n=61000).values():
        out = {}
        for bits in (4, 8):
            st = oracle.GradState(gamma=1.0, alpha=alpha, bits=bits)
            for _ in range(1200):
                oracle.quantize_grad(g, st)
                oracle.update_interval(st)
            out[bits] = st.gamma
        assert out[4] <= out[8] + 1e-3

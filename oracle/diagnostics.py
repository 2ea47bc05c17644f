"""Error measures and bounds of Sec. 3.2-3.3, in numpy double -- oracle-side only.

These are not on the hot path; they exist so that the oracle's quantizer and
update rule can be checked against what the paper derives:
  E(G), E(G_L)                       Eq. (5), (6), (7)
  G_L, G_in, G_out and their ratios  Sec. 3.2, Sec. 3.3 "ULG", Eq. (9), (10)
  U(G_L)                             Eq. (8) and supplement Eq. (i)
  dU/dgamma with dR_out/dgamma = 0   Eq. (12); optimal ratios Eq. (14)
TEST INFRASTRUCTURE: never imported by the product.
"""
from __future__ import annotations

import math

import numpy as np


def dequantized(code, s: float) -> np.ndarray:
    """Q(g) = s * round(g_n), Eq. (4)."""
    return np.asarray(code, dtype=np.float64) * float(s)


def error_all(g, code, s: float) -> float:
    """E(G) = sum |g - Q(g)| / (N(G) g_max), Eq. (5)."""
    g = np.asarray(g, dtype=np.float64).reshape(-1)
    gmax = np.abs(g).max()
    return float(np.abs(g - dequantized(code, s).reshape(-1)).sum() / (g.size * gmax))


def large_gradient_index(g, alpha: float) -> np.ndarray:
    """Indices of G_L: the ceil(alpha*N) largest magnitudes (ties: lower index first)."""
    a = np.abs(np.asarray(g, dtype=np.float64).reshape(-1))
    n_l = int(math.ceil(alpha * a.size - 1e-12))
    order = np.argsort(-a, kind="stable")
    return order[:n_l]


def split_large(g, alpha: float, gamma: float):
    """(idx of G_in, idx of G_out): large gradients inside / outside gamma*g_max."""
    gf = np.asarray(g, dtype=np.float64).reshape(-1)
    idx = large_gradient_index(gf, alpha)
    gmax = np.abs(gf).max()
    inside = np.abs(gf[idx]) <= gamma * gmax
    return idx[inside], idx[~inside]


def error_large(g, code, s: float, alpha: float) -> float:
    """E(G_L), Eq. (6)."""
    gf = np.asarray(g, dtype=np.float64).reshape(-1)
    idx = large_gradient_index(gf, alpha)
    gmax = np.abs(gf).max()
    qf = dequantized(code, s).reshape(-1)
    return float(np.abs(gf[idx] - qf[idx]).sum() / (idx.size * gmax))


def error_large_split(g, code, s: float, alpha: float, gamma: float) -> float:
    """E(G_L) written as the clip-in sum plus the clip-out sum, Eq. (7)."""
    gf = np.asarray(g, dtype=np.float64).reshape(-1)
    i_in, i_out = split_large(gf, alpha, gamma)
    gmax = np.abs(gf).max()
    qf = dequantized(code, s).reshape(-1)
    tot = np.abs(gf[i_in] - qf[i_in]).sum() + np.abs(gf[i_out] - qf[i_out]).sum()
    return float(tot / ((i_in.size + i_out.size) * gmax))


def ulg_counts(n_in: int, n_out: int, gamma: float, bits: int, gmax: float = 1.0) -> float:
    """U(G_L) from counts, supplement Eq. (i): (U_in N_in + U_out N_out)/(N(G_L) g_max)."""
    u_in = gamma * gmax / (2 ** bits - 2)
    u_out = (1.0 - gamma) * gmax
    return (u_in * n_in + u_out * n_out) / ((n_in + n_out) * gmax)


def ulg_ratios(r_in: float, r_out: float, gamma: float, bits: int, alpha: float) -> float:
    """U(G_L) from ratios, Eq. (8): (gamma/(2^b-2) R_in + (1-gamma) R_out)/alpha."""
    return (gamma / (2 ** bits - 2) * r_in + (1.0 - gamma) * r_out) / alpha


def dulg_dgamma_approx(r_in: float, r_out: float, bits: int, alpha: float) -> float:
    """Eq. (12): derivative of U(G_L) w.r.t. gamma with dR_out/dgamma taken as 0."""
    return (r_in / (2 ** bits - 2) - r_out) / alpha


def optimal_ratios(bits: int, alpha: float):
    """Eq. (14): (R_in*, R_out*)."""
    return (2 ** bits - 2) / (2 ** bits - 1) * alpha, alpha / (2 ** bits - 1)

"""Oracle for the offline budget allocation (sensitivity-conditioned token budgets, Eq. 1-5).

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).  Plain fp64 numpy, one function per
equation, in the paper's order and notation.  Readings where the paper is silent: the
percentiles of Eq. 2 over the m candidate layers use linear interpolation between order
statistics (fractional rank p(m-1)/100); P90 == P10 gives S~ = 0.5 for every layer; the
ceiling of Eq. 5 does not bump a product that is an integer up to fp64 rounding
(K = ceil(r V0 - 1e-9)).
"""
from __future__ import annotations

import math
from fractions import Fraction

import numpy as np


def sensitivity(diff_norm, ref_norm, eta: float) -> float:
    """Eq. 1 for one layer: median over calibration samples of ||x^q - x|| / (||x|| + eta)."""
    a = np.asarray(diff_norm, np.float64)
    b = np.asarray(ref_norm, np.float64)
    ratio = np.sort(a / (b + eta))
    n = ratio.size
    return float(ratio[n // 2]) if n % 2 else float(0.5 * (ratio[n // 2 - 1] + ratio[n // 2]))


def percentile_linear(values, p: float) -> float:
    v = np.sort(np.asarray(values, np.float64))
    pos = p * (v.size - 1) / 100.0
    lo = int(math.floor(pos))
    hi = min(lo + 1, v.size - 1)
    return float(v[lo] + (v[hi] - v[lo]) * (pos - lo))


def normalize_sensitivity(S):
    """Eq. 2: rescale by the 10th-90th percentile range, clip to [0.1, 0.9]."""
    S = np.asarray(S, np.float64)
    p10, p90 = percentile_linear(S, 10.0), percentile_linear(S, 90.0)
    if p90 == p10:
        return np.full(S.shape, 0.5)
    return np.clip((S - p10) / (p90 - p10), 0.1, 0.9)


def layer_shares(S_norm, tau: float):
    """Eq. 3: softmax of (1 - S~)/tau over the ordered candidate layers (less sensitive, more drop)."""
    z = (1.0 - np.asarray(S_norm, np.float64)) / tau
    e = np.exp(z - z.max())
    return e / e.sum()


def keep_schedule(pi, p_min: float):
    """Eq. 4: d_i = (1 - p_min) pi_i; r_i = max(p_min, 1 - sum_{j<=i} d_j): non-increasing, floored."""
    d = (1.0 - p_min) * np.asarray(pi, np.float64)
    r = np.empty(d.size)
    acc = 0.0
    for i in range(d.size):
        acc += d[i]
        r[i] = max(p_min, 1.0 - acc)
    return r


def budgets(r, V0: int):
    """Eq. 5: K = ceil(r V0), exact on the binary value of r, with the 1e-9 guard."""
    eps = Fraction(1, 10 ** 9)
    return np.array([int(math.ceil(Fraction(float(x)) * V0 - eps)) for x in np.asarray(r, np.float64)], np.int32)


def make_recipe(S, tau: float, p_min: float, V0: int):
    s_norm = normalize_sensitivity(S)
    pi = layer_shares(s_norm, tau)
    r = keep_schedule(pi, p_min)
    return dict(s_norm=s_norm, pi=pi, r=r, K=budgets(r, V0))


def layer_cost(S: int, d: int, F: int) -> float:
    """C_l as a function of the executed sequence length S = T + V_l (GFLOPs-estimation appendix).
    The paper names the two terms but prints no formula; the reading used here is the usual count
    for a LLaMA-style block, 2 FLOPs per multiply-add: token-wise projections and SwiGLU MLP
    2 S (4 d^2 + 3 d F), attention scores and values 4 S^2 d (full, not causal-halved)."""
    return 2.0 * S * (4.0 * d * d + 3.0 * d * F) + 4.0 * float(S) * S * d


def gflops_ratio(V_hat, V0: int, T: int, d: int, F: int, F_vt: float = 0.0, F_pj: float = 0.0) -> float:
    """GFLOPs ratio (percent) of a pruning recipe: (F_VT + F_PJ + sum_l C_l(V_l, T)) over the same with
    V_l = V0 in every layer.  V_hat[l] = visual tokens executed by layer l."""
    pruned = F_vt + F_pj + sum(layer_cost(T + int(v), d, F) for v in V_hat)
    base = F_vt + F_pj + len(V_hat) * layer_cost(T + V0, d, F)
    return 100.0 * pruned / base

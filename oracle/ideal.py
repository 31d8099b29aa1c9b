"""Analytic (fp64) statements of the paper's estimators.  TEST INFRASTRUCTURE ONLY.

These are the formulas of the paper written out in exact-arithmetic form; the tests hold
the C oracle's *behaviour* (frequencies over all 2^24 thresholds, sample moments) against
them, and hold them against brute force.  Nothing here is used by the product path.

Notation follows the paper: a block ``a`` of non-negative magnitudes, ranked
``a1 <= a2 <= a3 <= a4`` for 2:4 (App. A.2); ``p_ij`` the probability of keeping the
pair (i, j); ``p_i`` the marginal probability of keeping element i; kept elements
are emitted as ``a_i / p_i`` (eq. (8)).
"""
from __future__ import annotations

from itertools import combinations
from typing import Dict, Tuple

import numpy as np

PAIRS = list(combinations(range(4), 2))  # (0,1),(0,2),(0,3),(1,2),(1,3),(2,3) in 0-based ranks


# ---------------------------------------------------------------------------
# 1:2  (Sec. 4.1, App. A.1)
# ---------------------------------------------------------------------------
def p_keep_first_1of2(a1: float, a2: float) -> float:
    """eq. (6): probability that the first element of the pair is kept."""
    a1, a2 = abs(a1), abs(a2)
    if a1 + a2 == 0.0:
        return 1.0
    return a1 / (a1 + a2)


def var_block_1of2(a1: float, a2: float) -> float:
    """Total block variance of MVUE 1:2: 2 a1 a2 (end of Sec. 4.1)."""
    return 2.0 * abs(a1) * abs(a2)


def var_block_1of2_general(a1: float, a2: float, v1: float) -> float:
    """eq. (5): block variance of any unbiased 1:2 estimator as a function of v1 (a1, a2 > 0)."""
    return v1 * a1 - a1 ** 2 + a2 ** 2 * v1 / (v1 - a1) - a2 ** 2


# ---------------------------------------------------------------------------
# 2:4  (Sec. 4.2, App. A.2, App. A.3)
# ---------------------------------------------------------------------------
def marginals_opt_2of4(a_sorted) -> np.ndarray:
    """Optimal marginals: eq. (12) if no p_i would exceed 1, else eq. (14) with the largest kept surely."""
    a = np.asarray(a_sorted, dtype=np.float64)
    s = a.sum()
    if s == 0.0:
        return np.array([0.0, 0.0, 1.0, 1.0])
    if a[3] <= a[0] + a[1] + a[2]:
        return 2.0 * a / s
    rest = a[:3].sum()
    p = np.empty(4)
    p[3] = 1.0
    p[:3] = a[:3] / rest if rest > 0 else np.array([0.0, 0.0, 1.0])
    return p


def pair_probs_opt_2of4(a_sorted) -> Tuple[Dict[Tuple[int, int], float], int]:
    """App. A.2: the pair probabilities p_ij (0-based ranks) and the case number."""
    a1, a2, a3, a4 = (float(v) for v in a_sorted)
    s = a1 + a2 + a3 + a4
    p = {pr: 0.0 for pr in PAIRS}
    if a4 <= 2 * a1 + a3:
        case = 1
        p[(0, 2)] = (2 * a1 + a3 - a4) / (2 * s)
        p[(0, 3)] = (2 * a1 - a3 + a4) / (2 * s)
        p[(1, 2)] = (2 * a2 + a3 - a4) / (2 * s)
        p[(1, 3)] = (2 * a2 - a3 + a4) / (2 * s)
        p[(2, 3)] = (-a1 - a2 + a3 + a4) / s
    elif a4 <= a1 + a2 + a3:
        case = 2
        p[(0, 3)] = 2 * a1 / s
        p[(1, 2)] = (a1 + a2 + a3 - a4) / s
        p[(1, 3)] = (-a1 + a2 - a3 + a4) / s
        p[(2, 3)] = (-a1 - a2 + a3 + a4) / s
    else:
        case = 3
        rest = a1 + a2 + a3
        p[(0, 3)] = a1 / rest
        p[(1, 3)] = a2 / rest
        p[(2, 3)] = a3 / rest
    return p, case


def marginals_from_pairs(p: Dict[Tuple[int, int], float]) -> np.ndarray:
    m = np.zeros(4)
    for (i, j), v in p.items():
        m[i] += v
        m[j] += v
    return m


def var_block(a, p) -> float:
    """eq. (10): sum_i a_i^2/p_i - a_i^2 for an unbiased estimator with marginals p (0/0 -> 0)."""
    a = np.asarray(a, dtype=np.float64)
    p = np.asarray(p, dtype=np.float64)
    out = 0.0
    for ai, pi in zip(a, p):
        if ai == 0.0:
            continue
        if pi <= 0.0:
            return np.inf
        out += ai * ai / pi - ai * ai
    return out


def var_opt_2of4_closed(a_sorted) -> float:
    """Closed forms: sum_{i<j} a_i a_j - 1/2 sum a_i^2 when no element dominates (App. A.3);
    2(a1a2 + a1a3 + a2a3) when a4 >= a1+a2+a3 (eq. (10) with eq. (14))."""
    a = np.asarray(a_sorted, dtype=np.float64)
    if a[3] <= a[0] + a[1] + a[2]:
        cross = sum(a[i] * a[j] for i, j in PAIRS)
        return cross - 0.5 * float((a * a).sum())
    return 2.0 * (a[0] * a[1] + a[0] * a[2] + a[1] * a[2])


def marginals_approx_2of4(a) -> np.ndarray:
    """Sec. 4.4: two draws without replacement, each proportional to magnitude."""
    a = np.abs(np.asarray(a, dtype=np.float64))
    s = a.sum()
    p = np.zeros(4)
    for i in range(4):
        p[i] = a[i] / s + sum(a[k] / s * a[i] / (s - a[k]) for k in range(4) if k != i)
    return p


def pair_probs_approx_2of4(a) -> Dict[Tuple[int, int], float]:
    """Sec. 4.4: probability that the unordered pair (i, j) is kept = P(i then j) + P(j then i)."""
    a = np.abs(np.asarray(a, dtype=np.float64))
    s = a.sum()
    out = {}
    for i, j in PAIRS:
        out[(i, j)] = a[i] / s * a[j] / (s - a[i]) + a[j] / s * a[i] / (s - a[j])
    return out


def marginals_approx_alg1(a) -> np.ndarray:
    """Alg. 1 (App. B.1) writes the same inclusion probability as  v (1 + q - vv),  v = a/sum, vv = v/(1-v), q = sum vv."""
    a = np.abs(np.asarray(a, dtype=np.float64))
    v = a / a.sum()
    vv = v / (1.0 - v)
    return v * (1.0 + vv.sum() - vv)


def var_approx_2of4(a) -> float:
    """Block variance (eq. (10)) of approx-MVUE: sum_i a_i^2 (1/p_i - 1) with the marginals of Sec. 4.4."""
    a = np.abs(np.asarray(a, dtype=np.float64))
    return var_block(a, marginals_approx_2of4(a))


# ---------------------------------------------------------------------------
# the 1:2 comparison estimators of Table "1:2 ablation" (negative / positive controls)
# each maps (pairs [n,2], eps [n]) -> theta [n,2]
# ---------------------------------------------------------------------------
def _emit(x, keep_first, v_first, v_second):
    out = np.zeros_like(x, dtype=np.float64)
    out[:, 0] = np.where(keep_first, v_first, 0.0)
    out[:, 1] = np.where(keep_first, 0.0, v_second)
    return out


def est_greedy(x, eps):
    """keep the larger magnitude unchanged (minimum MSE)."""
    x = np.asarray(x, dtype=np.float64)
    return _emit(x, np.abs(x[:, 0]) > np.abs(x[:, 1]), x[:, 0], x[:, 1])


def est_biased(x, eps):
    """p = |a1|/(|a1|+|a2|) but values left unscaled."""
    x = np.asarray(x, dtype=np.float64)
    p = np.abs(x[:, 0]) / (np.abs(x[:, 0]) + np.abs(x[:, 1]))
    return _emit(x, eps < p, x[:, 0], x[:, 1])


def est_uniform(x, eps):
    x = np.asarray(x, dtype=np.float64)
    return _emit(x, eps < 0.5, x[:, 0], x[:, 1])


def est_unbiased_uniform(x, eps):
    """p = 1/2, values doubled: unbiased, block variance a1^2 + a2^2."""
    x = np.asarray(x, dtype=np.float64)
    return _emit(x, eps < 0.5, 2 * x[:, 0], 2 * x[:, 1])


def est_mvue_1of2(x, eps):
    """eq. (6) in fp64."""
    x = np.asarray(x, dtype=np.float64)
    s = np.abs(x[:, 0]) + np.abs(x[:, 1])
    p = np.abs(x[:, 0]) / s
    return _emit(x, eps < p, np.sign(x[:, 0]) * s, np.sign(x[:, 1]) * s)

"""Pins for the oracle's optimal MVUE 2:4 estimator (Sec. 4.2, 4.3, App. A.2, A.3 of the paper).

Three independent anchors:
  * the paper's printed pair probabilities / marginals / closed-form variances (``oracle.ideal``),
    against which the C oracle's counts over all 2^24 uniforms are held;
  * brute force over every 2:4 pair distribution on a simplex grid and a numerical solve of the
    constrained problem of Sec. 4.2: nothing unbiased has a smaller variance;
  * structure: what a degenerate block (two or more zeros) must produce.
"""
from itertools import combinations, product

import numpy as np
import pytest

from oracle import ideal

PAIR_ORDER = list(combinations(range(4), 2))

QUADS = [
    (1.0, 2.0, 3.0, 4.0),               # case 1
    (4.0, 3.0, 2.0, 1.0),               # case 1, reversed positions
    (1.0, 1.0, 1.0, 1.0),               # all equal
    (-2.0, 2.0, -2.0, 2.5),             # signs, near-equal
    (1.0, 5.0, 2.0, 7.0),               # case 2: 2*1+5=7 -> boundary case1/2
    (1.0, 5.0, 2.0, 7.5),               # case 2
    (1.0, 2.0, 3.0, 6.0),               # boundary case 2/3
    (0.5, -0.25, 0.125, 9.0),           # case 3
    (1e-3, 1.0, 1e3, 1e6),              # case 3, wide range
    (3.0, 0.0, 4.0, 5.0),               # one zero
    (0.0, 0.0, 4.0, 5.0),               # two zeros
    (0.0, -7.0, 0.0, 0.0),              # three zeros
    (0.0, 0.0, 0.0, 0.0),
    (0.3, 0.3, 0.9, 0.9),               # ties across pairs
    (2.0, 2.0, 2.0, 6.0),               # a4 = a1+a2+a3 exactly
    (1.25, 3.5, 3.5, 4.75),
    (1.1e-38, 2.3e-38, 0.9e-38, 3.0e-38),   # around the smallest normal
    (1e37, 2e37, 1.5e37, 3e37),
]


def _ranked(x):
    """ranks: magnitude ascending, higher position first among equals (the oracle's documented order)."""
    m = np.abs(np.asarray(x, dtype=np.float64))
    order = sorted(range(4), key=lambda i: (m[i], -i))
    return order, m[order]


# ---------------------------------------------------------------------------
# the paper's tables themselves
# ---------------------------------------------------------------------------
def test_printed_pair_probabilities_are_valid_and_meet_the_optimality_conditions():
    rng = np.random.default_rng(10)
    seen = set()
    for _ in range(20000):
        a = np.sort(np.exp(rng.normal(0, rng.choice([0.3, 1.0, 2.5]), 4)))
        p, case = ideal.pair_probs_opt_2of4(a)
        seen.add(case)
        v = np.array(list(p.values()))
        assert abs(v.sum() - 1) < 1e-12 and v.min() > -1e-12 and v.max() < 1 + 1e-12
        marg = ideal.marginals_from_pairs(p)
        assert np.allclose(marg, ideal.marginals_opt_2of4(a), atol=1e-12)       # eqs. (12) / (14)
        if case in (1, 2):
            assert np.isclose(marg[0] / marg[1], a[0] / a[1])                  # the example below the case-1 table
        assert p[(0, 1)] == 0.0
    assert seen == {1, 2, 3}


def test_cases_agree_on_their_common_boundaries():
    rng = np.random.default_rng(11)
    for _ in range(200):
        a1, a2, a3 = np.sort(np.exp(rng.normal(0, 1, 3)))
        for a4, pair in ((2 * a1 + a3, (1, 2)), (a1 + a2 + a3, (2, 3))):
            if a4 < a3:
                continue
            lo, _ = ideal.pair_probs_opt_2of4((a1, a2, a3, a4 * (1 - 1e-13)))
            hi, _ = ideal.pair_probs_opt_2of4((a1, a2, a3, a4 * (1 + 1e-13)))
            assert all(abs(lo[k] - hi[k]) < 1e-9 for k in lo)


def test_closed_form_variance_equals_definition_with_optimal_marginals():
    rng = np.random.default_rng(12)
    for _ in range(5000):
        a = np.sort(np.exp(rng.normal(0, 2, 4)))
        assert np.isclose(ideal.var_block(a, ideal.marginals_opt_2of4(a)), ideal.var_opt_2of4_closed(a), rtol=1e-9)


# ---------------------------------------------------------------------------
# the C oracle against the tables: every one of the 2^24 uniforms
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("quad", QUADS)
def test_pair_frequencies_unbiasedness_and_variance_over_all_uniforms(oracle, quad):
    x = np.array(quad, dtype=np.float32)
    order, a = _ranked(x)
    a = np.abs(x.astype(np.float64))[order]
    counts, mean, second = oracle.enumerate_2of4(x)
    assert counts.sum() == 1 << 24
    s = a.sum()
    if (a > 0).sum() >= 3:
        p_rank, case = ideal.pair_probs_opt_2of4(a)
        want = np.zeros(6)
        for (ri, rj), pv in p_rank.items():
            pi, pj = sorted((order[ri], order[rj]))
            want[PAIR_ORDER.index((pi, pj))] += pv
        assert np.abs(counts / 2.0 ** 24 - want).max() <= 3 * 2.0 ** -23
        var = (second - mean ** 2).sum()
        closed = ideal.var_opt_2of4_closed(a)
        assert np.isclose(var, closed, rtol=1e-5, atol=1e-6 * s * s)
    else:
        # two or more zeros: nothing random; non-zeros survive unchanged, pads are the lowest-index zeros
        assert (counts > 0).sum() == 1
        assert np.array_equal(mean, x.astype(np.float64))
        kept = PAIR_ORDER[int(np.argmax(counts))]
        nzpos = [i for i in range(4) if x[i] != 0]
        zeros = [i for i in range(4) if x[i] == 0]
        assert sorted(nzpos + zeros[: 2 - len(nzpos)]) == list(kept)
    assert np.all(np.abs(mean - x.astype(np.float64)) <= 3 * 2.0 ** -23 * s + 1e-300)


def test_kept_values_follow_a_over_p(oracle):
    rng = np.random.default_rng(13)
    n_case = {1: 0, 2: 0, 3: 0}
    for _ in range(6000):
        x = (rng.choice([-1, 1], 4) * np.exp(rng.normal(0, rng.choice([0.3, 1.5, 3.0]), 4))).astype(np.float32)
        eps = float(rng.integers(0, 1 << 24)) / (1 << 24)
        pos, val, case = oracle.select_2of4(x, eps)
        n_case[case] += 1
        assert pos[0] < pos[1]
        m = np.abs(x)
        order, _ = _ranked(x)
        a = m[order]                                         # float32 magnitudes, ranked
        s123 = np.float32(np.float32(a[0] + a[1]) + a[2])
        s = np.float32(s123 + a[3])
        for p_, v_ in zip(pos, val):
            assert np.sign(v_) == np.sign(x[p_])
        if case == 3:
            big = order[3]
            assert big in pos
            other = pos[0] if pos[1] == big else pos[1]
            assert val[pos.index(big)] == x[big]             # p = 1: unchanged
            assert abs(val[pos.index(other)]) == s123        # a_i / (a_i / (a1+a2+a3))
            assert a[3] > s123
        else:
            assert abs(val[0]) == abs(val[1]) == np.float32(0.5) * s   # a_i / (2 a_i / sum)
            assert a[3] <= s123
            assert (case == 1) == bool(a[3] <= np.float32(np.float32(2) * a[0] + a[2]))
    assert min(n_case.values()) > 300


# ---------------------------------------------------------------------------
# minimum variance: brute force, independent of the tables
# ---------------------------------------------------------------------------
def _simplex_grid(n_parts, dims):
    """all vectors of `dims` non-negative multiples of 1/n_parts summing to 1"""
    out = []
    for cuts in combinations(range(n_parts + dims - 1), dims - 1):
        prev, row = -1, []
        for c in cuts + (n_parts + dims - 1,):
            row.append(c - prev - 1)
            prev = c
        out.append(row)
    return np.array(out, dtype=np.float64) / n_parts


def test_no_pair_distribution_on_a_simplex_grid_beats_the_oracle(oracle):
    grid = _simplex_grid(20, 6)                                # 53 130 distributions over the 6 masks
    assert len(grid) == 53130
    member = np.zeros((6, 4))
    for k, (i, j) in enumerate(PAIR_ORDER):
        member[k, i] = member[k, j] = 1
    marg = grid @ member                                       # p_i of every grid point
    rng = np.random.default_rng(14)
    blocks = [np.sort(np.exp(rng.normal(0, sd, 4))) for sd in (0.2, 1.0, 2.0) for _ in range(12)]
    blocks += [np.array([1.0, 2.0, 3.0, 4.0]), np.array([1.0, 1.0, 1.0, 1.0]), np.array([1.0, 2.0, 3.0, 6.0]),
               np.array([0.1, 0.2, 0.3, 5.0]), np.array([1.0, 1.0, 4.0, 4.0])]
    for a in blocks:
        with np.errstate(divide="ignore"):
            var = ((a * a)[None, :] / marg - (a * a)[None, :]).sum(1)      # eq. (10); p_i = 0 -> inf (biased)
        best = var.min()
        # the oracle's variance, measured from its behaviour over all uniforms on a permuted block
        perm = rng.permutation(4)
        x = (a[np.argsort(perm)] * rng.choice([-1, 1], 4)).astype(np.float32)
        counts, mean, second = oracle.enumerate_2of4(x)
        got = (second - mean ** 2).sum()
        assert got <= best * (1 + 1e-5) + 1e-9, (a, got, best)
        assert np.isclose(got, ideal.var_opt_2of4_closed(a), rtol=2e-5)


def test_constrained_minimisation_reproduces_the_marginals():
    """min sum a_i^2/p_i  s.t. sum p_i = 2, 0 < p_i <= 1 (Sec. 4.2) solved numerically."""
    from scipy.optimize import minimize
    rng = np.random.default_rng(15)
    for _ in range(40):
        a = np.sort(np.exp(rng.normal(0, rng.choice([0.3, 1.5]), 4)))
        res = minimize(lambda p: float((a * a / p).sum()), x0=np.full(4, 0.5), method="SLSQP",
                       bounds=[(1e-9, 1.0)] * 4, constraints=[{"type": "eq", "fun": lambda p: p.sum() - 2}],
                       options={"ftol": 1e-13, "maxiter": 500})
        assert res.status in (0, 8)            # 8: line search stalls once converged on the p_i = 1 face
        want = ideal.marginals_opt_2of4(a)
        assert np.allclose(res.x, want, atol=1e-4)
        assert float((a * a / res.x).sum()) >= float((a * a / want).sum()) * (1 - 1e-9)


def test_value_that_depends_on_the_partner_only_adds_variance():
    """For fixed pair probabilities, unbiased values that vary with the partner raise the variance
    (the constant a_i/p_i of eq. (8) is the minimiser)."""
    rng = np.random.default_rng(16)
    for _ in range(200):
        a = np.sort(np.exp(rng.normal(0, 1, 4)))
        p, _ = ideal.pair_probs_opt_2of4(a)
        base = ideal.var_block(a, ideal.marginals_from_pairs(p))
        i = int(rng.integers(0, 4))
        pairs_i = [pr for pr in PAIR_ORDER if i in pr and p[pr] > 1e-6]
        if len(pairs_i) < 2:
            continue
        pi = sum(p[pr] for pr in PAIR_ORDER if i in pr)
        v = {pr: a[i] / pi for pr in pairs_i}
        d = 0.1 * a[i]
        v[pairs_i[0]] += d / p[pairs_i[0]]
        v[pairs_i[1]] -= d / p[pairs_i[1]]                       # still unbiased
        second = sum(p[pr] * v[pr] ** 2 for pr in pairs_i)
        assert second - a[i] ** 2 > a[i] ** 2 / pi - a[i] ** 2


# ---------------------------------------------------------------------------
# Sec. 4.3 / App. A.3
# ---------------------------------------------------------------------------
def test_2of4_never_worse_than_two_1of2_blocks():
    rng = np.random.default_rng(17)
    a = np.exp(rng.normal(0, 2, (100000, 4)))
    srt = np.sort(a, axis=1)
    dom = srt[:, 3] > srt[:, :3].sum(1)
    cross = sum(srt[:, i] * srt[:, j] for i, j in PAIR_ORDER)
    v24 = np.where(dom, 2 * (srt[:, 0] * srt[:, 1] + srt[:, 0] * srt[:, 2] + srt[:, 1] * srt[:, 2]),
                   cross - 0.5 * (srt ** 2).sum(1))
    v12 = 2 * a[:, 0] * a[:, 1] + 2 * a[:, 2] * a[:, 3]
    assert np.all(v24 <= v12 * (1 + 1e-12))
    # D = -(A+B)^2/2 with A = a1-a4, B = a2-a3 where the non-dominant closed form applies
    nd = ~dom
    D = (cross - 0.5 * (a ** 2).sum(1)) - v12                  # positions, as in the proof
    A, B = a[:, 0] - a[:, 3], a[:, 1] - a[:, 2]
    assert np.allclose(D[nd], -0.5 * (A[nd] + B[nd]) ** 2, rtol=1e-9, atol=1e-9)
    for j in np.flatnonzero(dom)[:50]:
        assert np.isclose(v24[j], ideal.var_opt_2of4_closed(srt[j]))


# ---------------------------------------------------------------------------
# tensor level
# ---------------------------------------------------------------------------
def test_tensor_prune_matches_block_rule_and_layout(oracle):
    rng = np.random.default_rng(18)
    T, O = 32, 40
    g = (rng.standard_normal((T, O)) * np.exp(3 * rng.standard_normal((T, O)))).astype(np.float32)
    g[rng.random((T, O)) < 0.5] = 0.0
    seed, stream = 2 ** 40 + 12345, 3
    vals, meta, dense = oracle.prune_2of4(g, seed, stream, want_dense=True)
    for q in range(T // 4):
        for o in range(O):
            u = oracle.block_u24(seed, stream, q * O + o)
            pos, val, _ = oracle.select_2of4(g[4 * q:4 * q + 4, o], u / 2.0 ** 24)
            G, i = q // 4, q % 4
            assert vals[G, o, 2 * i] == np.float32(val[0]) and vals[G, o, 2 * i + 1] == np.float32(val[1])
            nib = (int(meta[G, o]) >> (4 * i)) & 0xF
            assert (nib & 3, nib >> 2) == pos
            col = np.zeros(4, dtype=np.float32)
            col[pos[0]], col[pos[1]] = val
            assert np.array_equal(dense[4 * q:4 * q + 4, o], col)
    assert np.array_equal(oracle.nm_decompress(vals, meta), dense)
    assert ((dense != 0).reshape(T // 4, 4, O).sum(1) <= 2).all()


def test_tensor_unbiasedness_over_seeds(oracle):
    rng = np.random.default_rng(19)
    O = 128
    g = np.zeros((16, O), dtype=np.float32)
    g[:4] = (rng.choice([-1, 1], (4, O)) * np.exp(2.5 * rng.standard_normal((4, O)))).astype(np.float32)
    g[:4][rng.random((4, O)) < 0.1] = 0.0
    n = 6000
    acc = np.zeros((4, O))
    for seed in range(n):
        _, _, dense = oracle.prune_2of4(g, seed, 7, want_dense=True)
        acc += dense[:4]
    mean = acc / n
    a = np.abs(g[:4].astype(np.float64))
    var = np.zeros((4, O))
    for o in range(O):
        order, ar = _ranked(g[:4, o])
        if (ar > 0).sum() < 3:
            continue
        p = ideal.marginals_opt_2of4(ar)
        for r, pos in enumerate(order):
            var[pos, o] = ar[r] ** 2 / p[r] - ar[r] ** 2 if ar[r] > 0 else 0.0
    live = var > 1e-30
    z = (mean - g[:4])[live] / np.sqrt(var[live] / n)
    assert np.abs(z).max() < 4.7
    assert abs((z ** 2).sum() - live.sum()) < 6 * np.sqrt(2 * live.sum())
    assert np.array_equal(mean[~live], g[:4][~live].astype(np.float64))      # p = 1 elements are exact


def test_expected_macs_when_both_operands_are_2of4():
    """Sec. 6: two random 2:4 masks overlap in 0, 1 or 2 positions with probability 1/6, 4/6, 1/6 -> 1 MAC."""
    masks = [set(c) for c in combinations(range(4), 2)]
    overlaps = [len(m & masks[0]) for m in masks]
    assert sorted(overlaps) == [0, 1, 1, 1, 1, 2]
    assert sum(overlaps) / 6 == 1.0
    rows = [ln.split() for ln in open(__file__.replace("test_oracle_2of4.py", "golden/paper_worked_values.txt"))
            if ln.strip() and not ln.startswith("#")]
    vals = {r[0]: float(r[1]) for r in rows}
    assert vals["expected_macs_both_operands_2of4"] == sum(overlaps) / 6
    assert vals["op_cost_m4_mul_equiv"] == (22 + 5) / 4 + 10 * 4 + 4
    assert vals["op_cost_m2_mul_equiv"] == (1 + 1) / 4 + 3 * 4

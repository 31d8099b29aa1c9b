"""Pins for the oracle's approx-MVUE 2:4 estimator (Sec. 4.4; Alg. 1 of App. B.1).

Anchors other than the oracle itself:
  * the section's draw probabilities  a_i/sum  and  a_j/(sum - a_i), against the oracle's counts over
    all 2^24 uniforms of each draw;
  * the section's inclusion probability, and Alg. 1's  v(1+q-vv)  form of it (``oracle.ideal``, binary64);
  * unbiasedness and the variance definition (eq. (10)) evaluated with those exact counts;
  * the section's claim that the variance stays below twice the optimal one (its figure's scan);
  * structure: what blocks with zeros, ties, huge dynamic range must produce.
"""
from itertools import combinations

import numpy as np
import pytest

from oracle import ideal

PAIRS = list(combinations(range(4), 2))

QUADS = [
    (1.0, 2.0, 3.0, 4.0),
    (4.0, 3.0, 2.0, 1.0),
    (1.0, 1.0, 1.0, 1.0),
    (-2.0, 2.0, -2.0, 2.5),
    (0.5, -0.25, 0.125, 9.0),            # one dominant element
    (1e-3, 1.0, 1e3, 1e6),               # wide range
    (3.0, 0.0, 4.0, 5.0),                # one zero
    (1.25, 3.5, 3.5, 4.75),
    (1.1e-38, 2.3e-38, 0.9e-38, 3.0e-38),
    (1e37, 2e37, 1.5e37, 3e37),
]


def _draw_tables(oracle, x):
    """P1[i] and P2[i][j] from the oracle's counts over all 2^24 uniforms of each draw."""
    p1 = oracle.enumerate_approx_draw(x).astype(np.float64) / 2.0 ** 24
    p2 = np.zeros((4, 4))
    for i in range(4):
        if p1[i] > 0:
            p2[i] = oracle.enumerate_approx_draw(x, i).astype(np.float64) / 2.0 ** 24
    return p1, p2


@pytest.mark.parametrize("quad", QUADS)
def test_draw_frequencies_inclusion_probabilities_unbiasedness_variance(oracle, quad):
    x = np.array(quad, dtype=np.float32)
    a = np.abs(x.astype(np.float64))
    s = a.sum()
    p1, p2 = _draw_tables(oracle, x)
    # the two draws of Sec. 4.4
    assert np.abs(p1 - a / s).max() < 2.0 ** -22
    for i in range(4):
        if a[i] > 0:
            want = np.where(np.arange(4) == i, 0.0, a / (s - a[i]))
            assert np.abs(p2[i] - want).max() < 2.0 ** -22
            assert p2[i][i] == 0.0
    # inclusion probability: the section's formula and Alg. 1's v(1+q-vv)
    incl = p1 + (p1[:, None] * p2).sum(0)
    assert abs(incl.sum() - 2.0) < 1e-6
    assert np.abs(incl - ideal.marginals_approx_2of4(a)).max() < 1e-6
    assert np.abs(ideal.marginals_approx_2of4(a) - ideal.marginals_approx_alg1(a)).max() < 1e-12
    # kept values, expectation and variance with the enumerated probabilities
    mean = np.zeros(4)
    second = np.zeros(4)
    for i in range(4):
        for j in range(4):
            pij = p1[i] * p2[i][j]
            if pij == 0.0:
                continue
            # any uniforms that realise (i then j): bracket midpoints of the two walks
            e1 = (a[:i].sum() + 0.5 * a[i]) / s
            rest = np.where(np.arange(4) == i, 0.0, a)
            e2 = (rest[:j].sum() + 0.5 * rest[j]) / rest.sum()
            pos, val = oracle.select_2of4_approx(x, e1, e2)
            assert set(pos) == {i, j}
            for k, v in zip(pos, val):
                mean[k] += pij * v
                second[k] += pij * v * v
    # unbiased (Sec. 3, eq. (7)) up to the 2^-24 granularity of the uniforms: a probability is off by at most a
    # few 2^-24, and a kept value never exceeds the block's sum
    assert (np.abs(mean - x) <= 3e-6 * a + 4 * 2.0 ** -24 * s).all()
    var = float((second - x.astype(np.float64) ** 2).sum())
    want_var = ideal.var_approx_2of4(a)                                      # eq. (10) with the section's marginals
    assert abs(var - want_var) <= 2e-5 * max(want_var, float((a * a).sum())) + 8 * 2.0 ** -24 * s * s


def test_kept_values_follow_a_over_p(oracle):
    rng = np.random.default_rng(31)
    for _ in range(3000):
        x = (rng.choice([-1, 1], 4) * np.exp(rng.normal(0, rng.choice([0.3, 1.5, 3.0]), 4))).astype(np.float32)
        pos, val = oracle.select_2of4_approx(x, rng.random(), rng.random())
        a = np.abs(x.astype(np.float64))
        p = ideal.marginals_approx_2of4(a)
        assert pos[0] < pos[1]
        for k, v in zip(pos, val):
            assert np.sign(v) == np.sign(x[k])
            assert abs(abs(v) * p[k] / a[k] - 1.0) < 2e-6


def test_variance_is_between_the_optimal_one_and_twice_it():
    """The section's scan: blocks [a1, a2, a3, 1]; ratio to the optimal variance stays below 2 (and never below 1)."""
    worst = 0.0
    grid = np.arange(0.025, 1.0001, 0.025)
    for a1 in grid:
        for a2 in grid:
            for a3 in grid:
                a = np.sort(np.array([a1, a2, a3, 1.0]))
                vo = ideal.var_opt_2of4_closed(a)
                va = ideal.var_approx_2of4(a)
                assert va >= vo * (1 - 1e-9)
                worst = max(worst, va / vo)
    assert 1.8 < worst < 2.0
    # towards the edge where one element dominates (logarithmic steps, as the section's footnote does) the ratio
    # climbs to 2 without reaching it: there the dominant element is dropped with probability ~2(a1a2+a1a3+a2a3)/a4^2,
    # which costs as much variance again as the three small ones do.  (binary64 cancellation limits how far this
    # can be followed: 1e-4 is safe.)
    last = 0.0
    for e in (-1.0, -2.0, -3.0, -4.0):
        a = np.array([0.9 * 10.0 ** e, 1.3 * 10.0 ** e, 2.1 * 10.0 ** e, 1.0])
        r = ideal.var_approx_2of4(a) / ideal.var_opt_2of4_closed(a)
        assert last < r < 2.0
        last = r
    assert last > 1.999


def test_blocks_with_zeros_and_rounding_corners(oracle):
    eps = [0.0, 1e-7, 0.3, 0.5, 0.999, 1.0 - 2.0 ** -24]
    for e1 in eps:
        for e2 in eps:
            # all zero: positions 0 and 1, zeros keep the input sign bit
            pos, val = oracle.select_2of4_approx([0.0, -0.0, 0.0, 0.0], e1, e2)
            assert pos == (0, 1) and val[0] == 0.0 and val[1] == 0.0 and np.signbit(val[1]) and not np.signbit(val[0])
            # one non-zero: kept unchanged, padding on the lowest-index zero
            pos, val = oracle.select_2of4_approx([0.0, 0.0, -7.0, 0.0], e1, e2)
            assert pos == (0, 2) and val == (0.0, -7.0)
            pos, val = oracle.select_2of4_approx([5.0, 0.0, 0.0, 0.0], e1, e2)
            assert pos == (0, 1) and val == (5.0, 0.0)
            # two non-zeros: both kept (inclusion probability one), values within rounding of the inputs
            pos, val = oracle.select_2of4_approx([0.0, 3.0, 0.0, -4.0], e1, e2)
            assert pos == (1, 3) and abs(val[0] / 3.0 - 1) < 3e-7 and abs(val[1] / -4.0 - 1) < 3e-7
            # three non-zeros: the zero is never drawn
            pos, _ = oracle.select_2of4_approx([2.0, 0.0, 1.0, 3.0], e1, e2)
            assert 1 not in pos
            # subnormal sums lose resolution in eps*sum; a zero must still lose against a non-zero
            pos, _ = oracle.select_2of4_approx([1e-45, 0.0, 1e-45, 0.0], e1, e2)
            assert pos == (0, 2)


def test_huge_dynamic_range_keeps_small_elements_unbiased(oracle):
    """sum - a_l is the sum of the other three magnitudes: no cancellation when one element carries the sum."""
    x = np.array([1e-10, 2e-10, -3e-10, 1.0], dtype=np.float32)
    a = np.abs(x.astype(np.float64))
    p = ideal.marginals_approx_2of4(a)
    seen = set()
    for e1 in (0.0, 0.5):
        for e2 in np.linspace(0.01, 0.99, 23):
            pos, val = oracle.select_2of4_approx(x, e1 * 1e-10, e2)          # first draw lands on a small element
            pos2, val2 = oracle.select_2of4_approx(x, 0.9, e2)               # first draw lands on the dominant one
            for ps, vs in ((pos, val), (pos2, val2)):
                for k, v in zip(ps, vs):
                    assert np.isfinite(v) and abs(abs(v) * p[k] / a[k] - 1.0) < 2e-6
                    seen.add(k)
    assert seen == {0, 1, 2, 3}


def test_block_mapping_takes_two_words_of_a_separate_counter_stream(oracle):
    seed, stream = 0x0123456789ABCDEF, 77
    for blk in [0, 1, 2, 3, 5, 1022, (1 << 34) + 7, (1 << 41) + 2]:
        c = blk >> 1
        words = oracle.philox4x32_10([c & 0xFFFFFFFF, c >> 32, stream, 1], [seed & 0xFFFFFFFF, seed >> 32])
        assert oracle.block_u24_pair(seed, stream, blk) == (int(words[2 * (blk & 1)]) >> 8, int(words[2 * (blk & 1) + 1]) >> 8)
    # the two uniforms of a block are (empirically) uncorrelated, and unrelated to the one-uniform stream
    n = 1 << 16
    u = np.array([oracle.block_u24_pair(0, 0, b) for b in range(n)], dtype=np.float64) / 2.0 ** 24
    w = np.array([oracle.block_u24(0, 0, b) for b in range(n)], dtype=np.float64) / 2.0 ** 24
    for x, y in ((u[:, 0], u[:, 1]), (u[:, 0], w), (u[:, 1], w), (u[:-1, 1], u[1:, 0])):
        assert abs(np.corrcoef(x, y)[0, 1]) < 4.5 / np.sqrt(len(x))
    assert abs(u.mean() - 0.5) < 4.5 / np.sqrt(12 * 2 * n)


def test_tensor_prune_matches_block_rule_and_layout(oracle):
    rng = np.random.default_rng(38)
    T, O = 32, 40
    g = (rng.standard_normal((T, O)) * np.exp(3 * rng.standard_normal((T, O)))).astype(np.float32)
    g[rng.random((T, O)) < 0.5] = 0.0
    seed, stream = 2 ** 40 + 12345, 3
    vals, meta, dense = oracle.prune_2of4_approx(g, seed, stream, want_dense=True)
    for q in range(T // 4):
        for o in range(O):
            u1, u2 = oracle.block_u24_pair(seed, stream, q * O + o)
            pos, val = oracle.select_2of4_approx(g[4 * q:4 * q + 4, o], u1 / 2.0 ** 24, u2 / 2.0 ** 24)
            G, i = q // 4, q % 4
            assert vals[G, o, 2 * i] == np.float32(val[0]) and vals[G, o, 2 * i + 1] == np.float32(val[1])
            nib = (int(meta[G, o]) >> (4 * i)) & 0xF
            assert (nib & 3, nib >> 2) == pos
    assert np.array_equal(oracle.nm_decompress(vals, meta), dense)
    assert ((dense != 0).reshape(T // 4, 4, O).sum(1) <= 2).all()
    v2, m2, bad = oracle.nm_compress(dense, 2, 4)
    assert bad == 0 and np.array_equal(m2, meta) and np.array_equal(v2.view(np.uint32), vals.view(np.uint32))


def test_tensor_unbiasedness_over_seeds(oracle):
    rng = np.random.default_rng(39)
    O = 128
    g = np.zeros((16, O), dtype=np.float32)
    g[:4] = (rng.choice([-1, 1], (4, O)) * np.exp(2.5 * rng.standard_normal((4, O)))).astype(np.float32)
    g[:4][rng.random((4, O)) < 0.1] = 0.0
    n = 6000
    acc = np.zeros((4, O))
    for seed in range(n):
        _, _, dense = oracle.prune_2of4_approx(g, seed, 7, want_dense=True)
        acc += dense[:4]
    mean = acc / n
    a = np.abs(g[:4].astype(np.float64))
    var = np.zeros((4, O))
    for o in range(O):
        if (a[:, o] > 0).sum() < 3:
            continue
        p = ideal.marginals_approx_2of4(a[:, o])
        var[:, o] = np.where(a[:, o] > 0, a[:, o] ** 2 / np.maximum(p, 1e-300) - a[:, o] ** 2, 0.0)
    live = var > 1e-30
    z = (mean - g[:4])[live] / np.sqrt(var[live] / n)
    assert np.abs(z).max() < 4.7
    assert abs((z ** 2).sum() - live.sum()) < 6 * np.sqrt(2 * live.sum())

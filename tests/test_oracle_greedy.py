"""Pins for the oracle's Greedy N:M (the comparison method of the paper's tables: Sec. 4.1, the 1:2 ablation table
and its caption -- the traditional minimum-MSE method -- and Sec. 5, "keeping the N largest elements in each block").

Pinned by: a library sort on tie-free blocks, brute force over all masks for the minimum-MSE property the caption
states, hand-built ties, the bias the paper's illustration of the method shows (Sec. 4.1 figure: every sample of a
block is the same, so the average is biased), and the format round trip.
"""
from itertools import combinations

import numpy as np
import pytest

from paper_2203_10991_amd import synth


@pytest.mark.parametrize("m,n", [(2, 1), (4, 2)])
def test_keeps_the_n_largest_as_a_library_sort_ranks_them(oracle, m, n):
    rng = np.random.default_rng(m)
    for _ in range(3000):
        x = (rng.standard_normal(m) * np.exp(2 * rng.standard_normal(m))).astype(np.float32)
        if len(set(np.abs(x).tolist())) < m:
            continue
        want = sorted(np.argsort(np.abs(x))[-n:].tolist())
        assert oracle.select_greedy(x, n) == want


def test_greedy_is_the_minimum_mse_mask(oracle):
    """of all C(4,2) masks that keep values unchanged, the greedy one has the smallest squared error (the caption's claim)"""
    rng = np.random.default_rng(7)
    for _ in range(500):
        x = (rng.standard_normal(4) * np.exp(rng.standard_normal(4))).astype(np.float32)
        pos = oracle.select_greedy(x, 2)
        mse = lambda keep: float(sum(float(x[k]) ** 2 for k in range(4) if k not in keep))
        assert mse(pos) <= min(mse(c) for c in combinations(range(4), 2)) + 1e-12


def test_ties_keep_the_lower_positions(oracle):
    assert oracle.select_greedy([2.0, -2.0], 1) == [0]
    assert oracle.select_greedy([0.0, 0.0], 1) == [0]
    assert oracle.select_greedy([1.0, 1.0, 1.0, 1.0], 2) == [0, 1]
    assert oracle.select_greedy([0.0, 0.0, 5.0, 0.0], 2) == [0, 2]
    assert oracle.select_greedy([3.0, 7.0, -3.0, 3.0], 2) == [0, 1]
    assert oracle.select_greedy([-0.0, 0.0, -0.0, 4.0], 2) == [0, 3]


def test_greedy_is_biased_where_mvue_is_not(oracle):
    """the same block every time: the mean of any number of samples is the pruned block, off by the dropped element"""
    x = np.array([[3.0], [4.0]] * 8, dtype=np.float32)              # 8 pairs (3, 4) in one column
    _, _, dense = oracle.prune_greedy(x, 1, 2, want_dense=True)
    assert np.array_equal(dense[:, 0], np.array([0.0, 4.0] * 8, dtype=np.float32))
    # MVUE 1:2 on the same tensor averages to the input (z-test over seeds), greedy is 3 off at every even row
    acc = np.zeros_like(x, dtype=np.float64)
    n = 4000
    for seed in range(n):
        acc += oracle.prune_1of2(x, seed, 0, want_dense=True)[2]
    z = (acc / n - x) / np.sqrt(12.0 / n)                            # element variance |a1||a2| = 12 (Sec. 4.1)
    assert np.abs(z).max() < 4.5
    assert np.abs(dense - x).max() == 3.0


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n,m", [(1, 2), (2, 4)])
def test_tensor_prune_layout_and_round_trip(oracle, dtype, n, m):
    w = synth.Workload("greedy", 16 * 5, 24, 8, dtype, "2:4", 0.0, 2.0, 0.3)
    g = synth.make_g(w, seed=n)
    vals, meta, dense = oracle.prune_greedy(g, n, m, want_dense=True)
    assert np.array_equal(oracle.nm_decompress(vals, meta), dense)
    cv, cm, bad = oracle.nm_compress(dense, n, m)                   # the format's own compression agrees (zeros pad low)
    assert bad == 0 and np.array_equal(cm, meta) and np.array_equal(cv, vals)
    gf = g if dtype == "f32" else synth.bf16_to_f32(g)
    df = dense if dtype == "f32" else synth.bf16_to_f32(dense)
    for t0 in range(0, w.T, m):
        for o in range(w.O):
            blk = gf[t0:t0 + m, o]
            keep = oracle.select_greedy(blk, n)
            for k in range(m):
                want = blk[k] if k in keep else 0.0
                assert df[t0 + k, o] == want
    # values are copied bit for bit (a kept zero keeps its sign bit)
    kept = df != 0
    assert np.array_equal(df[kept], gf[kept])

"""Pins for the oracle's random source (Philox4x32-10 and the block -> uniform mapping)."""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_philox_known_answers(oracle):
    rows = [ln.split() for ln in open(GOLDEN) if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        w = [int(v, 16) for v in r]
        out = oracle.philox4x32_10(w[0:4], w[4:6])
        assert [int(v) for v in out] == w[6:10]


def test_block_mapping_uses_counter_blk_over_4_and_word_blk_mod_4(oracle):
    seed, stream = 0x0123456789ABCDEF, 77
    for blk in [0, 1, 2, 3, 4, 5, 1023, (1 << 34) + 6, (1 << 40) + 3]:
        c = blk >> 2
        words = oracle.philox4x32_10([c & 0xFFFFFFFF, c >> 32, stream, 0], [seed & 0xFFFFFFFF, seed >> 32])
        assert oracle.block_u24(seed, stream, blk) == int(words[blk & 3]) >> 8


def test_uniformity_and_independence_of_streams(oracle):
    n = 1 << 18
    u = np.array([oracle.block_u24(0, 0, b) for b in range(n)], dtype=np.float64)
    assert u.max() < (1 << 24) and u.min() >= 0
    eps = u / (1 << 24)
    # mean and variance of U[0,1): 1/2, 1/12 (5-sigma bands)
    assert abs(eps.mean() - 0.5) < 5 * np.sqrt(1 / 12 / n)
    assert abs(eps.var() - 1 / 12) < 5 * np.sqrt(1 / 180 / n)
    # chi-square on 256 equal buckets: mean 255, sd sqrt(510)
    hist = np.bincount((u // (1 << 16)).astype(np.int64), minlength=256)
    chi2 = ((hist - n / 256) ** 2 / (n / 256)).sum()
    assert abs(chi2 - 255) < 6 * np.sqrt(510)
    # lag-1 correlation across neighbouring blocks (which share a Philox call)
    r = np.corrcoef(eps[:-1], eps[1:])[0, 1]
    assert abs(r) < 5 / np.sqrt(n)
    # other seed / stream -> unrelated sequence
    v = np.array([oracle.block_u24(1, 0, b) for b in range(4096)])
    w = np.array([oracle.block_u24(0, 1, b) for b in range(4096)])
    assert (v != u[:4096]).mean() > 0.99 and (w != u[:4096]).mean() > 0.99 and (v != w).mean() > 0.99

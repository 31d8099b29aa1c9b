"""GPU: gradient values whose block sums overflow binary32, and infinities, through every other prune entry point
(transposed layout, Greedy, approx-MVUE 4:8, the 8-bit prunes with and without saturation, the producer form): both
sides follow IEEE arithmetic through the same formulas, so the outputs still agree bit for bit with the oracle.
(The token-major 16-bit prunes have the same test in test_gpu_prune.py.  A NaN is outside the contract.)"""
import numpy as np
import pytest
import torch

from paper_2203_10991_amd import synth
from gpu_util import to_dev, to_host

pytestmark = pytest.mark.gpu

BASE = [0.0, 1.0, -3.0, 1e37, 3.3e38, -3.3e38, 2.5e38, 1.7e38, 9e37, 3.4e38, 1.2e38, np.inf, -np.inf, 7.0, 1e30, 1e-40, -0.0]
T, O = 128, 256


def _tensor(dtype, seed):
    g = np.random.default_rng(seed).choice(np.array(BASE, dtype=np.float32), size=(T, O))
    return g if dtype == "f32" else synth.f32_to_bf16_bits(g)


def _same(got, want, what):
    for a, b, name in zip(got, want, what):
        a, b = np.ascontiguousarray(a), np.ascontiguousarray(b)
        assert a.shape == b.shape and np.array_equal(a.view(np.uint8), b.view(np.uint8)), name


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_transposed_greedy_and_4of8(oracle, dtype):
    import paper_2203_10991_amd as nm
    g = _tensor(dtype, 2)
    gd, gT = to_dev(g), to_dev(np.ascontiguousarray(g.T))
    for mode, cpu in ((0, oracle.prune_2of4), (1, oracle.prune_2of4_approx)):
        ov, om, _ = cpu(g, 1, 0)
        v, m = nm.mvue_prune_2of4_t(gT, seed=1, stream_id=0, mode=mode)
        _same((to_host(v), to_host(m)), (ov, om), (f"transposed 2:4 mode {mode} vals", "meta"))
    ov, om, _ = oracle.prune_1of2(g, 1, 0)
    v, m = nm.mvue_prune_1of2_t(gT, seed=1, stream_id=0)
    _same((to_host(v), to_host(m)), (ov, om), ("transposed 1:2 vals", "meta"))
    for n, mm in ((2, 4), (1, 2)):
        ov, om, od = oracle.prune_greedy(g, n, mm, want_dense=True)
        v, m, d = nm.nm_prune_greedy(gd, n, mm, want_dense=True)
        _same((to_host(v), to_host(m), to_host(d)), (ov, om, od), (f"greedy {n}:{mm} vals", "meta", "dense"))
    ov, om, od = oracle.prune_4of8_approx(g, 1, 0, want_dense=True)
    v, m, d = nm.mvue_prune_4of8_approx(gd, 1, 0, want_dense=True)
    torch.cuda.synchronize()
    _same((to_host(v), m.cpu().numpy().view(np.uint32), to_host(d)), (ov, om, od), ("4:8 vals", "meta", "dense"))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("scale", [2.0 ** -112, 1.0])            # the huge values in range of e5m2 / saturating
def test_8_bit_prunes(oracle, dtype, scale):
    import paper_2203_10991_amd as nm
    g = _tensor(dtype, 3)
    gd = to_dev(g)
    ov, om = oracle.prune_2of4_q8(g, seed=1, stream_id=0, mode=0, scale=scale)
    v, m = nm.mvue_prune_2of4_q8(gd, seed=1, stream_id=0, mode=0, scale=scale)
    _same((v.cpu().numpy(), m.cpu().numpy().view(np.uint32)), (ov, om), ("q8 2:4 codes", "meta"))
    ov, om = oracle.prune_1of2_q8(g, seed=1, stream_id=0, scale=scale)
    v, m = nm.mvue_prune_1of2_q8(gd, seed=1, stream_id=0, scale=scale)
    _same((v.cpu().numpy(), m.cpu().numpy().view(np.uint32)), (ov, om), ("q8 1:2 codes", "meta"))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_producer(oracle, dtype):
    import paper_2203_10991_amd as nm
    g = _tensor(dtype, 4)
    d32 = np.random.default_rng(5).choice(np.array([1.0, 0.5, 2.0, -1.0], dtype=np.float32), size=(T, O))   # no zeros: inf * 0 would be a NaN
    d = d32 if dtype == "f32" else synth.f32_to_bf16_bits(d32)
    og = oracle.act_backward(g, d)
    ov, om, _ = oracle.prune_2of4(og, 1, 0)
    gout, v, m = nm.mvue_prune_producer(to_dev(g), to_dev(d), nm="2:4", seed=1, stream_id=0)
    torch.cuda.synchronize()
    _same((to_host(gout), to_host(v), to_host(m)), (og, ov, om), ("producer g", "vals", "meta"))

"""Pins for the oracle's compressed format and update GEMM (eq. (3) of the paper).

The GEMM has a plain definition, so the anchor is a library routine: numpy's fp64 matmul
on an operand decompressed *in this file* (not by the oracle).  The format is anchored by
round trips, by invariants of N:M structure and by hand-built cases.
"""
import numpy as np
import pytest

from paper_2203_10991_amd import synth


def _decompress_here(vals, meta):
    """independent expansion of the group format (pure numpy)"""
    G, O, _ = vals.shape
    dense = np.zeros((G * 16, O), dtype=vals.dtype)
    for i in range(4):
        for s in range(2):
            pos = (meta.astype(np.int64) >> (4 * i + 2 * s)) & 3            # [G, O]
            rows = (np.arange(G)[:, None] * 16 + 4 * i + pos)                 # [G, O]
            dense[rows, np.arange(O)[None, :]] = vals[:, :, 2 * i + s]
    return dense


def _as_f64(a):
    return a.astype(np.float64) if a.dtype == np.float32 else synth.bf16_to_f32(a).astype(np.float64)


def _case(dtype, nm, T=64, O=24, I=20, seed=3):
    w = synth.Workload("t", T, O, I, dtype, nm, 0.0, 2.0, 0.3)
    return synth.make_g(w, seed), synth.make_h(w, seed)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("nm", ["1:2", "2:4"])
def test_round_trips_and_fused_equals_compress_of_dense(oracle, dtype, nm):
    g, _ = _case(dtype, nm)
    prune = oracle.prune_1of2 if nm == "1:2" else oracle.prune_2of4
    n, m = (1, 2) if nm == "1:2" else (2, 4)
    vals, meta, dense = prune(g, 11, 2, want_dense=True)
    # N:M structure along T
    nz = (_as_f64(dense) != 0).reshape(-1, m, g.shape[1]).sum(1)
    assert nz.max() <= n
    # metadata invariants
    for i in range(4):
        k0 = (meta >> (4 * i)) & 3
        k1 = (meta >> (4 * i + 2)) & 3
        assert (k0 < k1).all()
        if nm == "1:2":
            assert (k0 < 2).all() and (k1 >= 2).all()
    assert np.array_equal(_decompress_here(vals, meta), dense)
    assert np.array_equal(oracle.nm_decompress(vals, meta), dense)
    v2, m2, bad = oracle.nm_compress(dense, n, m)
    assert bad == 0 and np.array_equal(v2, vals) and np.array_equal(m2, meta)


def test_compress_hand_built_blocks(oracle):
    d = np.zeros((16, 3), dtype=np.float32)
    d[0:4, 0] = [5, 0, 0, 0]        # 2:4 -> keep (0,1); 1:2 -> keep 0 and 2
    d[4:8, 0] = [0, 0, 0, -2]       # 2:4 -> (0,3); 1:2 -> (0,3)
    d[8:12, 0] = [0, 7, 8, 0]       # both -> (1,2)
    d[12:16, 0] = [0, 0, 0, 0]      # 2:4 -> (0,1); 1:2 -> (0,2)
    d[0:4, 1] = [1, 2, 3, 0]        # too many non-zeros for either pattern
    d[0:4, 2] = [1, 2, 0, 0]        # valid 2:4, invalid 1:2
    v, m, bad = oracle.nm_compress(d, 2, 4)
    assert bad == 1
    assert [(int(m[0, 0]) >> (4 * i)) & 0xF for i in range(4)] == [0 | 1 << 2, 0 | 3 << 2, 1 | 2 << 2, 0 | 1 << 2]
    assert list(v[0, 0]) == [5, 0, 0, -2, 7, 8, 0, 0]
    assert (int(m[0, 2]) & 0xF) == (0 | 1 << 2) and list(v[0, 2, :2]) == [1, 2]
    v, m, bad = oracle.nm_compress(d, 1, 2)
    assert bad == 2
    assert [(int(m[0, 0]) >> (4 * i)) & 0xF for i in range(4)] == [0 | 2 << 2, 0 | 3 << 2, 1 | 2 << 2, 0 | 2 << 2]
    assert list(v[0, 0]) == [5, 0, 0, -2, 7, 8, 0, 0]
    with pytest.raises(ValueError):
        oracle.nm_compress(d[:12], 2, 4)
    with pytest.raises(ValueError):
        oracle.nm_compress(d, 2, 3)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("nm", ["1:2", "2:4"])
def test_update_gemm_equals_library_matmul(oracle, dtype, nm):
    g, h = _case(dtype, nm, T=96, O=40, I=28)
    prune = oracle.prune_1of2 if nm == "1:2" else oracle.prune_2of4
    vals, meta, _ = prune(g, 5, 0)
    dW, absdW = oracle.update_gemm(vals, meta, h)
    gt = _as_f64(_decompress_here(vals, meta))
    hh = _as_f64(h)
    want = gt.T @ hh
    wabs = np.abs(gt).T @ np.abs(hh)
    assert np.allclose(dW, want, rtol=0, atol=1e-12 * wabs.max())
    assert np.allclose(absdW, wabs, rtol=1e-12)
    # orientation: rows of dW index columns of g
    o, i = 7, 3
    assert np.isclose(dW[o, i], sum(gt[t, o] * hh[t, i] for t in range(gt.shape[0])), atol=1e-12 * wabs[o, i])
    # entries form
    oi = np.array([[0, 0], [o, i], [39, 27], [12, 5]])
    e, ea = oracle.update_gemm_entries(vals, meta, h, oi)
    assert np.allclose(e, want[oi[:, 0], oi[:, 1]], atol=1e-12 * wabs.max())
    assert np.allclose(ea, wabs[oi[:, 0], oi[:, 1]], rtol=1e-12)


def test_update_gemm_beta_and_zero_operand(oracle):
    g, h = _case("f32", "2:4", T=32, O=16, I=8)
    vals, meta, _ = oracle.prune_2of4(g, 1, 0)
    prior = np.random.default_rng(0).standard_normal((16, 8)).astype(np.float32)
    d0, _ = oracle.update_gemm(vals, meta, h)
    d1, _ = oracle.update_gemm(vals, meta, h, beta=1.0, dW_in=prior)
    assert np.allclose(d1, d0 + prior.astype(np.float64), atol=1e-12 * np.abs(d0).max())
    z, _ = oracle.update_gemm(np.zeros_like(vals), meta, h)
    assert not z.any()


def test_weight_gradient_is_unbiased(oracle):
    """E_seed[theta(g)^T h] = g^T h: an unbiased neural gradient gives an unbiased weight
    gradient (Sec. 3).  Variance from the 1:2 element variances |a1||a2| and the perfect
    anti-correlation inside a pair."""
    w = synth.Workload("t", 64, 16, 8, "f32", "1:2", 0.0, 1.0, 0.2)
    g, h = synth.make_g(w, 1), synth.make_h(w, 1)
    g64, h64 = g.astype(np.float64), h.astype(np.float64)
    want = g64.T @ h64
    a0, a1 = np.abs(g64[0::2]), np.abs(g64[1::2])                         # [pairs, O]
    s0, s1 = np.sign(g64[0::2]), np.sign(g64[1::2])
    # theta_pair . (h_t, h_t') has variance a0 a1 (s0 h_t - s1 h_t')^2
    var = np.einsum("po,poi->oi", a0 * a1, (s0[:, :, None] * h64[0::2][:, None, :] - s1[:, :, None] * h64[1::2][:, None, :]) ** 2)
    n = 3000
    acc = np.zeros_like(want)
    for seed in range(n):
        vals, meta, _ = oracle.prune_1of2(g, seed, 0)
        acc += oracle.update_gemm(vals, meta, h)[0]
    z = (acc / n - want) / np.sqrt(var / n)
    assert np.abs(z).max() < 4.5
    assert abs((z ** 2).sum() - z.size) < 6 * np.sqrt(2 * z.size)


def test_synthetic_inputs_have_the_stated_statistics():
    w = synth.scaled(synth.WORKLOADS["c3_conv_2of4"], T=4096, name="c3s")
    g, h = synth.make_g(w, 0), synth.make_h(w, 0)
    gf, hf = synth.bf16_to_f32(g), synth.bf16_to_f32(h)
    assert abs((gf == 0).mean() - 0.5) < 0.01 and abs((hf == 0).mean() - 0.5) < 0.01
    assert (hf >= 0).all()
    nzg = gf[gf != 0]
    assert abs((nzg > 0).mean() - 0.5) < 0.01
    assert abs(np.log(np.abs(nzg)).std() - 3.0) < 0.05 and abs(np.log(np.abs(nzg)).mean()) < 0.05
    # chunked generation: a row range equals the same rows of the full tensor
    part = synth.make_g(w, 0, rows=(1024, 2048))
    assert np.array_equal(part, g[1024:2048])
    # bf16 helper against the library cast
    import torch
    x = np.random.default_rng(1).standard_normal(10000).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(synth.f32_to_bf16_bits(x), want)

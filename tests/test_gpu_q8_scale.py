"""GPU parity of the 8-bit path's device-side scales and activation cast (nm_q8_scale, nm_cast_e4m3 and the _ds entry
points) against the CPU oracle, through the C ABI: scale records bit for bit, e4m3 codes bit for bit over EVERY bf16
input, and the device-scale prune / GEMM against their host-scale forms."""
import numpy as np
import pytest
import torch

from paper_2203_10991_amd import synth
from gpu_util import DEV, to_dev, to_host

pytestmark = pytest.mark.gpu


def _rec(nm, t, top):
    rec = nm.nm_q8_scale(t, top)
    torch.cuda.synchronize()
    return rec, rec.cpu().numpy()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_scale_record_matches_the_oracle(oracle, dtype):
    import paper_2203_10991_amd as nm
    rng = np.random.default_rng(0)
    cases = []
    for k in range(12):
        R, C = int(rng.integers(1, 70)), 8 * int(rng.integers(1, 40))
        t = (rng.standard_normal((R, C)) * np.exp2(rng.uniform(-30, 30))).astype(np.float32)
        cases.append(t)
    cases.append(np.zeros((5, 16), dtype=np.float32))
    t = np.ones((3, 8), dtype=np.float32); t[2, 7] = -7.0; cases.append(t)                 # exact boundary: 7 * 64 = 448
    t = np.ones((3, 8), dtype=np.float32); t[1, 1] = np.inf; cases.append(t)
    t = np.ones((3, 8), dtype=np.float32); t[0, 5] = np.nan; cases.append(t)
    cases.append(np.full((2, 8), 1e-44, dtype=np.float32))
    cases.append(np.full((2, 8), 3e38, dtype=np.float32))
    big = (rng.standard_normal((4096, 1024)) * 3).astype(np.float32); big[3071, 77] = 1234.5; cases.append(big)
    for t in cases:
        h = t if dtype == "f32" else synth.f32_to_bf16_bits(t)
        for top in (448.0, 57344.0 / 4.0, 2.0 ** -20):
            _, rec = _rec(nm, to_dev(h), top)
            want = np.float32(oracle.pow2_scale(h, top))
            assert rec[0] == want and rec[1] == np.float32(1.0) / want, (t.shape, top, rec, want)
            hb = (h.view(np.uint32) if dtype == "f32" else h.astype(np.uint32) << 16) & 0x7FFFFFFF
            assert rec.view(np.uint32)[2] == hb.max() and rec[3] == 0
    # a padded row stride: the padding is not looked at
    wide = np.full((6, 24), 1e9, dtype=np.float32); wide[:, :16] = 1.5
    d = to_dev(wide)
    _, rec = _rec(nm, d[:, :16], 448.0)
    assert rec[0] == 256.0


def test_e4m3_cast_of_every_bf16_value(oracle):
    import paper_2203_10991_amd as nm
    allbits = np.arange(65536, dtype=np.uint16).reshape(4096, 16)
    finite = (allbits & 0x7F80) != 0x7F80
    nan = ((allbits & 0x7F80) == 0x7F80) & ((allbits & 0x7F) != 0)
    for s in (1.0, 0.25, 64.0, 2.0 ** -100, 2.0 ** 100):
        rec = torch.tensor([s, 1.0 / s, 0.0, 0.0], dtype=torch.float32, device=DEV)
        h8 = nm.nm_cast_e4m3(to_dev(allbits), rec)
        torch.cuda.synchronize()
        got, want = h8.cpu().numpy(), oracle.cast_e4m3(allbits, s)
        # zeros: the sign of a zero result is the input's on both sides
        assert np.array_equal(got[~nan], want[~nan]), (s, np.argwhere(got[~nan] != want[~nan])[:5])
        assert finite.sum() > 65000


def test_e4m3_cast_of_binary32_values_and_strides(oracle):
    import paper_2203_10991_amd as nm
    rng = np.random.default_rng(1)
    x = (rng.standard_normal((37, 48)) * np.exp2(rng.uniform(-12, 10, (37, 48)))).astype(np.float32)
    grid = np.array(sorted(oracle.e4m3_value(c) for c in range(0x7F)), dtype=np.float64)
    mids = ((grid[:-1] + grid[1:]) / 2).astype(np.float32)                              # ties
    x[0, :48] = np.resize(mids, 48); x[1, :48] = -np.resize(mids[40:], 48)
    rec, r = _rec(nm, to_dev(x), 448.0)
    out = torch.full((37, 64), 0xAA, dtype=torch.uint8, device=DEV)
    nm.nm_cast_e4m3(to_dev(x), rec, h8=out[:, :48])
    torch.cuda.synchronize()
    assert np.array_equal(out[:, :48].cpu().numpy(), oracle.cast_e4m3(x, float(r[0])))
    assert bool((out[:, 48:] == 0xAA).all())
    one = torch.tensor([1.0, 1.0, 0.0, 0.0], dtype=torch.float32, device=DEV)
    got = nm.nm_cast_e4m3(to_dev(x), one).cpu().numpy()
    assert np.array_equal(got, oracle.cast_e4m3(x, 1.0))                                # includes saturation beyond 448


@pytest.mark.parametrize("nmode", ["2:4", "1:2"])
def test_device_scale_entry_points_equal_the_host_scale_ones(oracle, nmode):
    import paper_2203_10991_amd as nm
    w = synth.Workload("ds", 32 * 20, 8 * 23, 16 * 9, "bf16", nmode, 0.0, 2.0, 0.3)
    g, h = synth.make_g(w, 3), synth.make_h(w, 3)
    gd, hd = to_dev(g), to_dev(h)
    top_g = 57344.0 / (4.0 if nmode == "2:4" else 2.0)
    rg, rgh = _rec(nm, gd, top_g)
    rh, rhh = _rec(nm, hd, 448.0)
    sg, sh = float(rgh[0]), float(rhh[0])
    assert sg == oracle.pow2_scale(g, top_g) and sh == oracle.pow2_scale(h, 448.0)
    h8 = nm.nm_cast_e4m3(hd, rh)
    prune = nm.mvue_prune_2of4_q8 if nmode == "2:4" else nm.mvue_prune_1of2_q8
    v_ds, m_ds = prune(gd, seed=4, stream_id=1, scale=rg)
    v_h, m_h = prune(gd, seed=4, stream_id=1, scale=sg)
    dW_ds = nm.nm_update_gemm_q8(v_ds, m_ds, h8, alpha=(rg, rh))
    dW_h = nm.nm_update_gemm_q8(v_h, m_h, h8, alpha=1.0 / (sg * sh))
    torch.cuda.synchronize()
    assert torch.equal(v_ds, v_h) and torch.equal(m_ds, m_h) and torch.equal(dW_ds, dW_h)
    # and the whole chain against the oracle's
    ov, om = (oracle.prune_2of4_q8(g, 4, 1, 0, sg) if nmode == "2:4" else oracle.prune_1of2_q8(g, 4, 1, sg))
    assert np.array_equal(v_ds.cpu().numpy(), ov) and np.array_equal(m_ds.cpu().numpy().view(np.uint32), om)
    o8 = oracle.cast_e4m3(h, sh)
    assert np.array_equal(h8.cpu().numpy(), o8)
    want, wabs = oracle.update_gemm_q8(ov, om, o8, alpha=1.0 / (sg * sh))
    rel = float((np.abs(dW_ds.cpu().numpy().astype(np.float64) - want) / np.maximum(wabs, 1e-300)).max())
    assert rel <= 1e-3
    # split-K shape (few tiles, long reduction): the scale is applied in the second pass
    w2 = synth.Workload("ds2", 32 * 96, 64, 64, "bf16", "2:4", 0.0, 2.0, 0.3)
    g2, h2 = to_dev(synth.make_g(w2, 1)), to_dev(synth.make_h(w2, 1))
    r2g, r2h = nm.nm_q8_scale(g2, 57344.0 / 4.0), nm.nm_q8_scale(h2, 448.0)
    h82 = nm.nm_cast_e4m3(h2, r2h)
    assert nm.nm_update_gemm_q8_workspace(w2.T, w2.O, w2.I) > 0
    v2, m2 = nm.mvue_prune_2of4_q8(g2, seed=0, stream_id=0, scale=r2g)
    a = nm.nm_update_gemm_q8(v2, m2, h82, alpha=(r2g, r2h))
    torch.cuda.synchronize()
    b = nm.nm_update_gemm_q8(v2, m2, h82, alpha=float(r2g.cpu()[1]) * float(r2h.cpu()[1]))
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_scale_and_cast_argument_errors():
    import paper_2203_10991_amd as nm
    t = torch.zeros((4, 12), dtype=torch.float32, device=DEV)
    with pytest.raises(nm.NmError) as ei:
        nm.nm_q8_scale(t, 448.0)
    assert ei.value.status == 2
    t = torch.zeros((4, 16), dtype=torch.float32, device=DEV)
    with pytest.raises(nm.NmError) as ei:
        nm.nm_q8_scale(t, -1.0)
    assert ei.value.status == 2
    rec = nm.nm_q8_scale(t, 1.0)
    with pytest.raises(nm.NmError) as ei:
        nm.nm_cast_e4m3(torch.zeros((4, 24), dtype=torch.float32, device=DEV), rec)
    assert ei.value.status == 2
    empty = nm.nm_cast_e4m3(torch.zeros((0, 16), dtype=torch.bfloat16, device=DEV), rec)
    assert empty.numel() == 0

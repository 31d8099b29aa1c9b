"""GPU parity of mvue_prune_2of4_t and mvue_prune_1of2_t (gradient stored transposed, tokens contiguous) through the C ABI:
vals and meta equal the CPU oracle's prune of the transposed tensor bit for bit, and so equal what
mvue_prune_2of4 writes for it; the compressed operand then feeds the same update GEMM.  The same for the 8-bit
prunes (mvue_prune_2of4_q8_t, mvue_prune_1of2_q8_t) against the oracle's 8-bit prune of the transposed tensor."""
import numpy as np
import pytest
import torch

from paper_2203_10991_amd import synth
from gpu_util import DEV, first_mismatch, to_dev, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nm():
    import paper_2203_10991_amd as p
    p.load()
    return p


def _bits(a):
    return a.view(np.uint32) if a.dtype == np.float32 else a


SHAPES = [(16, 8), (16 * 37, 8 * 29), (16 * 5, 8 * 64 + 8), (16 * 17, 16), (16 * 64, 1024), (16 * 130, 8 * 3)]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("shape", SHAPES)
def test_transposed_prune_bit_exact(nm, oracle, dtype, mode, shape):
    T, O = shape
    print(f"case dtype={dtype} mode={mode} T={T} O={O}", flush=True)
    w = synth.Workload("t", T, O, 8, dtype, "2:4", 0.0, 2.5, 0.3)
    g = synth.make_g(w, seed=T + O + 1)                      # [T x O]
    gT = to_dev(np.ascontiguousarray(g.T))                    # [O x T], tokens contiguous
    seed, stream = 0x51 + (3 << 40), 5
    cpu = oracle.prune_2of4_approx if mode else oracle.prune_2of4
    ov, om, _ = cpu(g, seed, stream, want_dense=False)
    v, m = nm.mvue_prune_2of4_t(gT, seed=seed, stream_id=stream, mode=mode)
    torch.cuda.synchronize()
    hv, hm = to_host(v), to_host(m)
    assert first_mismatch(hm, om) is None, ("meta", first_mismatch(hm, om))
    assert first_mismatch(_bits(hv), _bits(ov)) is None, ("vals", first_mismatch(_bits(hv), _bits(ov)))
    # and the token-major entry point on the same tensor
    v2, m2, _ = nm.mvue_prune_2of4(to_dev(g), seed=seed, stream_id=stream, mode=mode)
    it = torch.int16 if dtype == "bf16" else torch.int32
    assert torch.equal(m2, m) and torch.equal(v2.view(it), v.view(it))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", SHAPES)
def test_transposed_prune_1of2_bit_exact(nm, oracle, dtype, shape):
    T, O = shape
    print(f"case 1:2 dtype={dtype} T={T} O={O}", flush=True)
    w = synth.Workload("t", T, O, 8, dtype, "1:2", 0.0, 2.5, 0.3)
    g = synth.make_g(w, seed=T + O + 2)
    seed, stream = 0x77 + (5 << 40), 2
    ov, om, _ = oracle.prune_1of2(g, seed, stream, want_dense=False)
    v, m = nm.mvue_prune_1of2_t(to_dev(np.ascontiguousarray(g.T)), seed=seed, stream_id=stream)
    torch.cuda.synchronize()
    hv, hm = to_host(v), to_host(m)
    assert first_mismatch(hm, om) is None, ("meta", first_mismatch(hm, om))
    assert first_mismatch(_bits(hv), _bits(ov)) is None, ("vals", first_mismatch(_bits(hv), _bits(ov)))
    v2, m2, _ = nm.mvue_prune_1of2(to_dev(g), seed=seed, stream_id=stream)
    it = torch.int16 if dtype == "bf16" else torch.int32
    assert torch.equal(m2, m) and torch.equal(v2.view(it), v.view(it))


def test_transposed_prune_row_stride_and_edge_values(nm, oracle):
    """row stride larger than T; zeros, ties, infinities and subnormals in the quads"""
    T, O = 16 * 6, 24
    w = synth.Workload("t", T, O, 8, "bf16", "2:4", 0.0, 3.0, 0.5)
    g = synth.make_g(w, seed=2)
    g[0:4, :] = 0                                             # all-zero quads
    g[4:8, :] = g[4:5, :]                                     # four equal magnitudes
    g[8, :] = 0x0001                                          # a subnormal next to ordinary values
    g[12, :] = 0x8000                                         # negative zero
    wide = torch.zeros((O, T + 40), dtype=torch.bfloat16, device=DEV)
    wide[:, :T] = to_dev(np.ascontiguousarray(g.T))
    for mode, cpu in ((0, oracle.prune_2of4), (1, oracle.prune_2of4_approx)):
        ov, om, _ = cpu(g, 9, 1, want_dense=False)
        v, m = nm.mvue_prune_2of4_t(wide[:, :T], seed=9, stream_id=1, mode=mode)
        torch.cuda.synchronize()
        assert first_mismatch(to_host(m), om) is None
        assert first_mismatch(to_host(v), ov) is None
    ov, om, _ = oracle.prune_1of2(g, 9, 1, want_dense=False)
    v, m = nm.mvue_prune_1of2_t(wide[:, :T], seed=9, stream_id=1)
    torch.cuda.synchronize()
    assert first_mismatch(to_host(m), om) is None
    assert first_mismatch(to_host(v), ov) is None


def test_transposed_prune_feeds_the_update_gemm(nm, oracle):
    T, O, I = 16 * 24, 136, 96
    w = synth.Workload("t", T, O, I, "bf16", "2:4", 0.0, 2.0, 0.3)
    g, h = synth.make_g(w, seed=3), synth.make_h(w, seed=4)
    v, m = nm.mvue_prune_2of4_t(to_dev(np.ascontiguousarray(g.T)), seed=1, stream_id=0)
    dW = nm.nm_update_gemm(v, m, to_dev(h))
    torch.cuda.synchronize()
    ov, om, _ = oracle.prune_2of4(g, 1, 0, want_dense=False)
    want, wabs = oracle.update_gemm(ov, om, h)
    got = dW.cpu().numpy().astype(np.float64)
    assert float((np.abs(got - want) / np.maximum(wabs, 1e-300)).max()) <= 1e-2


def test_transposed_prune_empty_and_errors(nm):
    e = torch.zeros((8, 0), dtype=torch.bfloat16, device=DEV)
    v, m = nm.mvue_prune_2of4_t(e)
    assert v.numel() == 0 and m.numel() == 0
    with pytest.raises(nm.NmError):
        nm.mvue_prune_2of4_t(torch.zeros((8, 24), dtype=torch.bfloat16, device=DEV))     # T not a multiple of 16
    with pytest.raises(nm.NmError):
        nm.mvue_prune_2of4_t(torch.zeros((12, 32), dtype=torch.bfloat16, device=DEV))    # O not a multiple of 8
    with pytest.raises(nm.NmError):
        nm.mvue_prune_2of4_t(torch.zeros((8, 32), dtype=torch.bfloat16, device=DEV), mode=2)


Q8_SHAPES = [(32, 8), (32 * 19, 8 * 29), (32 * 3, 8 * 64 + 8), (32 * 17, 16), (32 * 33, 1024), (32 * 70, 8 * 3)]


def _fit_scale(g):
    f = g if g.dtype == np.float32 else synth.bf16_to_f32(g)
    return float(2.0 ** np.floor(np.log2(57344.0 / (4.0 * max(float(np.abs(f).max()), 1e-30)))))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("shape", Q8_SHAPES)
def test_transposed_q8_prune_bit_exact(nm, oracle, dtype, mode, shape):
    T, O = shape
    print(f"case q8 dtype={dtype} mode={mode} T={T} O={O}", flush=True)
    w = synth.Workload("t", T, O, 16, dtype, "2:4", 0.0, 2.5, 0.3)
    g = synth.make_g(w, seed=T + O + 3)
    scale = _fit_scale(g)
    seed, stream = 0x91 + (7 << 40), 6
    ov, om = oracle.prune_2of4_q8(g, seed=seed, stream_id=stream, mode=mode, scale=scale)
    v, m = nm.mvue_prune_2of4_q8_t(to_dev(np.ascontiguousarray(g.T)), seed=seed, stream_id=stream, mode=mode, scale=scale)
    torch.cuda.synchronize()
    hv, hm = v.cpu().numpy(), m.cpu().numpy().view(np.uint32)
    assert first_mismatch(hm, om) is None, ("meta32", first_mismatch(hm, om))
    assert first_mismatch(hv, ov) is None, ("vals8", first_mismatch(hv, ov))
    # the token-major entry point on the same tensor, and the scale as a device record
    v2, m2 = nm.mvue_prune_2of4_q8(to_dev(g), seed=seed, stream_id=stream, mode=mode, scale=scale)
    assert torch.equal(m2, m) and torch.equal(v2, v)
    rec = torch.tensor([scale, 1.0 / scale, 0.0, 0.0], dtype=torch.float32, device=DEV)
    v3, m3 = nm.mvue_prune_2of4_q8_t(to_dev(np.ascontiguousarray(g.T)), seed=seed, stream_id=stream, mode=mode, scale=rec)
    assert torch.equal(m3, m) and torch.equal(v3, v)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", Q8_SHAPES)
def test_transposed_q8_prune_1of2_bit_exact(nm, oracle, dtype, shape):
    T, O = shape
    print(f"case q8 1:2 dtype={dtype} T={T} O={O}", flush=True)
    w = synth.Workload("t", T, O, 16, dtype, "1:2", 0.0, 2.5, 0.3)
    g = synth.make_g(w, seed=T + O + 4)
    scale = 2.0 * _fit_scale(g)
    seed, stream = 0x93 + (9 << 40), 1
    ov, om = oracle.prune_1of2_q8(g, seed=seed, stream_id=stream, scale=scale)
    v, m = nm.mvue_prune_1of2_q8_t(to_dev(np.ascontiguousarray(g.T)), seed=seed, stream_id=stream, scale=scale)
    torch.cuda.synchronize()
    hv, hm = v.cpu().numpy(), m.cpu().numpy().view(np.uint32)
    assert first_mismatch(hm, om) is None, ("meta32", first_mismatch(hm, om))
    assert first_mismatch(hv, ov) is None, ("vals8", first_mismatch(hv, ov))
    v2, m2 = nm.mvue_prune_1of2_q8(to_dev(g), seed=seed, stream_id=stream, scale=scale)
    assert torch.equal(m2, m) and torch.equal(v2, v)


def test_transposed_q8_prune_row_stride(nm, oracle):
    """row stride larger than T; saturating scale"""
    T, O = 32 * 5, 24
    w = synth.Workload("t", T, O, 16, "bf16", "2:4", 0.0, 3.0, 0.5)
    g = synth.make_g(w, seed=9)
    wide = torch.zeros((O, T + 40), dtype=torch.bfloat16, device=DEV)
    wide[:, :T] = to_dev(np.ascontiguousarray(g.T))
    for scale in (_fit_scale(g), 64.0 * _fit_scale(g)):
        ov, om = oracle.prune_2of4_q8(g, seed=4, stream_id=2, mode=0, scale=scale)
        v, m = nm.mvue_prune_2of4_q8_t(wide[:, :T], seed=4, stream_id=2, scale=scale)
        torch.cuda.synchronize()
        assert np.array_equal(m.cpu().numpy().view(np.uint32), om) and np.array_equal(v.cpu().numpy(), ov)

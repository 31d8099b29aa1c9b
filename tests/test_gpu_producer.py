"""GPU parity of the prune fused into the producer of the neural gradient (mvue_prune_*_producer: g_l = u * d of
eq. (2) written dense and pruned in one pass) against the CPU oracle, bit for bit, through the C ABI: the dense g_l
against the oracle's producer step, vals / meta against the oracle's prune of that g_l, and the fused call against the
unfused pair of calls on the device."""
import numpy as np
import pytest
import torch

from paper_2203_10991_amd import synth
from gpu_util import DEV, first_mismatch, to_dev, to_host

pytestmark = pytest.mark.gpu


def _bits(a):
    return a.view(np.uint32) if a.dtype == np.float32 else a


def _derivative(rng, shape, dtype):
    """activation derivatives: ReLU masks mixed with GELU-like slopes"""
    d = np.where(rng.random(shape) < 0.5, (rng.random(shape) < 0.6).astype(np.float32),
                 rng.uniform(-0.2, 1.13, shape).astype(np.float32)).astype(np.float32)
    return d if dtype == "f32" else synth.f32_to_bf16_bits(d)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("nmode,mode", [("2:4", 0), ("2:4", 1), ("1:2", 0)])
@pytest.mark.parametrize("shape", [(16, 8), (16 * 23, 8 * 31), (16 * 40, 1024)])
def test_fused_producer_prune_bit_exact(oracle, dtype, nmode, mode, shape):
    import paper_2203_10991_amd as nm
    T, O = shape
    print(f"producer case dtype={dtype} nm={nmode} mode={mode} T={T} O={O}", flush=True)
    rng = np.random.default_rng(T + O)
    u = synth.make_g(synth.Workload("u", T, O, 8, dtype, nmode, 0.0, 2.5, 0.1), seed=T)
    d = _derivative(rng, (T, O), dtype)
    seed, stream = 77 + (1 << 35), 4
    # padded row strides on every tensor
    ud = torch.zeros((T, O + 8), dtype=to_dev(u).dtype, device=DEV); ud[:, :O] = to_dev(u)
    dd = torch.zeros((T, O + 16), dtype=ud.dtype, device=DEV); dd[:, :O] = to_dev(d)
    gbuf = torch.full((T, O + 24), 5.0, dtype=ud.dtype, device=DEV)
    g_out, v, m = nm.mvue_prune_producer(ud[:, :O], dd[:, :O], nm=nmode, seed=seed, stream_id=stream, mode=mode, g_out=gbuf[:, :O])
    torch.cuda.synchronize()
    og = oracle.act_backward(u, d)
    hg = to_host(g_out)
    assert first_mismatch(_bits(hg), _bits(og)) is None, ("g_out", first_mismatch(_bits(hg), _bits(og)))
    assert bool((gbuf[:, O:] == 5.0).all())
    oprune = oracle.prune_1of2 if nmode == "1:2" else (oracle.prune_2of4_approx if mode else oracle.prune_2of4)
    ov, om, _ = oprune(og, seed, stream)
    assert first_mismatch(to_host(m), om) is None and first_mismatch(_bits(to_host(v)), _bits(ov)) is None
    # the unfused pair of calls on the device gives the same compressed operand
    if nmode == "1:2":
        v2, m2, _ = nm.mvue_prune_1of2(g_out.contiguous(), seed=seed, stream_id=stream)
    else:
        v2, m2, _ = nm.mvue_prune_2of4(g_out.contiguous(), seed=seed, stream_id=stream, mode=mode)
    torch.cuda.synchronize()
    assert torch.equal(m2, m) and np.array_equal(_bits(to_host(v2)), _bits(to_host(v)))


def test_fused_producer_in_a_layer_backward(oracle):
    """eq. (2) on a small MLP layer: u from torch's dense backward GEMM, d = ReLU'(z); the fused call's g_l equals
    torch's own activation backward, and the update GEMM on its compressed output estimates the dense dW"""
    import paper_2203_10991_amd as nm
    torch.manual_seed(0)
    T, I, Hd, O = 256, 64, 128, 32
    x = torch.randn(T, I, device=DEV).bfloat16()
    W1 = (torch.randn(Hd, I, device=DEV) / 8).bfloat16()
    W2 = (torch.randn(O, Hd, device=DEV) / 8).bfloat16()
    z = x @ W1.t()
    g_next = (torch.randn(T, O, device=DEV) * torch.exp(torch.randn(T, O, device=DEV))).bfloat16()
    u = g_next @ W2                                   # W^T g_{l+1}
    d = (z > 0).to(torch.bfloat16)                    # ReLU'
    g_l, v, m = nm.mvue_prune_producer(u, d, nm="2:4", seed=3, stream_id=0)
    assert torch.equal(g_l, u * d)
    dW = nm.nm_update_gemm(v, m, x)
    torch.cuda.synchronize()
    ov, om, _ = oracle.prune_2of4(to_host(g_l), 3, 0)
    want, wabs = oracle.update_gemm(ov, om, to_host(x))
    rel = float((np.abs(dW.cpu().numpy().astype(np.float64) - want) / np.maximum(wabs, 1e-300)).max())
    assert rel <= 1e-2


def test_fused_producer_argument_errors():
    import paper_2203_10991_amd as nm
    u = torch.zeros((16, 8), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(nm.NmError) as ei:
        nm.mvue_prune_producer(u, u.clone(), g_out=u)
    assert ei.value.status == 5
    with pytest.raises(nm.NmError) as ei:
        nm.mvue_prune_producer(torch.zeros((24, 8), dtype=torch.bfloat16, device=DEV), torch.zeros((24, 8), dtype=torch.bfloat16, device=DEV),
                               vals=torch.zeros((1, 8, 8), dtype=torch.bfloat16, device=DEV), meta=torch.zeros((1, 8), dtype=torch.int16, device=DEV))
    assert ei.value.status == 2

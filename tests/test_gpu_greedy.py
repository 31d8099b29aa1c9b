"""GPU parity of nm_prune_greedy (the paper's biased baseline: keep the n largest of every block, unchanged) against
the CPU oracle, bit for bit, through the C ABI; and the check the paper's ablation is about: the same z-test that
MVUE 1:2 passes on the device, the greedy method fails."""
import numpy as np
import pytest
import torch

from paper_2203_10991_amd import synth
from gpu_util import DEV, first_mismatch, to_dev, to_host

pytestmark = pytest.mark.gpu


def _bits(a):
    return a.view(np.uint32) if a.dtype == np.float32 else a


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n,m", [(1, 2), (2, 4)])
@pytest.mark.parametrize("shape", [(16, 8), (16 * 37, 8 * 29), (16 * 64, 1024)])
def test_greedy_prune_bit_exact(oracle, dtype, n, m, shape):
    import paper_2203_10991_amd as nm
    T, O = shape
    print(f"greedy case dtype={dtype} {n}:{m} T={T} O={O}", flush=True)
    w = synth.Workload("t", T, O, 8, dtype, "2:4", 0.0, 2.5, 0.3)
    g = synth.make_g(w, seed=T + O)
    # ties and signed zeros in the first group
    g[:16, :8] = np.array([3, -3, 3, 0, -0.0, 0, 1, -1, 2, 2, -2, 2, 0, 0, 0, 5], dtype=np.float32)[:, None] if dtype == "f32" else \
        synth.f32_to_bf16_bits(np.array([3, -3, 3, 0, -0.0, 0, 1, -1, 2, 2, -2, 2, 0, 0, 0, 5], dtype=np.float32))[:, None]
    v, mt, d = nm.nm_prune_greedy(to_dev(g), n, m, want_dense=True)
    torch.cuda.synchronize()
    ov, om, od = oracle.prune_greedy(g, n, m, want_dense=True)
    hv, hm, hd = to_host(v), to_host(mt), to_host(d)
    assert first_mismatch(hm, om) is None, ("meta", first_mismatch(hm, om))
    assert first_mismatch(_bits(hv), _bits(ov)) is None, ("vals", first_mismatch(_bits(hv), _bits(ov)))
    assert first_mismatch(_bits(hd), _bits(od)) is None, ("dense", first_mismatch(_bits(hd), _bits(od)))
    # without the dense output (another kernel instance): same compressed tensors
    v2, m2, _ = nm.nm_prune_greedy(to_dev(g), n, m)
    torch.cuda.synchronize()
    assert torch.equal(v2.view(torch.int16 if dtype == "bf16" else torch.int32), v.view(torch.int16 if dtype == "bf16" else torch.int32))
    assert torch.equal(m2, mt)


def test_greedy_fails_the_unbiasedness_test_mvue_passes():
    import paper_2203_10991_amd as nm
    w = synth.scaled(synth.WORKLOADS["c1_fp32_1of2"], T=16, O=256)
    g = synth.make_g(w, seed=0)
    gd = to_dev(g)
    n = 2000
    acc = torch.zeros((16, 256), dtype=torch.float64, device=DEV)
    for seed in range(n):
        acc += nm.mvue_prune_1of2(gd, seed=seed, stream_id=0, want_dense=True)[2].double()
    a = np.abs(g.astype(np.float64)).reshape(8, 2, 256)
    var = np.repeat(a[:, 0] * a[:, 1], 2, axis=0).reshape(16, 256)              # element variance |a1||a2| (Sec. 4.1)
    live = var > 0
    z_mvue = ((acc / n).cpu().numpy() - g)[live] / np.sqrt(var[live] / n)
    assert np.abs(z_mvue).max() < 4.8
    # greedy: every "sample" is the same tensor, so the mean over any number of samples is that tensor
    dense = nm.nm_prune_greedy(gd, 1, 2, want_dense=True)[2]
    again = nm.nm_prune_greedy(gd, 1, 2, want_dense=True)[2]
    torch.cuda.synchronize()
    assert torch.equal(dense, again)
    z_greedy = (dense.cpu().numpy().astype(np.float64) - g)[live] / np.sqrt(var[live] / n)
    assert np.abs(z_greedy).max() > 20.0                                         # the dropped element is lost for good
    assert (np.abs(z_greedy) > 4.8).mean() > 0.4                                 # about half of the live elements


def test_greedy_argument_errors():
    import paper_2203_10991_amd as nm
    g = torch.zeros((16, 8), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(nm.NmError) as ei:
        nm.nm_prune_greedy(g, 2, 8)
    assert ei.value.status == 7
    with pytest.raises(nm.NmError) as ei:
        nm.nm_prune_greedy(torch.zeros((24, 8), dtype=torch.bfloat16, device=DEV), 2, 4,
                           vals=torch.zeros((1, 8, 8), dtype=torch.bfloat16, device=DEV),
                           meta=torch.zeros((1, 8), dtype=torch.int16, device=DEV))
    assert ei.value.status == 2

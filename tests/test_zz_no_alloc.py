"""nm_update_gemm_static (the entry point for callers that cannot allocate: split-K partial sums in the library's
static device array) against nm_update_gemm, through the C ABI.  Two calls in a row, the second on a smaller
problem, so that the second runs over what the first left in the array; both entry points run the same kernels on
the same plan, so the results are compared bit for bit (and, once, against the oracle at the update GEMM's
tolerance).  Collected last: the file name sorts after every other test file."""
import numpy as np
import pytest
import torch

from paper_2203_10991_amd import synth
from gpu_util import DEV, to_dev

pytestmark = pytest.mark.gpu


def _case(nm, w, seed):
    g, h = synth.make_g(w, seed), synth.make_h(w, seed)
    gd, hd = to_dev(g), to_dev(h)
    v, m, _ = (nm.mvue_prune_1of2 if w.nm == "1:2" else nm.mvue_prune_2of4)(gd, seed=seed, stream_id=0)
    return g, h, hd, v, m


def test_static_scratch_entry_point_matches_the_workspace_one(oracle):
    import paper_2203_10991_amd as nm
    nm.load()
    limit = nm.nm_update_gemm_static_max()
    assert limit == 64 << 20
    # first call: a split-K problem whose partial sums fill the array to the last byte (the transformer-MLP shape:
    # 64 tiles of 256 x 256, four slabs); second: a smaller one on the other tile shape
    shapes = [synth.scaled(synth.WORKLOADS["c2_mlp_1of2"], name="static_first"),
              synth.Workload("static_second", 16 * 150, 8 * 41, 8 * 35, "bf16", "2:4", 0.0, 2.0, 0.3)]
    for k, w in enumerate(shapes):
        need = nm.nm_update_gemm_workspace(w.T, w.O, w.I, torch.bfloat16)
        print(f"static scratch case {w.name}: T={w.T} O={w.O} I={w.I}, split-K scratch {need} bytes", flush=True)
        assert 0 < need <= limit
        g, h, hd, v, m = _case(nm, w, seed=k)
        ref = nm.nm_update_gemm(v, m, hd)
        out = torch.full((w.O, w.I), float("nan"), dtype=torch.float32, device=DEV)
        nm.nm_update_gemm_static(v, m, hd, out)
        torch.cuda.synchronize()
        assert torch.equal(out, ref)
        # beta = 1 accumulates onto what is there
        nm.nm_update_gemm_static(v, m, hd, out, beta=1.0)
        ref2 = nm.nm_update_gemm(v, m, hd, dW=ref.clone(), beta=1.0)
        torch.cuda.synchronize()
        assert torch.equal(out, ref2)
        if k == 1:
            ov, om, _ = oracle.prune_2of4(g, k, 0)
            want, wabs = oracle.update_gemm(ov, om, h)
            rel = float((np.abs(ref.cpu().numpy().astype(np.float64) - want) / np.maximum(wabs, 1e-300)).max())
            assert rel <= 1e-2


def test_static_scratch_entry_point_binary32_and_no_workspace_problems():
    import paper_2203_10991_amd as nm
    nm.load()
    # binary32 split-K (dense fp32 MFMA path)
    w = synth.Workload("static_f32", 16 * 96, 8 * 30, 8 * 40, "f32", "1:2", 0.0, 2.0, 0.3)
    g, h, hd, v, m = _case(nm, w, seed=5)
    ref = nm.nm_update_gemm(v, m, hd)
    out = torch.full((w.O, w.I), float("nan"), dtype=torch.float32, device=DEV)
    nm.nm_update_gemm_static(v, m, hd, out)
    torch.cuda.synchronize()
    assert torch.equal(out, ref)
    # a problem that runs in one pass needs no scratch: any size is accepted
    w = synth.Workload("static_none", 64, 16 * 256, 16 * 256, "bf16", "2:4", 0.0, 2.0, 0.3)
    assert nm.nm_update_gemm_workspace(w.T, w.O, w.I, torch.bfloat16) == 0
    g, h, hd, v, m = _case(nm, w, seed=6)
    ref = nm.nm_update_gemm(v, m, hd)
    out = torch.full((w.O, w.I), float("nan"), dtype=torch.float32, device=DEV)
    nm.nm_update_gemm_static(v, m, hd, out)
    torch.cuda.synchronize()
    assert torch.equal(out, ref)


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    import paper_2203_10991_amd as nm
    nm.load()
    # a split-K problem whose partial sums exceed the array: rejected on the host, nothing enqueued, dW untouched
    T, O, I = 12608, 1536, 1536
    need = nm.nm_update_gemm_workspace(T, O, I, torch.float32)
    assert need > nm.nm_update_gemm_static_max(), need
    v, m = nm.alloc_compressed(T, O, torch.float32, DEV)
    h = torch.zeros((T, I), dtype=torch.float32, device=DEV)
    dW = torch.full((O, I), 7.0, dtype=torch.float32, device=DEV)
    with pytest.raises(nm.NmError) as ei:
        nm.nm_update_gemm_static(v, m, h, dW)
    assert ei.value.status == 6
    torch.cuda.synchronize()
    assert bool((dW == 7.0).all())

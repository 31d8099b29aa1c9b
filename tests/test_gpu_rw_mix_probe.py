"""nm_rw_mix_probe (the benchmark's yardstick kernel with the prune's 16:9 read:write mix): its output against the
definition in the header, computed with numpy.  Not part of the paper's method: there is no oracle function for it."""
import numpy as np
import pytest
import torch

from gpu_util import DEV

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n_blocks", [1, 3, 517])
def test_rw_mix_probe_matches_its_definition(n_blocks):
    import paper_2203_10991_amd as nm
    nm.load()
    rng = np.random.default_rng(n_blocks)
    src = rng.integers(0, 2**32, size=(n_blocks, 16, 256, 4), dtype=np.uint64).astype(np.uint32)
    want = src[:, 0:9] ^ src[:, 7:16]
    s = torch.from_numpy(src.view(np.int32)).to(DEV)
    d = torch.full((n_blocks + 1, 9, 256, 4), -1, dtype=torch.int32, device=DEV)       # one block more: must stay untouched
    nm.nm_rw_mix_probe(s, d, n_blocks)
    torch.cuda.synchronize()
    got = d.cpu().numpy().view(np.uint32)
    assert np.array_equal(got[:n_blocks], want)
    assert (got[n_blocks] == 0xFFFFFFFF).all()

"""Update GEMM on a compressed operand larger than 4 GiB (byte offsets beyond 32 bits), in the large-tile launch
configuration of the benchmark.  The operand is synthetic compressed data made on the device (random kept values,
random valid index words); the activations are zero except in three token windows -- the first groups, the groups
that straddle the 4 GiB mark of `vals`, and the last groups (an odd count, so the last stage is ragged) -- so the
CPU oracle only has to multiply those windows, and every entry of dW is compared."""
import numpy as np
import pytest
import torch

from gpu_util import DEV, to_host

pytestmark = pytest.mark.gpu

NIBBLES = [0x4, 0x8, 0xC, 0x9, 0xD, 0xE]          # p0 | p1 << 2 for the six pairs p0 < p1


def test_update_gemm_operand_beyond_4_gib(oracle):
    import paper_2203_10991_amd as nm
    nm.load()
    O, I = 28672, 1024
    G = 10241                                       # odd; vals = G * O * 16 bytes = 4.70 GB
    T = 16 * G
    assert G * O * 16 > 2 ** 32
    print(f"large offsets: T={T} O={O} I={I}, vals {G * O * 16 / 2**30:.2f} GiB", flush=True)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(11)
    vals = torch.empty((G, O, 8), dtype=torch.bfloat16, device=DEV)
    meta = torch.empty((G, O), dtype=torch.int16, device=DEV)
    table = torch.tensor(NIBBLES, dtype=torch.int32, device=DEV)
    step = 1024
    for a in range(0, G, step):
        b = min(G, a + step)
        vals[a:b].normal_(generator=gen)
        pick = torch.randint(0, 6, (b - a, O, 4), generator=gen, device=DEV)
        nib = table[pick]
        word = nib[..., 0] | (nib[..., 1] << 4) | (nib[..., 2] << 8) | (nib[..., 3] << 12)
        meta[a:b] = word.to(torch.int16)                     # (values above 0x7fff wrap to the same 16 bits)
        del pick, nib, word
    g_mark = (2 ** 32) // (O * 16)                           # the group whose values straddle the 4 GiB mark
    windows = [(0, 3), (g_mark - 2, g_mark + 3), (G - 3, G)]
    h = torch.zeros((T, I), dtype=torch.bfloat16, device=DEV)
    for a, b in windows:
        h[16 * a:16 * b].normal_(generator=gen)
    need = nm.nm_update_gemm_workspace(T, O, I, torch.bfloat16)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=DEV)
    dW = torch.full((O, I), float("nan"), device=DEV)
    nm.nm_update_gemm(vals, meta, h, dW=dW, beta=0.0, workspace=ws)
    torch.cuda.synchronize()
    got = dW.cpu().numpy().astype(np.float64)
    del dW
    want = np.zeros((O, I))
    wabs = np.zeros((O, I))
    for a, b in windows:
        print(f"oracle window groups {a}..{b - 1}", flush=True)
        d, dabs = oracle.update_gemm(to_host(vals[a:b]), to_host(meta[a:b]), to_host(h[16 * a:16 * b]))
        want += d
        wabs += dabs
    assert np.isfinite(got).all()
    rel = float((np.abs(got - want) / np.maximum(wabs, 1e-300)).max())
    print(f"max |err|/sum|ab| = {rel:.3e}", flush=True)
    assert rel <= 1e-2


def test_update_gemm_q8_operand_beyond_4_gib(oracle):
    """the same for the 8-bit path: 32-token groups, e5m2 codes and 32-bit index words, e4m3 activations"""
    import paper_2203_10991_amd as nm
    nm.load()
    O, I = 28672, 1024
    G = 10241
    T = 32 * G
    print(f"large offsets, 8 bit: T={T} O={O} I={I}, vals8 {G * O * 16 / 2**30:.2f} GiB", flush=True)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(12)
    vals8 = torch.empty((G, O, 16), dtype=torch.uint8, device=DEV)
    meta32 = torch.empty((G, O), dtype=torch.int32, device=DEV)
    table = torch.tensor(NIBBLES, dtype=torch.int64, device=DEV)
    step = 1024
    for a in range(0, G, step):
        b = min(G, a + step)
        # finite e5m2 codes of moderate size (exponent field 8..19) with a random sign
        mag = torch.randint(8 << 2, 20 << 2, (b - a, O, 16), generator=gen, device=DEV)
        sign = torch.randint(0, 2, (b - a, O, 16), generator=gen, device=DEV) << 7
        vals8[a:b] = (mag | sign).to(torch.uint8)
        nib = table[torch.randint(0, 6, (b - a, O, 8), generator=gen, device=DEV)]
        word = torch.zeros((b - a, O), dtype=torch.int64, device=DEV)
        for q in range(8):
            word |= nib[..., q] << (4 * q)
        meta32[a:b] = torch.where(word >= 2 ** 31, word - 2 ** 32, word).to(torch.int32)
        del mag, sign, nib, word
    g_mark = (2 ** 32) // (O * 16)
    windows = [(0, 2), (g_mark - 1, g_mark + 2), (G - 3, G)]
    h8 = torch.zeros((T, I), dtype=torch.uint8, device=DEV)
    for a, b in windows:
        x = torch.empty((32 * (b - a), I), device=DEV).normal_(generator=gen) * 4.0
        h8[32 * a:32 * b] = x.to(torch.float8_e4m3fn).view(torch.uint8)
    alpha = 2.0 ** -6
    dW = torch.full((O, I), float("nan"), device=DEV)
    nm.nm_update_gemm_q8(vals8, meta32, h8, dW=dW, alpha=alpha, beta=0.0)
    torch.cuda.synchronize()
    got = dW.cpu().numpy().astype(np.float64)
    del dW
    want = np.zeros((O, I))
    wabs = np.zeros((O, I))
    for a, b in windows:
        print(f"oracle window groups {a}..{b - 1}", flush=True)
        d, dabs = oracle.update_gemm_q8(vals8[a:b].cpu().numpy(), meta32[a:b].cpu().numpy().view(np.uint32),
                                        h8[32 * a:32 * b].cpu().numpy(), alpha=alpha)
        want += d
        wabs += dabs
    assert np.isfinite(got).all()
    rel = float((np.abs(got - want) / np.maximum(wabs, 1e-300)).max())
    print(f"max |err|/sum|ab| = {rel:.3e}", flush=True)
    assert rel <= 1e-3

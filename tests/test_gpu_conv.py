"""GPU parity of the im2col-free update GEMM of a convolution (row-shifted views of the padded channels-last
activation grid) against the oracle's binary64 sums, through the C ABI; and against the plain update GEMM of the
library on a materialised im2col matrix."""
import numpy as np
import pytest
import torch

from paper_2203_10991_amd import synth
from gpu_util import DEV, to_dev, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nm():
    import paper_2203_10991_amd as p
    p.load()
    return p


def tap_shifts(k, wp):
    r = k // 2
    return [(ky - r) * wp + (kx - r) for ky in range(k) for kx in range(k)]


def make_case(N, H, W, C, O, k, seed):
    """bf16 bit patterns: x_full [margin + T + margin, C] on the padded grid, g [T, O] on the same grid"""
    rng = np.random.default_rng(seed)
    pad = k // 2
    Hp, Wp = H + 2 * pad, W + 2 * pad
    rows = N * Hp * Wp
    T = (rows + 15) // 16 * 16
    margin = pad * Wp + pad
    a = np.maximum(rng.standard_normal((N, H, W, C)), 0).astype(np.float32)                    # post-ReLU activations
    gy = (rng.standard_normal((N, H, W, O)) * np.exp(2 * rng.standard_normal((N, H, W, O)))).astype(np.float32)
    gy[rng.random((N, H, W, O)) < 0.3] = 0
    xg = np.zeros((N, Hp, Wp, C), dtype=np.float32); xg[:, pad:pad + H, pad:pad + W] = a
    gg = np.zeros((N, Hp, Wp, O), dtype=np.float32); gg[:, pad:pad + H, pad:pad + W] = gy
    x_full = np.zeros((T + 2 * margin, C), dtype=np.float32); x_full[margin:margin + rows] = xg.reshape(rows, C)
    g = np.zeros((T, O), dtype=np.float32); g[:rows] = gg.reshape(rows, O)
    return synth.f32_to_bf16_bits(x_full), synth.f32_to_bf16_bits(g), T, margin, tap_shifts(k, Wp)


@pytest.mark.parametrize("N,H,W,C,O,k", [(2, 6, 6, 8, 8, 3),          # tiny
                                         (3, 14, 14, 64, 64, 3),       # ResNet-like block, few tiles: split-K path
                                         (2, 9, 11, 24, 200, 3),       # ragged rows and columns (C not a power of two)
                                         (2, 8, 8, 16, 40, 5),         # 5x5 taps: 25 views
                                         (1, 20, 20, 32, 72, 1),       # 1x1: one view, no shift
                                         (8, 14, 14, 256, 504, 3)])    # 2 x 18 tiles of 256 x 128 (the mid-sized plan), ragged rows
def test_shifted_gemm_matches_oracle(nm, oracle, N, H, W, C, O, k):
    x_full, g, T, margin, shifts = make_case(N, H, W, C, O, k, seed=H + C + k)
    ov, om, _ = oracle.prune_2of4(g, 5, 1)
    want, wabs = oracle.update_gemm_shifted(ov, om, x_full, margin, shifts)
    v, m, _ = nm.mvue_prune_2of4(to_dev(g), seed=5, stream_id=1)
    xd = to_dev(x_full)
    dW = nm.nm_update_gemm_shifted(v, m, xd, margin, shifts)
    torch.cuda.synchronize()
    assert np.array_equal(to_host(m), om) and np.array_equal(to_host(v), ov)
    got = dW.cpu().numpy().astype(np.float64)
    rel = float((np.abs(got - want) / np.maximum(wabs, 1e-300)).max())
    print(f"conv N={N} {H}x{W} C={C} O={O} k={k}: T={T} I={len(shifts) * C} max |err|/sum|ab| = {rel:.3e}", flush=True)
    assert np.isfinite(got).all() and rel <= 1e-2
    # the library's plain GEMM on the materialised im2col matrix gives the same sums (same kernels, same order)
    h = torch.cat([xd[margin + s: margin + s + T] for s in shifts], dim=1).contiguous()
    dW2 = nm.nm_update_gemm(v, m, h)
    torch.cuda.synchronize()
    assert torch.allclose(dW, dW2, rtol=1e-5, atol=1e-5 * float(dW2.abs().max()))
    # beta = 1 accumulates
    dW3 = dW2.clone()
    nm.nm_update_gemm_shifted(v, m, xd, margin, shifts, dW=dW3, beta=1.0)
    torch.cuda.synchronize()
    assert torch.allclose(dW3, 2 * dW2, rtol=1e-5, atol=1e-5 * float(dW2.abs().max()))


def test_shifted_gemm_large_tiles(nm, oracle):
    """enough output tiles for the 256 x 256 kernel: O = 2048, I = 9 * 256"""
    x_full, g, T, margin, shifts = make_case(1, 12, 12, 256, 2048, 3, seed=1)
    ov, om, _ = oracle.prune_2of4(g, 2, 0)
    want, wabs = oracle.update_gemm_shifted(ov, om, x_full, margin, shifts)
    v, m, _ = nm.mvue_prune_2of4(to_dev(g), seed=2, stream_id=0)
    dW = nm.nm_update_gemm_shifted(v, m, to_dev(x_full), margin, shifts)
    torch.cuda.synchronize()
    got = dW.cpu().numpy().astype(np.float64)
    rel = float((np.abs(got - want) / np.maximum(wabs, 1e-300)).max())
    print(f"conv large tiles: T={T} O=2048 I={9 * 256} max |err|/sum|ab| = {rel:.3e}", flush=True)
    assert rel <= 1e-2


@pytest.mark.parametrize("N,H,W,C,O,k", [(2, 6, 6, 16, 8, 3), (3, 14, 14, 64, 64, 3), (2, 9, 11, 32, 200, 3), (1, 12, 12, 256, 2048, 3)])
def test_q8_shifted_gemm_matches_oracle(nm, oracle, N, H, W, C, O, k):
    """the 8-bit form: e5m2 kept values pruned on the padded grid, e4m3 activations as shifted views"""
    x_full, g, T, margin, shifts = make_case(N, H, W, C, O, k, seed=H + C)
    T32 = (T + 31) // 32 * 32                                    # 32-token groups
    g32 = np.zeros((T32, O), dtype=np.uint16); g32[:T] = g
    xf = np.zeros((T32 + 2 * margin, C), dtype=np.uint16); xf[:T + 2 * margin] = x_full
    gmax = float(np.abs(synth.bf16_to_f32(g32)).max())
    scale = float(2.0 ** np.floor(np.log2(57344.0 / (4.0 * gmax))))
    x8 = torch.from_numpy(synth.bf16_to_f32(xf) * 16.0).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    ov, om = oracle.prune_2of4_q8(g32, 5, 1, 0, scale)
    alpha = 1.0 / (16.0 * scale)
    if O * C * k * k <= 1 << 20:
        want, wabs = oracle.update_gemm_q8_shifted(ov, om, x8, margin, shifts, alpha=alpha)
        pick = None
    else:                                                        # large case: a band of rows is enough for the oracle
        pick = np.r_[0:8, O // 2:O // 2 + 8, O - 8:O]
        want, wabs = oracle.update_gemm_q8_shifted(np.ascontiguousarray(ov[:, pick]), np.ascontiguousarray(om[:, pick]), x8, margin, shifts, alpha=alpha)
    v, m = nm.mvue_prune_2of4_q8(to_dev(g32), seed=5, stream_id=1, mode=0, scale=scale)
    dW = nm.nm_update_gemm_q8_shifted(v, m, torch.from_numpy(x8).to(DEV), margin, shifts, alpha=alpha)
    torch.cuda.synchronize()
    assert np.array_equal(v.cpu().numpy(), ov) and np.array_equal(m.cpu().numpy().view(np.uint32), om)
    got = dW.cpu().numpy().astype(np.float64)
    if pick is not None:
        got = got[pick]
    rel = float((np.abs(got - want) / np.maximum(wabs, 1e-300)).max())
    print(f"q8 conv N={N} {H}x{W} C={C} O={O}: max |err|/sum|ab| = {rel:.3e}", flush=True)
    assert np.isfinite(got).all() and rel <= 1e-3

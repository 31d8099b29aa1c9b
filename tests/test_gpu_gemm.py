"""GPU parity: the update GEMM against the fp64 oracle, through the C ABI.

Tolerance (component-wise, against the sum of absolute products the oracle returns):
fp32 inputs 1e-5, bf16 inputs 1e-2 (bf16 products are exact in binary32, so only the
binary32 accumulation rounds; the observed error is printed)."""
import numpy as np
import pytest
import torch

from paper_2203_10991_amd import synth
from gpu_util import DEV, to_dev, to_host

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-5, "bf16": 1e-2}


@pytest.fixture(scope="module")
def nm():
    import paper_2203_10991_amd as p
    p.load()
    return p


def run_case(nm, oracle, w, seed=0, beta=0.0):
    g, h = synth.make_g(w, seed), synth.make_h(w, seed)
    oprune = oracle.prune_1of2 if w.nm == "1:2" else oracle.prune_2of4
    ov, om, _ = oprune(g, seed, 0)
    prior = None
    if beta:
        prior = np.random.default_rng(1).standard_normal((w.O, w.I)).astype(np.float32)
    want, wabs = oracle.update_gemm(ov, om, h, beta=beta, dW_in=prior)
    # device side: its own prune output feeds its GEMM
    gprune = nm.mvue_prune_1of2 if w.nm == "1:2" else nm.mvue_prune_2of4
    v, m, _ = gprune(to_dev(g), seed=seed, stream_id=0)
    dW = to_dev(prior) if beta else torch.full((w.O, w.I), float("nan"), device=DEV)
    nm.nm_update_gemm(v, m, to_dev(h), dW=dW, beta=beta)
    torch.cuda.synchronize()
    got = dW.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    scale = wabs + (np.abs(prior) if beta else 0.0)
    err = np.abs(got - want)
    rel = float((err / np.maximum(scale, 1e-300)).max())
    fro = float(np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300))
    print(f"{w.name}: T={w.T} O={w.O} I={w.I} max |err|/sum|ab| = {rel:.3e}, frobenius = {fro:.3e}", flush=True)
    assert rel <= TOL[w.dtype] and fro <= TOL[w.dtype]


SHAPES = [(64, 64, 64), (16, 8, 8), (16 * 11, 8 * 9, 8 * 7), (16 * 33, 64 * 3 + 8, 64 * 2 + 24), (1024, 256, 320)]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("nmode", ["1:2", "2:4"])
@pytest.mark.parametrize("shape", SHAPES)
def test_update_gemm_matches_fp64_oracle(nm, oracle, dtype, nmode, shape):
    T, O, I = shape
    run_case(nm, oracle, synth.Workload(f"s{T}x{O}x{I}_{dtype}_{nmode}", T, O, I, dtype, nmode, 0.0, 2.0, 0.3), seed=T)


@pytest.mark.parametrize("T,O,I", [(112, 16 * 256, 16 * 256),            # 16 x 16 tiles of 256 x 256: the 2 x 4 XCD grid
                                   (80, 50 * 256 - 40, 8 * 256),         # 50 x 8 tiles: banded map with a short last band
                                   (80, 25 * 256, 10 * 256 - 8),         # 25 x 10 tiles: the map for other tile counts
                                   (96, 17 * 256 - 40, 16 * 256),        # 12 x 16 tiles of 384 x 256 alone, ragged last tile row
                                   (96, 32 * 384, 16 * 256),             # 32 x 16 tiles of 384 x 256 alone
                                   (80, 16 * 384 + 16 * 256, 16 * 256)]) # rows split: 16 tile rows of 384, then 16 of 256
def test_large_tile_kernels_and_their_tile_maps(nm, oracle, T, O, I):
    """Enough output tiles for the 8-wave kernels (256 x 256, 384 x 256, or both on a row split), at short
    reductions with a ragged last stage.  Which kernel a shape takes follows from the plan's cost rule."""
    run_case(nm, oracle, synth.Workload(f"big{T}x{O}x{I}", T, O, I, "bf16", "2:4", 0.0, 2.0, 0.3), seed=T)


@pytest.mark.parametrize("T,O,I,slabs,beta", [(8208, 3064, 1528, 3, 0.0), (16400, 2296, 760, 4, 1.0), (10784, 2472, 888, 3, 1.0), (6416, 2296, 2040, 0, 0.0)])
def test_large_tiles_with_split_k(nm, oracle, T, O, I, slabs, beta):
    """Mid-sized problems (fewer than 256 tiles of 256 x 256, a long reduction) run on the 256 x 256 kernel with the
    token axis cut into slabs: ragged last tile row and column, a ragged last slab, and the second pass over the
    partial sums.  The slab count identifies the plan of the first (256 // tiles of 256 x 256 = 3; the other plans would
    take one slab); the next two are sizes the plan gives to 256 x 128 tiles cut into slabs (54 and 70 tiles), with
    beta = 1; the last to 144 tiles of 256 x 128 in one pass."""
    need = nm.nm_update_gemm_workspace(T, O, I, torch.bfloat16)
    assert need == (slabs * O * I * 4 if slabs > 1 else 0)
    run_case(nm, oracle, synth.Workload(f"mid{T}x{O}x{I}", T, O, I, "bf16", "2:4", 0.0, 2.0, 0.3), seed=T, beta=beta)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_beta_one_accumulates(nm, oracle, dtype):
    run_case(nm, oracle, synth.Workload("beta", 16 * 20, 8 * 21, 8 * 19, dtype, "2:4", 0.0, 2.0, 0.3), seed=2, beta=1.0)


def test_beta_one_accumulates_in_the_large_tile_kernels(nm, oracle):
    run_case(nm, oracle, synth.Workload("beta_big", 48, 16 * 384 + 16 * 256 - 16, 16 * 256, "bf16", "2:4", 0.0, 2.0, 0.3),
             seed=3, beta=1.0)


def test_zero_operand_and_empty_reduction(nm):
    v, m = nm.alloc_compressed(64, 64, torch.bfloat16, DEV)
    v.zero_(); m.fill_(0x4E4E)                       # index (2,3) everywhere: valid pattern, zero values
    h = torch.randn((64, 32), device=DEV).bfloat16()
    dW = nm.nm_update_gemm(v, m, h)
    assert not bool(dW.any())
    v0, m0 = nm.alloc_compressed(0, 64, torch.bfloat16, DEV)
    dW = torch.full((64, 32), 3.0, device=DEV)
    nm.nm_update_gemm(v0, m0, torch.zeros((0, 32), dtype=torch.bfloat16, device=DEV), dW=dW, beta=0.0)
    assert not bool(dW.any())


@pytest.mark.parametrize("name,T,O,I", [("c1_fp32_1of2", 1024, 256, 256), ("c2_mlp_1of2", 2048, 512, 256),
                                        ("c3_conv_2of4", 16384, 64, 576), ("c4_vit_qkv_2of4", 1600, 384, 256),
                                        ("c4_vit_fc2_1of2", 1600, 256, 512), ("c5_decoder_mlp_2of4", 2048, 512, 512)])
def test_config_recipes_reduced(nm, oracle, name, T, O, I):
    run_case(nm, oracle, synth.scaled(synth.WORKLOADS[name], T=T, O=O, I=I, name=name + "_reduced"))


def test_update_gemm_consumes_the_1of4_container(nm, oracle):
    """MVUE 1:4 output is stored in the 2:4 group format: the same GEMM multiplies it"""
    w = synth.Workload("g14", 16 * 21, 200, 136, "bf16", "2:4", 0.0, 2.0, 0.3)
    g, h = synth.make_g(w, 3), synth.make_h(w, 3)
    ov, om, _ = oracle.prune_1of4(g, 3, 0)
    want, wabs = oracle.update_gemm(ov, om, h)
    v, m, _ = nm.mvue_prune_1of4(to_dev(g), seed=3, stream_id=0)
    dW = nm.nm_update_gemm(v, m, to_dev(h))
    torch.cuda.synchronize()
    assert np.array_equal(to_host(m), om) and np.array_equal(to_host(v), ov)
    rel = float((np.abs(dW.cpu().numpy().astype(np.float64) - want) / np.maximum(wabs, 1e-300)).max())
    assert rel <= TOL["bf16"]


def _random_shapes(n, seed, t_mult, i_mult):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        T = int(rng.integers(1, 300)) * t_mult
        O = int(rng.integers(1, 80)) * 8
        I = int(rng.integers(1, 60)) * i_mult
        out.append((T, O, I))
    return out


@pytest.mark.parametrize("T,O,I", _random_shapes(14, 2024, 16, 8))
def test_update_gemm_random_shapes(nm, oracle, T, O, I):
    """seeded random problem sizes: every branch of the split-K plan (slab counts, tile counts that are and are not
    multiples of 8, ragged tiles, ragged last stages) against the oracle"""
    run_case(nm, oracle, synth.Workload(f"r{T}x{O}x{I}", T, O, I, "bf16", "2:4", 0.0, 2.0, 0.3), seed=T + O + I)


def _random_mid_shapes(n, seed):
    rng = np.random.default_rng(seed)
    return [(int(rng.integers(200, 900)) * 16, int(rng.integers(100, 400)) * 8, int(rng.integers(100, 400)) * 8) for _ in range(n)]


@pytest.mark.parametrize("T,O,I", _random_mid_shapes(5, 31))
def test_update_gemm_random_mid_sized_shapes(nm, oracle, T, O, I):
    """seeded random mid-sized problems (tens of tiles of 256 x 256, thousands of tokens): the plans that choose between
    128 x 128 and 256 x 256 tiles with split-K, ragged in every dimension, against the oracle"""
    run_case(nm, oracle, synth.Workload(f"m{T}x{O}x{I}", T, O, I, "bf16", "2:4", 0.0, 2.0, 0.3), seed=T + O + I)


@pytest.mark.parametrize("dtype", ["bf16", "f32", "q8"])
@pytest.mark.parametrize("T,O,I", [(4096, 64, 576), (12608 - 12608 % 32, 768, 768), (2048, 1000, 528), (32 * 300, 256, 2304)])
def test_update_gemm_is_bitwise_reproducible(nm, dtype, T, O, I):
    """The reduction over the token slabs of a split-K plan has a fixed order: the same call gives the same bits,
    whatever ran on the device in between."""
    gen = torch.Generator(device=DEV)
    gen.manual_seed(T + O)
    if dtype == "q8":
        g = torch.empty((T, O), dtype=torch.bfloat16, device=DEV).normal_(generator=gen)
        v, m = nm.mvue_prune_2of4_q8(g, seed=3, stream_id=0, mode=0, scale=64.0)
        h = (torch.empty((T, I), device=DEV).normal_(generator=gen) * 4.0).to(torch.float8_e4m3fn).view(torch.uint8)
        call = lambda: nm.nm_update_gemm_q8(v, m, h, alpha=1.0 / 64.0)
    else:
        td = torch.bfloat16 if dtype == "bf16" else torch.float32
        g = torch.empty((T, O), dtype=td, device=DEV).normal_(generator=gen)
        h = torch.empty((T, I), dtype=td, device=DEV).normal_(generator=gen)
        v, m, _ = nm.mvue_prune_2of4(g, seed=3, stream_id=0)
        call = lambda: nm.nm_update_gemm(v, m, h)
    first = call().clone()
    for k in range(3):
        torch.mm(torch.empty((1024, 1024), device=DEV).normal_(generator=gen), torch.ones((1024, 1024), device=DEV))
        again = call()
        torch.cuda.synchronize()
        assert torch.equal(again.view(torch.int32), first.view(torch.int32)), (dtype, T, O, I, k)


def split_case(nm, oracle, T, O, I, seed, beta=0.0, sigma=2.5, sample=None):
    """binary32 tensors through the three-bf16-term mode of nm_update_gemm, against the oracle's binary64 sums at the
    binary32 tolerance (the dropped third-order products are below 2^-24 of a product)"""
    w = synth.Workload(f"x3_{T}x{O}x{I}", T, O, I, "f32", "2:4", 0.0, sigma, 0.3)
    g, h = synth.make_g(w, seed), synth.make_h(w, seed)
    ov, om, _ = oracle.prune_2of4(g, seed, 0)
    prior = np.random.default_rng(1).standard_normal((O, I)).astype(np.float32) if beta else None
    v, m, _ = nm.mvue_prune_2of4(to_dev(g), seed=seed, stream_id=0)
    dW = to_dev(prior) if beta else torch.full((O, I), float("nan"), device=DEV)
    nm.nm_update_gemm(v, m, to_dev(h), dW=dW, beta=beta, f32_as_bf16x3=True)
    torch.cuda.synchronize()
    got = dW.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    if sample is None:
        want, wabs = oracle.update_gemm(ov, om, h, beta=beta, dW_in=prior)
        if beta:
            wabs = wabs + np.abs(prior)
    else:
        rng = np.random.default_rng(seed)
        oi = np.stack([rng.integers(0, O, sample), rng.integers(0, I, sample)], axis=1)
        want, wabs = oracle.update_gemm_entries(ov, om, h, oi)
        got = got[oi[:, 0], oi[:, 1]]
    rel = float((np.abs(got - want) / np.maximum(wabs, 1e-300)).max())
    print(f"bf16x3 T={T} O={O} I={I} beta={beta}: max |err|/sum|ab| = {rel:.3e}", flush=True)
    assert rel <= TOL["f32"]


@pytest.mark.parametrize("T,O,I", [(64, 64, 64), (16, 8, 8), (16 * 11, 8 * 9, 8 * 7), (16 * 33, 64 * 3 + 8, 64 * 2 + 24),
                                   (1024, 256, 320), (4096, 64, 576)])
def test_update_gemm_f32_as_three_bf16_terms(nm, oracle, T, O, I):
    split_case(nm, oracle, T, O, I, seed=T + I)


def test_update_gemm_f32_as_three_bf16_terms_beta_one_and_wide_range(nm, oracle):
    split_case(nm, oracle, 16 * 20, 136, 96, seed=2, beta=1.0)
    split_case(nm, oracle, 512, 128, 128, seed=3, sigma=6.0)           # magnitudes over many binades
    split_case(nm, oracle, 2048, 16 * 256, 8 * 256, seed=4, sample=2000)  # large-tile kernels


def test_update_gemm_f32_split_special_values(nm):
    """an infinity in the compressed operand makes its row of dW non-finite (infinity times a zero low-order term of h
    is a NaN, so it need not stay an infinity); the other rows are untouched"""
    T, O, I = 64, 16, 16
    g = torch.randn((T, O), device=DEV)
    h = torch.rand((T, I), device=DEV) + 0.5
    v, m, _ = nm.mvue_prune_2of4(g, seed=1, stream_id=0)
    v[0, 3, 0] = float("inf")
    dW = nm.nm_update_gemm(v, m, h, f32_as_bf16x3=True)
    ref = nm.nm_update_gemm(v, m, h)
    torch.cuda.synchronize()
    assert not torch.isfinite(dW[3]).any()
    keep = [r for r in range(O) if r != 3]
    assert torch.allclose(dW[keep], ref[keep], rtol=1e-5, atol=1e-5)

"""Seeded synthetic inputs for the MVUE N:M prune + update-GEMM path.

This module only *draws inputs*: neural gradients ``g`` [T x O] and layer
inputs ``h`` [T x I] with the shapes and value statistics of the layers the
paper trains (ResNet conv as im2col, ViT / BERT / Transformer linear layers;
Table 3 and App. A.4 give the models and batch sizes, Sec. 2 the lognormal
view of neural gradients).  It contains none of the method's arithmetic and
is imported by the tests, the benchmark and the smoke check; neither the
oracle nor the HIP library imports it.

bf16 tensors are carried as ``uint16`` bit patterns on the host (numpy has no
bf16); ``bf16_to_f32`` / ``f32_to_bf16_bits`` convert.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, Tuple

import numpy as np

CHUNK_ROWS = 512  # rows per independently seeded chunk (fixed: part of the recipe)
_TAG_G, _TAG_H = 0x67, 0x68


@dataclass(frozen=True)
class Workload:
    """One update-GEMM problem: dW[O x I] = theta(g)^T h, blocks along T."""

    name: str
    T: int
    O: int
    I: int
    dtype: str            # "f32" | "bf16"
    nm: str               # "1:2" | "2:4"
    mu: float
    sigma: float
    zero_frac: float
    h_kind: str = "normal"  # "normal" | "relu" (half-normal with 50 % zeros)
    note: str = ""

    @property
    def flops_dense_equiv(self) -> int:
        return 2 * self.T * self.O * self.I

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def prune_bytes(self) -> int:
        """Algorithmic bytes of prune+compress: read g, write half of it, 1/8 B of index per element."""
        n = self.T * self.O
        return n * self.elem_bytes + n * self.elem_bytes // 2 + n // 8


def _w(name, T, O, I, dtype, nm, mu, sigma, zf, h_kind="normal", note=""):
    return Workload(name, T, O, I, dtype, nm, mu, sigma, zf, h_kind, note)


# The five benchmark configurations (names used by tests and bench.py).
WORKLOADS: Dict[str, Workload] = {w.name: w for w in [
    _w("c1_fp32_1of2", 1024, 1024, 1024, "f32", "1:2", 0.0, 2.0, 0.30),
    _w("c2_mlp_1of2", 16384, 4096, 1024, "bf16", "1:2", 0.0, 2.5, 0.40,
       note="transformer MLP, hidden 1024, FFN 4096, 32x512 tokens"),
    _w("c3_conv_2of4", 802816, 64, 576, "bf16", "2:4", 0.0, 3.0, 0.50, "relu",
       note="ResNet-50 stage-1 3x3 conv as im2col, batch 256, 56x56"),
    _w("c4_vit_qkv_1of2", 12608, 2304, 768, "bf16", "1:2", 0.0, 2.0, 0.20),
    _w("c4_vit_qkv_2of4", 12608, 2304, 768, "bf16", "2:4", 0.0, 2.0, 0.20),
    _w("c4_vit_proj_1of2", 12608, 768, 768, "bf16", "1:2", 0.0, 2.0, 0.20),
    _w("c4_vit_proj_2of4", 12608, 768, 768, "bf16", "2:4", 0.0, 2.0, 0.20),
    _w("c4_vit_fc1_1of2", 12608, 3072, 768, "bf16", "1:2", 0.0, 2.0, 0.20),
    _w("c4_vit_fc1_2of4", 12608, 3072, 768, "bf16", "2:4", 0.0, 2.0, 0.20),
    _w("c4_vit_fc2_1of2", 12608, 768, 3072, "bf16", "1:2", 0.0, 2.0, 0.20),
    _w("c4_vit_fc2_2of4", 12608, 768, 3072, "bf16", "2:4", 0.0, 2.0, 0.20),
    _w("c5_decoder_mlp_2of4", 32768, 28672, 8192, "bf16", "2:4", 0.0, 2.5, 0.10,
       note="large decoder MLP, hidden 8192, FFN 28672, 32768 tokens"),
    # not one of the five: the binary32 path at a size that is not launch-bound (c1 is 2 GFLOP)
    _w("x_fp32_mlp_2of4", 16384, 8192, 8192, "f32", "2:4", 0.0, 2.5, 0.10,
       note="binary32 operands, 16384 tokens, 8192 x 8192"),
]}


# ----------------------------------------------------------------------------
# bf16 <-> fp32 on the host (bit patterns)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns (finite inputs)."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + (np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------
# numpy generators (chunked: any row range can be produced on its own)
# ----------------------------------------------------------------------------
def _rng(seed: int, tag: int, chunk: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(seed), tag, int(chunk)])))


def _g_chunk(w: Workload, seed: int, chunk: int, rows: int) -> np.ndarray:
    r = _rng(seed, _TAG_G, chunk)
    n = (rows, w.O)
    sign = r.integers(0, 2, size=n, dtype=np.int8).astype(np.float32) * 2.0 - 1.0
    z = r.standard_normal(size=n, dtype=np.float32)
    keep = r.random(size=n, dtype=np.float32) >= np.float32(w.zero_frac)
    g = sign * np.exp(np.float32(w.mu) + np.float32(w.sigma) * z, dtype=np.float32)
    g = np.where(keep, g, np.float32(0.0)).astype(np.float32)
    return g


def _h_chunk(w: Workload, seed: int, chunk: int, rows: int) -> np.ndarray:
    r = _rng(seed, _TAG_H, chunk)
    n = (rows, w.I)
    h = r.standard_normal(size=n, dtype=np.float32)
    if w.h_kind == "relu":
        keep = r.random(size=n, dtype=np.float32) >= np.float32(0.5)
        h = np.where(keep, np.abs(h), np.float32(0.0)).astype(np.float32)
    return h


def _assemble(fn, w: Workload, seed: int, row0: int, row1: int, width: int, threads: int) -> np.ndarray:
    assert row0 % CHUNK_ROWS == 0, "row ranges start on a chunk boundary"
    out_dtype = np.float32 if w.dtype == "f32" else np.uint16
    out = np.empty((row1 - row0, width), dtype=out_dtype)

    def job(c):
        a = c * CHUNK_ROWS
        b = min(a + CHUNK_ROWS, row1)
        x = fn(w, seed, c, CHUNK_ROWS)[: b - a]
        out[a - row0: b - row0] = x if w.dtype == "f32" else f32_to_bf16_bits(x)

    chunks = range(row0 // CHUNK_ROWS, (row1 + CHUNK_ROWS - 1) // CHUNK_ROWS)
    if threads > 1 and len(chunks) > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(job, chunks))
    else:
        for c in chunks:
            job(c)
    return out


def make_g(w: Workload, seed: int = 0, rows: Tuple[int, int] | None = None, threads: int = 8) -> np.ndarray:
    """g[T x O] (or the row range ``rows``): sign * lognormal(mu, sigma) with iid exact zeros.

    f32 workloads return float32; bf16 workloads return uint16 bit patterns (RNE from fp32).
    """
    r0, r1 = rows if rows is not None else (0, w.T)
    return _assemble(_g_chunk, w, seed, r0, r1, w.O, threads)


def make_h(w: Workload, seed: int = 0, rows: Tuple[int, int] | None = None, threads: int = 8) -> np.ndarray:
    """h[T x I]: N(0,1); for ``relu`` workloads |N(0,1)| with 50 % iid zeros."""
    r0, r1 = rows if rows is not None else (0, w.T)
    return _assemble(_h_chunk, w, seed, r0, r1, w.I, threads)


def scaled(w: Workload, T: int | None = None, O: int | None = None, I: int | None = None, name: str | None = None) -> Workload:
    """The same value recipe at a reduced shape (parity cases the oracle finishes in seconds)."""
    return Workload(name or (w.name + "_small"), T or w.T, O or w.O, I or w.I, w.dtype, w.nm,
                    w.mu, w.sigma, w.zero_frac, w.h_kind, w.note)


# ----------------------------------------------------------------------------
# device generator (full-size tensors drawn directly in HBM)
# ----------------------------------------------------------------------------
def make_device(w: Workload, seed: int = 0, device: str = "cuda:0", rows_per_pass: int = 4096):
    """Draw (g, h) for ``w`` on ``device`` with torch's seeded generator.

    Same recipe as the numpy path (sign, lognormal magnitude, iid zero mask; h normal or
    half-normal with zeros) but a different bit stream, so host and device tensors of the
    same seed are *not* equal: a test that needs both sides copies the device tensor back.
    Generated in row slabs so that no fp32 copy of the full tensor is ever resident.
    """
    import torch

    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed) * 7919 + 17)
    tdt = torch.float32 if w.dtype == "f32" else torch.bfloat16
    g = torch.empty((w.T, w.O), dtype=tdt, device=device)
    h = torch.empty((w.T, w.I), dtype=tdt, device=device)
    for a in range(0, w.T, rows_per_pass):
        b = min(a + rows_per_pass, w.T)
        n = (b - a, w.O)
        z = torch.randn(n, generator=gen, device=device, dtype=torch.float32)
        mag = torch.exp(w.mu + w.sigma * z)
        sign = torch.randint(0, 2, n, generator=gen, device=device, dtype=torch.int8).to(torch.float32) * 2 - 1
        keep = torch.rand(n, generator=gen, device=device, dtype=torch.float32) >= w.zero_frac
        g[a:b] = torch.where(keep, sign * mag, torch.zeros((), device=device)).to(tdt)
        n = (b - a, w.I)
        x = torch.randn(n, generator=gen, device=device, dtype=torch.float32)
        if w.h_kind == "relu":
            keep = torch.rand(n, generator=gen, device=device, dtype=torch.float32) >= 0.5
            x = torch.where(keep, x.abs(), torch.zeros((), device=device))
        h[a:b] = x.to(tdt)
    return g, h


def make_device_from_host(w: Workload, seed: int = 0, device: str = "cuda:0", threads: int = 8, rows_per_pass: int = 4096):
    """(g, h) of ``w`` on ``device`` from the HOST recipe (numpy PCG64, the arrays make_g / make_h return), drawn and
    copied in row slabs: the device tensors equal what a test or the CPU oracle gets from make_g / make_h for the same
    seed, element for element."""
    import torch

    tdt = torch.float32 if w.dtype == "f32" else torch.bfloat16
    g = torch.empty((w.T, w.O), dtype=tdt, device=device)
    h = torch.empty((w.T, w.I), dtype=tdt, device=device)

    def put(dst, a):
        if w.dtype == "f32":
            dst.copy_(torch.from_numpy(a))
        else:
            dst.view(torch.int16).copy_(torch.from_numpy(a.view(np.int16)))

    for a in range(0, w.T, rows_per_pass):
        b = min(a + rows_per_pass, w.T)
        put(g[a:b], make_g(w, seed, rows=(a, b), threads=threads))
        put(h[a:b], make_h(w, seed, rows=(a, b), threads=threads))
    return g, h

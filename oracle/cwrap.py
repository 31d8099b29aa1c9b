"""ctypes loader for the C oracle (``mvue_oracle.c``).  TEST INFRASTRUCTURE ONLY.

Only the tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this module; the product package never does.

Arrays: f32 tensors are ``numpy.float32``; bf16 tensors are ``numpy.uint16`` bit
patterns.  The compressed operand is ``vals[T/16, O, 8]`` + ``meta[T/16, O]``
(uint16), the group format described at the top of the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mvue_oracle.c")
_LIB = os.path.join(_HERE, "libmvue_oracle.so")

DT_F32, DT_BF16 = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no contraction, no fast-math, OpenMP over independent blocks)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        vp, i64, u64, u32, i32, dbl = C.c_void_p, C.c_int64, C.c_uint64, C.c_uint32, C.c_int, C.c_double
        _lib.oracle_philox4x32_10.argtypes = [vp, vp, vp]
        _lib.oracle_philox4x32_10.restype = None
        _lib.oracle_block_u24.argtypes = [u64, u32, u64]
        _lib.oracle_block_u24.restype = u32
        _lib.oracle_select_1of2.argtypes = [vp, C.c_float, vp, vp]
        _lib.oracle_select_1of2.restype = None
        _lib.oracle_select_2of4.argtypes = [vp, C.c_float, vp, vp, vp]
        _lib.oracle_select_2of4.restype = None
        _lib.oracle_enumerate_1of2.argtypes = [vp, vp, vp, vp]
        _lib.oracle_enumerate_1of2.restype = None
        _lib.oracle_enumerate_2of4.argtypes = [vp, vp, vp, vp]
        _lib.oracle_enumerate_2of4.restype = None
        _lib.oracle_block_u24_pair.argtypes = [u64, u32, u64, vp]
        _lib.oracle_block_u24_pair.restype = None
        _lib.oracle_select_2of4_approx.argtypes = [vp, C.c_float, C.c_float, vp, vp]
        _lib.oracle_select_2of4_approx.restype = None
        _lib.oracle_enumerate_approx_draw.argtypes = [vp, i32, vp]
        _lib.oracle_enumerate_approx_draw.restype = None
        _lib.oracle_select_1of4.argtypes = [vp, C.c_float, vp, vp]
        _lib.oracle_select_1of4.restype = None
        _lib.oracle_enumerate_1of4.argtypes = [vp, vp, vp, vp]
        _lib.oracle_enumerate_1of4.restype = None
        for f in (_lib.oracle_prune_1of2, _lib.oracle_prune_2of4, _lib.oracle_prune_2of4_approx, _lib.oracle_prune_1of4):
            f.argtypes = [vp, i64, i64, i64, i32, u64, u32, vp, vp, vp, i64]
            f.restype = i32
        _lib.oracle_nm_compress.argtypes = [vp, i64, i64, i64, i32, i32, i32, vp, vp]
        _lib.oracle_nm_compress.restype = i64
        _lib.oracle_nm_decompress.argtypes = [vp, vp, i64, i64, i32, vp, i64]
        _lib.oracle_nm_decompress.restype = None
        _lib.oracle_update_gemm.argtypes = [vp, vp, vp, i64, i64, i64, i64, i32, dbl, vp, vp, vp]
        _lib.oracle_update_gemm.restype = None
        _lib.oracle_update_gemm_entries.argtypes = [vp, vp, vp, i64, i64, i64, i64, i32, vp, i64, vp, vp]
        _lib.oracle_update_gemm_entries.restype = None
        u8, flt = C.c_uint8, C.c_float
        _lib.oracle_e5m2_value.argtypes = [u8]
        _lib.oracle_e5m2_value.restype = dbl
        _lib.oracle_e4m3_value.argtypes = [u8]
        _lib.oracle_e4m3_value.restype = dbl
        _lib.oracle_sr_e5m2.argtypes = [flt, u32]
        _lib.oracle_sr_e5m2.restype = u8
        _lib.oracle_block_r16_pair.argtypes = [u64, u32, u64, vp]
        _lib.oracle_block_r16_pair.restype = None
        _lib.oracle_prune_2of4_q8.argtypes = [vp, i64, i64, i64, i32, u64, u32, i32, flt, vp, vp]
        _lib.oracle_prune_2of4_q8.restype = i32
        _lib.oracle_prune_1of2_q8.argtypes = [vp, i64, i64, i64, i32, u64, u32, flt, vp, vp]
        _lib.oracle_prune_1of2_q8.restype = i32
        _lib.oracle_nm_decompress_q8.argtypes = [vp, vp, i64, i64, vp]
        _lib.oracle_nm_decompress_q8.restype = None
        _lib.oracle_update_gemm_q8.argtypes = [vp, vp, vp, i64, i64, i64, i64, dbl, vp, i64, vp, vp]
        _lib.oracle_update_gemm_q8.restype = None
        _lib.oracle_update_gemm_shifted.argtypes = [vp, vp, vp, i64, i64, vp, i32, i64, i64, i32, vp, vp]
        _lib.oracle_update_gemm_shifted.restype = None
        _lib.oracle_update_gemm_q8_shifted.argtypes = [vp, vp, vp, i64, i64, vp, i32, i64, i64, dbl, vp, vp]
        _lib.oracle_update_gemm_q8_shifted.restype = None
        _lib.oracle_select_greedy.argtypes = [vp, i32, i32, vp]
        _lib.oracle_select_greedy.restype = None
        _lib.oracle_prune_greedy.argtypes = [vp, i64, i64, i64, i32, i32, i32, vp, vp, vp, i64]
        _lib.oracle_prune_greedy.restype = i32
        _lib.oracle_block_u24_quad.argtypes = [u64, u32, u64, vp]
        _lib.oracle_block_u24_quad.restype = None
        _lib.oracle_draw8.argtypes = [vp, flt, u32]
        _lib.oracle_draw8.restype = i32
        _lib.oracle_inclusion_4of8.argtypes = [vp, vp]
        _lib.oracle_inclusion_4of8.restype = None
        _lib.oracle_select_4of8_approx.argtypes = [vp, vp, vp, vp]
        _lib.oracle_select_4of8_approx.restype = None
        _lib.oracle_enumerate_draw8.argtypes = [vp, u32, vp]
        _lib.oracle_enumerate_draw8.restype = None
        _lib.oracle_prune_4of8_approx.argtypes = [vp, i64, i64, i64, i32, u64, u32, vp, vp, vp, i64]
        _lib.oracle_prune_4of8_approx.restype = i32
        _lib.oracle_nm_decompress_4of8.argtypes = [vp, vp, i64, i64, i32, vp, i64]
        _lib.oracle_nm_decompress_4of8.restype = None
        _lib.oracle_pow2_scale.argtypes = [vp, i64, i64, i64, i32, flt]
        _lib.oracle_pow2_scale.restype = flt
        _lib.oracle_e4m3_rne.argtypes = [flt]
        _lib.oracle_e4m3_rne.restype = u8
        _lib.oracle_cast_e4m3.argtypes = [vp, i64, i64, i64, i32, flt, vp, i64]
        _lib.oracle_cast_e4m3.restype = None
        _lib.oracle_act_backward.argtypes = [vp, i64, vp, i64, i64, i64, i32, vp, i64]
        _lib.oracle_act_backward.restype = None
        _lib.oracle_num_threads.argtypes = []
        _lib.oracle_num_threads.restype = i32
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _dt(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return DT_F32
    if a.dtype == np.uint16:
        return DT_BF16
    raise TypeError(f"oracle tensors are float32 or uint16 (bf16 bits), got {a.dtype}")


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def philox4x32_10(ctr, key) -> np.ndarray:
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    out = np.zeros(4, dtype=np.uint32)
    lib().oracle_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def block_u24(seed: int, stream_id: int, blk: int) -> int:
    return int(lib().oracle_block_u24(seed, stream_id, blk))


def select_1of2(x, eps: float) -> Tuple[int, float]:
    xa = np.asarray(x, dtype=np.float32).copy()
    k = C.c_int(0)
    v = C.c_float(0)
    lib().oracle_select_1of2(_p(xa), C.c_float(eps), C.byref(k), C.byref(v))
    return k.value, v.value


def select_2of4(x, eps: float):
    xa = np.asarray(x, dtype=np.float32).copy()
    pos = np.zeros(2, dtype=np.int32)
    val = np.zeros(2, dtype=np.float32)
    wc = C.c_int(0)
    lib().oracle_select_2of4(_p(xa), C.c_float(eps), _p(pos), _p(val), C.byref(wc))
    return (int(pos[0]), int(pos[1])), (float(val[0]), float(val[1])), wc.value


def enumerate_1of2(x):
    xa = np.asarray(x, dtype=np.float32).copy()
    counts = np.zeros(2, dtype=np.uint64)
    mean = np.zeros(2)
    second = np.zeros(2)
    lib().oracle_enumerate_1of2(_p(xa), _p(counts), _p(mean), _p(second))
    return counts, mean, second


PAIR_ORDER = [(0, 1), (0, 2), (0, 3), (1, 2), (1, 3), (2, 3)]


def enumerate_2of4(x):
    xa = np.asarray(x, dtype=np.float32).copy()
    counts = np.zeros(6, dtype=np.uint64)
    mean = np.zeros(4)
    second = np.zeros(4)
    lib().oracle_enumerate_2of4(_p(xa), _p(counts), _p(mean), _p(second))
    return counts, mean, second


def block_u24_pair(seed: int, stream_id: int, blk: int) -> Tuple[int, int]:
    u = np.zeros(2, dtype=np.uint32)
    lib().oracle_block_u24_pair(seed, stream_id, blk, _p(u))
    return int(u[0]), int(u[1])


def select_2of4_approx(x, eps1: float, eps2: float):
    xa = np.asarray(x, dtype=np.float32).copy()
    pos = np.zeros(2, dtype=np.int32)
    val = np.zeros(2, dtype=np.float32)
    lib().oracle_select_2of4_approx(_p(xa), C.c_float(eps1), C.c_float(eps2), _p(pos), _p(val))
    return (int(pos[0]), int(pos[1])), (float(val[0]), float(val[1]))


def enumerate_approx_draw(x, first: int = -1) -> np.ndarray:
    """Counts, over all 2^24 uniforms, of the position drawn (second draw when `first` >= 0)."""
    xa = np.asarray(x, dtype=np.float32).copy()
    counts = np.zeros(4, dtype=np.uint64)
    lib().oracle_enumerate_approx_draw(_p(xa), first, _p(counts))
    return counts


def _prune(fn, g: np.ndarray, seed: int, stream_id: int, want_dense: bool, logical_O: Optional[int] = None):
    assert g.ndim == 2
    T, O = g.shape
    ld = g.strides[0] // g.itemsize
    assert g.strides[1] == g.itemsize
    vals = np.zeros((T // 16, O, 8), dtype=g.dtype)
    meta = np.zeros((T // 16, O), dtype=np.uint16)
    dense = np.zeros((T, O), dtype=g.dtype) if want_dense else None
    rc = fn(_p(g), T, O, ld, _dt(g), seed, stream_id, _p(vals), _p(meta), _p(dense), O)
    if rc != 0:
        raise ValueError("oracle: shape not representable (T must be a multiple of 16)")
    return vals, meta, dense


def prune_1of2(g: np.ndarray, seed: int = 0, stream_id: int = 0, want_dense: bool = False):
    return _prune(lib().oracle_prune_1of2, g, seed, stream_id, want_dense)


def prune_2of4(g: np.ndarray, seed: int = 0, stream_id: int = 0, want_dense: bool = False):
    return _prune(lib().oracle_prune_2of4, g, seed, stream_id, want_dense)


def prune_2of4_approx(g: np.ndarray, seed: int = 0, stream_id: int = 0, want_dense: bool = False):
    return _prune(lib().oracle_prune_2of4_approx, g, seed, stream_id, want_dense)


def select_1of4(x, eps: float) -> Tuple[int, float]:
    xa = np.ascontiguousarray(x, dtype=np.float32)
    k = C.c_int(0)
    v = C.c_float(0)
    lib().oracle_select_1of4(_p(xa), C.c_float(eps), C.byref(k), C.byref(v))
    return int(k.value), float(v.value)


def enumerate_1of4(x):
    """Over all 2^24 uniforms: (counts[4], mean[4], second_moment[4]) of the kept position / emitted value."""
    xa = np.ascontiguousarray(x, dtype=np.float32)
    counts = np.zeros(4, dtype=np.uint64)
    mean = np.zeros(4, dtype=np.float64)
    second = np.zeros(4, dtype=np.float64)
    lib().oracle_enumerate_1of4(_p(xa), _p(counts), _p(mean), _p(second))
    return counts, mean, second


def prune_1of4(g: np.ndarray, seed: int = 0, stream_id: int = 0, want_dense: bool = False):
    return _prune(lib().oracle_prune_1of4, g, seed, stream_id, want_dense)


def nm_compress(dense: np.ndarray, n: int, m: int):
    T, O = dense.shape
    ld = dense.strides[0] // dense.itemsize
    vals = np.zeros((T // 16, O, 8), dtype=dense.dtype)
    meta = np.zeros((T // 16, O), dtype=np.uint16)
    bad = lib().oracle_nm_compress(_p(dense), T, O, ld, _dt(dense), n, m, _p(vals), _p(meta))
    if bad < 0:
        raise ValueError("oracle: bad shape or (n, m)")
    return vals, meta, int(bad)


def nm_decompress(vals: np.ndarray, meta: np.ndarray) -> np.ndarray:
    G, O, _ = vals.shape
    dense = np.zeros((G * 16, O), dtype=vals.dtype)
    lib().oracle_nm_decompress(_p(vals), _p(meta), G * 16, O, _dt(vals), _p(dense), O)
    return dense


def update_gemm(vals: np.ndarray, meta: np.ndarray, h: np.ndarray, beta: float = 0.0,
                dW_in: Optional[np.ndarray] = None):
    """fp64 dW[O x I] and the absolute-value sum used to scale error bounds."""
    G, O, _ = vals.shape
    T, I = h.shape
    assert T == G * 16 and h.dtype == vals.dtype
    ldh = h.strides[0] // h.itemsize
    dW = np.zeros((O, I), dtype=np.float64)
    absdW = np.zeros((O, I), dtype=np.float64)
    if dW_in is not None:
        dW_in = np.ascontiguousarray(dW_in, dtype=np.float32)
    lib().oracle_update_gemm(_p(vals), _p(meta), _p(h), ldh, T, O, I, _dt(vals), float(beta), _p(dW_in),
                             _p(dW), _p(absdW))
    return dW, absdW


def update_gemm_entries(vals: np.ndarray, meta: np.ndarray, h: np.ndarray, oi: np.ndarray):
    G, O, _ = vals.shape
    T, I = h.shape
    assert T == G * 16 and h.dtype == vals.dtype
    ldh = h.strides[0] // h.itemsize
    oi = np.ascontiguousarray(oi, dtype=np.int64).reshape(-1, 2)
    out = np.zeros(len(oi))
    out_abs = np.zeros(len(oi))
    lib().oracle_update_gemm_entries(_p(vals), _p(meta), _p(h), ldh, T, O, I, _dt(vals), _p(oi), len(oi),
                                     _p(out), _p(out_abs))
    return out, out_abs


# ---- 8-bit neural gradients (e5m2, stochastic rounding) on top of 2:4 sparsity; 32-token groups:
# vals8[T/32, O, 16] uint8 + meta32[T/32, O] uint32

def e5m2_value(code: int) -> float:
    return float(lib().oracle_e5m2_value(int(code) & 0xFF))


def e4m3_value(code: int) -> float:
    return float(lib().oracle_e4m3_value(int(code) & 0xFF))


def sr_e5m2(x: float, r16: int) -> int:
    return int(lib().oracle_sr_e5m2(C.c_float(float(x)), int(r16) & 0xFFFFFFFF))


def block_r16_pair(seed: int, stream_id: int, blk: int) -> Tuple[int, int]:
    r = np.zeros(2, dtype=np.uint32)
    lib().oracle_block_r16_pair(int(seed), int(stream_id), int(blk), _p(r))
    return int(r[0]), int(r[1])


def prune_2of4_q8(g: np.ndarray, seed: int = 0, stream_id: int = 0, mode: int = 0, scale: float = 1.0):
    """g: [T, O] float32 or uint16 (bf16 bits), T % 32 == 0.  Returns (vals8 [T/32, O, 16], meta32 [T/32, O])."""
    g = np.ascontiguousarray(g)
    T, O = g.shape
    vals8 = np.zeros((T // 32, O, 16), dtype=np.uint8)
    meta32 = np.zeros((T // 32, O), dtype=np.uint32)
    rc = lib().oracle_prune_2of4_q8(_p(g), T, O, O, _dt(g), int(seed), int(stream_id), int(mode),
                                    C.c_float(float(scale)), _p(vals8), _p(meta32))
    if rc != 0:
        raise ValueError("oracle_prune_2of4_q8: bad shape or mode")
    return vals8, meta32


def prune_1of2_q8(g: np.ndarray, seed: int = 0, stream_id: int = 0, scale: float = 1.0):
    """MVUE 1:2 with e5m2 output.  g: [T, O] float32 or uint16 (bf16 bits), T % 32 == 0.  Returns (vals8, meta32)."""
    g = np.ascontiguousarray(g)
    T, O = g.shape
    vals8 = np.zeros((T // 32, O, 16), dtype=np.uint8)
    meta32 = np.zeros((T // 32, O), dtype=np.uint32)
    rc = lib().oracle_prune_1of2_q8(_p(g), T, O, O, _dt(g), int(seed), int(stream_id), C.c_float(float(scale)),
                                    _p(vals8), _p(meta32))
    if rc != 0:
        raise ValueError("oracle_prune_1of2_q8: bad shape")
    return vals8, meta32


def nm_decompress_q8(vals8: np.ndarray, meta32: np.ndarray) -> np.ndarray:
    G, O = meta32.shape
    dense = np.zeros((G * 32, O), dtype=np.float64)
    lib().oracle_nm_decompress_q8(_p(np.ascontiguousarray(vals8)), _p(np.ascontiguousarray(meta32)), G * 32, O, _p(dense))
    return dense


def update_gemm_q8(vals8: np.ndarray, meta32: np.ndarray, h8: np.ndarray, alpha: float = 1.0,
                   oi: Optional[np.ndarray] = None):
    """h8: [T, I] uint8 (e4m3 codes).  Returns (dW, absdW) as float64: [O, I], or [n] for the entries oi [n, 2]."""
    G, O = meta32.shape
    h8 = np.ascontiguousarray(h8)
    T, I = h8.shape
    assert T == G * 32
    if oi is None:
        n, shape, oip = O * I, (O, I), None
    else:
        oi = np.ascontiguousarray(oi, dtype=np.int64)
        n, shape, oip = oi.shape[0], (oi.shape[0],), _p(oi)
    out = np.zeros(shape, dtype=np.float64)
    out_abs = np.zeros(shape, dtype=np.float64)
    lib().oracle_update_gemm_q8(_p(np.ascontiguousarray(vals8)), _p(np.ascontiguousarray(meta32)), _p(h8), I, T, O, I,
                                float(alpha), oip, n, _p(out), _p(out_abs))
    return out, out_abs


def update_gemm_shifted(vals: np.ndarray, meta: np.ndarray, x_full: np.ndarray, margin: int, shifts):
    """x_full: [margin + T + margin, C] (row 0 of the grid at index `margin`); shifts: one row shift per kernel tap.
    Returns (dW, absdW) as float64 [O, len(shifts)*C]."""
    G, O = meta.shape
    T = G * 16
    x_full = np.ascontiguousarray(x_full)
    assert x_full.shape[0] == T + 2 * margin and max(abs(int(v)) for v in shifts) <= margin
    Cc = x_full.shape[1]
    sh = np.ascontiguousarray(shifts, dtype=np.int64)
    dW = np.zeros((O, len(sh) * Cc), dtype=np.float64)
    absdW = np.zeros_like(dW)
    xp = C.c_void_p(x_full.ctypes.data + margin * Cc * x_full.itemsize)
    lib().oracle_update_gemm_shifted(_p(np.ascontiguousarray(vals)), _p(np.ascontiguousarray(meta)), xp, Cc, Cc, _p(sh), len(sh),
                                     T, O, _dt(x_full), _p(dW), _p(absdW))
    return dW, absdW


def update_gemm_q8_shifted(vals8: np.ndarray, meta32: np.ndarray, x8_full: np.ndarray, margin: int, shifts, alpha: float = 1.0):
    """x8_full: [margin + T + margin, C] uint8 e4m3 codes (row 0 of the grid at index `margin`).  Returns (dW, absdW) float64."""
    G, O = meta32.shape
    T = G * 32
    x8_full = np.ascontiguousarray(x8_full)
    assert x8_full.dtype == np.uint8 and x8_full.shape[0] == T + 2 * margin and max(abs(int(v)) for v in shifts) <= margin
    Cc = x8_full.shape[1]
    sh = np.ascontiguousarray(shifts, dtype=np.int64)
    dW = np.zeros((O, len(sh) * Cc), dtype=np.float64)
    absdW = np.zeros_like(dW)
    xp = C.c_void_p(x8_full.ctypes.data + margin * Cc)
    lib().oracle_update_gemm_q8_shifted(_p(np.ascontiguousarray(vals8)), _p(np.ascontiguousarray(meta32)), xp, Cc, Cc, _p(sh), len(sh),
                                        T, O, float(alpha), _p(dW), _p(absdW))
    return dW, absdW


# ---- Greedy N:M (the comparison method of the paper's tables): keep the n largest magnitudes, unchanged

def select_greedy(x, n: int):
    xa = np.ascontiguousarray(x, dtype=np.float32)
    pos = np.zeros(n, dtype=np.int32)
    lib().oracle_select_greedy(_p(xa), len(xa), n, _p(pos))
    return [int(v) for v in pos]


def prune_greedy(g: np.ndarray, n: int, m: int, want_dense: bool = False):
    T, O = g.shape
    ld = g.strides[0] // g.itemsize
    vals = np.zeros((T // 16, O, 8), dtype=g.dtype)
    meta = np.zeros((T // 16, O), dtype=np.uint16)
    dense = np.zeros((T, O), dtype=g.dtype) if want_dense else None
    if lib().oracle_prune_greedy(_p(g), T, O, ld, _dt(g), n, m, _p(vals), _p(meta), _p(dense), O) != 0:
        raise ValueError("oracle: bad shape or (n, m)")
    return vals, meta, dense


# ---- approx-MVUE 4:8: four magnitude-proportional draws out of eight; vals[T/16, O, 8] + meta32[T/16, O] (uint32:
# octet b of the group in bits [16b, 16b+12), 3 bits per kept position)

def block_u24_quad(seed: int, stream_id: int, blk: int):
    u = np.zeros(4, dtype=np.uint32)
    lib().oracle_block_u24_quad(seed, stream_id, blk, _p(u))
    return [int(v) for v in u]


def draw8(m, eps: float, taken: int = 0) -> int:
    ma = np.ascontiguousarray(m, dtype=np.float32)
    return int(lib().oracle_draw8(_p(ma), C.c_float(eps), taken))


def inclusion_4of8(m) -> np.ndarray:
    ma = np.ascontiguousarray(m, dtype=np.float32)
    p = np.zeros(8, dtype=np.float32)
    lib().oracle_inclusion_4of8(_p(ma), _p(p))
    return p


def select_4of8_approx(x, eps):
    xa = np.ascontiguousarray(x, dtype=np.float32)
    ea = np.ascontiguousarray(eps, dtype=np.float32)
    pos = np.zeros(4, dtype=np.int32)
    val = np.zeros(4, dtype=np.float32)
    lib().oracle_select_4of8_approx(_p(xa), _p(ea), _p(pos), _p(val))
    return [int(v) for v in pos], val


def enumerate_draw8(x, taken: int = 0) -> np.ndarray:
    """How often each position is drawn over all 2^24 uniforms, given the bit mask of positions already drawn."""
    xa = np.ascontiguousarray(x, dtype=np.float32)
    counts = np.zeros(8, dtype=np.uint64)
    lib().oracle_enumerate_draw8(_p(xa), taken, _p(counts))
    return counts


def prune_4of8_approx(g: np.ndarray, seed: int = 0, stream_id: int = 0, want_dense: bool = False):
    T, O = g.shape
    ld = g.strides[0] // g.itemsize
    vals = np.zeros((T // 16, O, 8), dtype=g.dtype)
    meta32 = np.zeros((T // 16, O), dtype=np.uint32)
    dense = np.zeros((T, O), dtype=g.dtype) if want_dense else None
    if lib().oracle_prune_4of8_approx(_p(g), T, O, ld, _dt(g), seed, stream_id, _p(vals), _p(meta32), _p(dense), O) != 0:
        raise ValueError("oracle: shape not representable (T must be a multiple of 16)")
    return vals, meta32, dense


def nm_decompress_4of8(vals: np.ndarray, meta32: np.ndarray) -> np.ndarray:
    G, O, _ = vals.shape
    dense = np.zeros((G * 16, O), dtype=vals.dtype)
    lib().oracle_nm_decompress_4of8(_p(vals), _p(meta32), G * 16, O, _dt(vals), _p(dense), O)
    return dense


# ---- per-tensor power-of-two scale and the activations' e4m3 cast of the 8-bit path

def pow2_scale(t: np.ndarray, top: float) -> float:
    R, Cc = t.shape
    return float(lib().oracle_pow2_scale(_p(t), R, Cc, t.strides[0] // t.itemsize, _dt(t), C.c_float(top)))


def e4m3_rne(x: float) -> int:
    return int(lib().oracle_e4m3_rne(C.c_float(x)))


def cast_e4m3(h: np.ndarray, scale: float) -> np.ndarray:
    R, Cc = h.shape
    h8 = np.zeros((R, Cc), dtype=np.uint8)
    lib().oracle_cast_e4m3(_p(h), R, Cc, h.strides[0] // h.itemsize, _dt(h), C.c_float(scale), _p(h8), Cc)
    return h8


# ---- the producer of the neural gradient: g = u * d elementwise (eq. (2): d = f'(z), u = W^T g_next), rounded to the dtype

def act_backward(u: np.ndarray, d: np.ndarray) -> np.ndarray:
    assert u.shape == d.shape and u.dtype == d.dtype
    T, O = u.shape
    g = np.zeros((T, O), dtype=u.dtype)
    lib().oracle_act_backward(_p(u), u.strides[0] // u.itemsize, _p(d), d.strides[0] // d.itemsize, T, O, _dt(u), _p(g), O)
    return g

"""Thin Python binding of libnm_mvue (the C ABI declared in include/nm_mvue.h).

Argument marshalling only: torch supplies device memory and the current HIP stream, every
step of the path runs in the library's kernels.  There is no fallback: if the shared library
is missing, or a call returns an error status, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libnm_mvue.so")

NM_F32, NM_BF16, NM_F32_BF16X3 = 0, 1, 2
_lib = None


class NmError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"nm_status {status}: {message}")
        self.status = status


def load():
    """Load libnm_mvue.so (built in-tree by ``python -m paper_2203_10991_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built: run `python -m paper_2203_10991_amd.build` (needs hipcc)")
    lib = C.CDLL(LIB_PATH)
    vp, i64, u64, u32, i32, f32, sz = C.c_void_p, C.c_int64, C.c_uint64, C.c_uint32, C.c_int, C.c_float, C.c_size_t
    lib.mvue_prune_1of2.argtypes = [vp, i64, i64, i64, i32, u64, u32, vp, vp, vp, i64, vp]
    lib.mvue_prune_2of4.argtypes = [vp, i64, i64, i64, i32, u64, u32, i32, vp, vp, vp, i64, vp]
    lib.mvue_prune_1of4.argtypes = [vp, i64, i64, i64, i32, u64, u32, vp, vp, vp, i64, vp]
    lib.mvue_prune_1of4.restype = i32
    lib.mvue_prune_2of4_producer.argtypes = [vp, i64, vp, i64, i64, i64, i32, u64, u32, i32, vp, i64, vp, vp, vp]
    lib.mvue_prune_2of4_producer.restype = i32
    lib.mvue_prune_1of2_producer.argtypes = [vp, i64, vp, i64, i64, i64, i32, u64, u32, vp, i64, vp, vp, vp]
    lib.mvue_prune_1of2_producer.restype = i32
    lib.mvue_prune_4of8_approx.argtypes = [vp, i64, i64, i64, i32, u64, u32, vp, vp, vp, i64, vp]
    lib.mvue_prune_4of8_approx.restype = i32
    lib.nm_prune_greedy.argtypes = [vp, i64, i64, i64, i32, i32, i32, vp, vp, vp, i64, vp]
    lib.nm_prune_greedy.restype = i32
    lib.nm_rw_mix_probe.argtypes = [vp, vp, i64, vp]
    lib.nm_rw_mix_probe.restype = i32
    lib.mvue_prune_2of4_t.argtypes = [vp, i64, i64, i64, i32, u64, u32, i32, vp, vp, vp]
    lib.mvue_prune_2of4_t.restype = i32
    lib.mvue_prune_1of2_t.argtypes = [vp, i64, i64, i64, i32, u64, u32, vp, vp, vp]
    lib.mvue_prune_1of2_t.restype = i32
    lib.nm_compress.argtypes = [vp, i64, i64, i64, i32, i32, i32, vp, vp, vp, vp]
    lib.nm_update_gemm.argtypes = [vp, vp, vp, i64, vp, i64, i64, i64, i64, i32, f32, vp, sz, vp]
    lib.nm_update_gemm_workspace.argtypes = [i64, i64, i64, i32]
    lib.nm_update_gemm_static.argtypes = [vp, vp, vp, i64, vp, i64, i64, i64, i64, i32, f32, vp]
    lib.nm_update_gemm_static.restype = i32
    lib.nm_update_gemm_static_max.argtypes = []
    lib.nm_update_gemm_static_max.restype = sz
    lib.nm_update_gemm_shifted.argtypes = [vp, vp, vp, i64, i64, vp, i32, vp, i64, i64, i64, i32, f32, vp, sz, vp]
    lib.nm_update_gemm_shifted.restype = i32
    lib.nm_update_gemm_shifted_workspace.argtypes = [i64, i64, i64, i32]
    lib.nm_update_gemm_shifted_workspace.restype = sz
    lib.nm_update_gemm_q8_shifted.argtypes = [vp, vp, vp, i64, i64, vp, i32, vp, i64, i64, i64, f32, f32, vp, sz, vp]
    lib.nm_update_gemm_q8_shifted.restype = i32
    lib.nm_update_gemm_q8_shifted_workspace.argtypes = [i64, i64, i64, i32]
    lib.nm_update_gemm_q8_shifted_workspace.restype = sz
    lib.mvue_prune_2of4_q8.argtypes = [vp, i64, i64, i64, i32, u64, u32, i32, f32, vp, vp, vp]
    lib.mvue_prune_1of2_q8.argtypes = [vp, i64, i64, i64, i32, u64, u32, f32, vp, vp, vp]
    lib.mvue_prune_1of2_q8.restype = i32
    lib.nm_update_gemm_q8.argtypes = [vp, vp, vp, i64, vp, i64, i64, i64, i64, f32, f32, vp, sz, vp]
    lib.nm_update_gemm_q8_workspace.argtypes = [i64, i64, i64]
    lib.nm_q8_scale.argtypes = [vp, i64, i64, i64, i32, f32, vp, vp]
    lib.nm_q8_scale.restype = i32
    lib.nm_cast_e4m3.argtypes = [vp, i64, i64, i64, i32, vp, vp, i64, vp]
    lib.nm_cast_e4m3.restype = i32
    lib.mvue_prune_2of4_q8_ds.argtypes = [vp, i64, i64, i64, i32, u64, u32, i32, vp, vp, vp, vp]
    lib.mvue_prune_2of4_q8_ds.restype = i32
    lib.mvue_prune_1of2_q8_ds.argtypes = [vp, i64, i64, i64, i32, u64, u32, vp, vp, vp, vp]
    lib.mvue_prune_1of2_q8_ds.restype = i32
    lib.mvue_prune_2of4_q8_t.argtypes = [vp, i64, i64, i64, i32, u64, u32, i32, f32, vp, vp, vp, vp]
    lib.mvue_prune_2of4_q8_t.restype = i32
    lib.mvue_prune_1of2_q8_t.argtypes = [vp, i64, i64, i64, i32, u64, u32, f32, vp, vp, vp, vp]
    lib.mvue_prune_1of2_q8_t.restype = i32
    lib.nm_update_gemm_q8_ds.argtypes = [vp, vp, vp, i64, vp, i64, i64, i64, i64, vp, vp, f32, vp, sz, vp]
    lib.nm_update_gemm_q8_ds.restype = i32
    lib.nm_update_gemm_q8_shifted_ds.argtypes = [vp, vp, vp, i64, i64, vp, i32, vp, i64, i64, i64, vp, vp, f32, vp, sz, vp]
    lib.nm_update_gemm_q8_shifted_ds.restype = i32
    for f in (lib.mvue_prune_1of2, lib.mvue_prune_2of4, lib.nm_compress, lib.nm_update_gemm, lib.mvue_prune_2of4_q8,
              lib.nm_update_gemm_q8):
        f.restype = i32
    lib.nm_update_gemm_workspace.restype = sz
    lib.nm_update_gemm_q8_workspace.restype = sz
    lib.nm_last_error.restype = C.c_char_p
    lib.nm_version.restype = C.c_char_p
    _lib = lib
    return lib


def _check(rc: int):
    if rc != 0:
        raise NmError(rc, load().nm_last_error().decode())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return NM_F32
    if t.dtype == torch.bfloat16:
        return NM_BF16
    raise TypeError(f"nm_mvue tensors are float32 or bfloat16, got {t.dtype}")


def _stream(t: torch.Tensor) -> int:
    return torch.cuda.current_stream(t.device).cuda_stream


def _rowmajor(t: torch.Tensor, what: str) -> int:
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError(f"{what} must be a 2-D tensor with unit column stride")
    return t.stride(0) if t.shape[0] > 1 else max(t.shape[1], t.stride(0))


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def alloc_compressed(T: int, O: int, dtype: torch.dtype, device) -> Tuple[torch.Tensor, torch.Tensor]:
    """Buffers of the group format: vals[T/16, O, 8] and meta[T/16, O] (int16 holds the uint16 words)."""
    return (torch.empty((T // 16, O, 8), dtype=dtype, device=device),
            torch.empty((T // 16, O), dtype=torch.int16, device=device))


def _prune(which: str, g, seed, stream_id, mode, vals, meta, dense_out, want_dense):
    lib = load()
    if not g.is_cuda:
        raise ValueError("g must live on the GPU")
    T, O = g.shape
    ldg = _rowmajor(g, "g")
    if vals is None or meta is None:
        vals, meta = alloc_compressed(T - T % 16, O, g.dtype, g.device)
    if dense_out is None and want_dense:
        dense_out = torch.empty((T, O), dtype=g.dtype, device=g.device)
    ldd = _rowmajor(dense_out, "dense_out") if dense_out is not None else 0
    if which == "1of4":
        rc = lib.mvue_prune_1of4(_ptr(g), T, O, ldg, _dtype_code(g), seed, stream_id, _ptr(vals), _ptr(meta),
                                 _ptr(dense_out), ldd, _stream(g))
    elif which == "1of2":
        rc = lib.mvue_prune_1of2(_ptr(g), T, O, ldg, _dtype_code(g), seed, stream_id, _ptr(vals), _ptr(meta),
                                 _ptr(dense_out), ldd, _stream(g))
    else:
        rc = lib.mvue_prune_2of4(_ptr(g), T, O, ldg, _dtype_code(g), seed, stream_id, mode, _ptr(vals), _ptr(meta),
                                 _ptr(dense_out), ldd, _stream(g))
    _check(rc)
    return vals, meta, dense_out


def mvue_prune_1of2(g: torch.Tensor, seed: int = 0, stream_id: int = 0, vals=None, meta=None, dense_out=None,
                    want_dense: bool = False):
    """MVUE 1:2 prune + compress of g[T x O] along T.  Returns (vals, meta, dense_out or None)."""
    return _prune("1of2", g, seed, stream_id, 0, vals, meta, dense_out, want_dense)


def mvue_prune_1of4(g: torch.Tensor, seed: int = 0, stream_id: int = 0, vals=None, meta=None, dense_out=None,
                    want_dense: bool = False):
    """MVUE 1:4 prune of g[T x O] along T, stored in the 2:4 group format.  Returns (vals, meta, dense_out or None)."""
    return _prune("1of4", g, seed, stream_id, 0, vals, meta, dense_out, want_dense)


def mvue_prune_2of4(g: torch.Tensor, seed: int = 0, stream_id: int = 0, mode: int = 0, vals=None, meta=None,
                    dense_out=None, want_dense: bool = False):
    """Optimal MVUE 2:4 prune + compress of g[T x O] along T.  Returns (vals, meta, dense_out or None)."""
    return _prune("2of4", g, seed, stream_id, mode, vals, meta, dense_out, want_dense)


def mvue_prune_producer(u: torch.Tensor, d: torch.Tensor, nm: str = "2:4", seed: int = 0, stream_id: int = 0, mode: int = 0,
                        g_out=None, vals=None, meta=None):
    """g = u * d (eq. (2): d = f'(z), u = W^T g_next) written dense, and its MVUE prune + compress, in one pass.
    Returns (g_out, vals, meta)."""
    lib = load()
    if not (u.is_cuda and d.is_cuda) or u.shape != d.shape or u.dtype != d.dtype:
        raise ValueError("u and d must be GPU tensors of one shape and dtype")
    T, O = u.shape
    if g_out is None:
        g_out = torch.empty((T, O), dtype=u.dtype, device=u.device)
    if vals is None or meta is None:
        vals, meta = alloc_compressed(T - T % 16, O, u.dtype, u.device)
    if nm == "1:2":
        rc = lib.mvue_prune_1of2_producer(_ptr(u), _rowmajor(u, "u"), _ptr(d), _rowmajor(d, "d"), T, O, _dtype_code(u), seed, stream_id,
                                          _ptr(g_out), _rowmajor(g_out, "g_out"), _ptr(vals), _ptr(meta), _stream(u))
    else:
        rc = lib.mvue_prune_2of4_producer(_ptr(u), _rowmajor(u, "u"), _ptr(d), _rowmajor(d, "d"), T, O, _dtype_code(u), seed, stream_id,
                                          mode, _ptr(g_out), _rowmajor(g_out, "g_out"), _ptr(vals), _ptr(meta), _stream(u))
    _check(rc)
    return g_out, vals, meta


def mvue_prune_4of8_approx(g: torch.Tensor, seed: int = 0, stream_id: int = 0, vals=None, meta32=None, dense_out=None,
                           want_dense: bool = False):
    """approx-MVUE 4:8 prune + compress of g[T x O] along T.  Returns (vals[T/16, O, 8], meta32[T/16, O] int32, dense_out or None)."""
    lib = load()
    if not g.is_cuda:
        raise ValueError("g must live on the GPU")
    T, O = g.shape
    ldg = _rowmajor(g, "g")
    if vals is None or meta32 is None:
        vals = torch.empty(((T - T % 16) // 16, O, 8), dtype=g.dtype, device=g.device)
        meta32 = torch.empty(((T - T % 16) // 16, O), dtype=torch.int32, device=g.device)
    if dense_out is None and want_dense:
        dense_out = torch.empty((T, O), dtype=g.dtype, device=g.device)
    ldd = _rowmajor(dense_out, "dense_out") if dense_out is not None else 0
    _check(lib.mvue_prune_4of8_approx(_ptr(g), T, O, ldg, _dtype_code(g), seed, stream_id, _ptr(vals), _ptr(meta32),
                                      _ptr(dense_out), ldd, _stream(g)))
    return vals, meta32, dense_out


def nm_prune_greedy(g: torch.Tensor, n: int, m: int, vals=None, meta=None, dense_out=None, want_dense: bool = False):
    """Greedy n:m prune + compress (keep the n largest magnitudes of every block along T, unchanged): the paper's
    biased baseline.  Returns (vals, meta, dense_out or None)."""
    lib = load()
    if not g.is_cuda:
        raise ValueError("g must live on the GPU")
    T, O = g.shape
    ldg = _rowmajor(g, "g")
    if vals is None or meta is None:
        vals, meta = alloc_compressed(T - T % 16, O, g.dtype, g.device)
    if dense_out is None and want_dense:
        dense_out = torch.empty((T, O), dtype=g.dtype, device=g.device)
    ldd = _rowmajor(dense_out, "dense_out") if dense_out is not None else 0
    _check(lib.nm_prune_greedy(_ptr(g), T, O, ldg, _dtype_code(g), n, m, _ptr(vals), _ptr(meta), _ptr(dense_out), ldd, _stream(g)))
    return vals, meta, dense_out


def _prune_transposed(gT: torch.Tensor, vals, meta):
    if not gT.is_cuda:
        raise ValueError("gT must live on the GPU")
    O, T = gT.shape
    ldt = _rowmajor(gT, "gT")
    if vals is None or meta is None:
        vals, meta = alloc_compressed(T - T % 16, O, gT.dtype, gT.device)
    return T, O, ldt, vals, meta


def mvue_prune_2of4_t(gT: torch.Tensor, seed: int = 0, stream_id: int = 0, mode: int = 0, vals=None, meta=None):
    """MVUE 2:4 prune + compress of a gradient stored transposed, gT[O x T] (tokens contiguous).  Returns (vals, meta)."""
    lib = load()
    T, O, ldt, vals, meta = _prune_transposed(gT, vals, meta)
    _check(lib.mvue_prune_2of4_t(_ptr(gT), T, O, ldt, _dtype_code(gT), seed, stream_id, mode, _ptr(vals), _ptr(meta), _stream(gT)))
    return vals, meta


def mvue_prune_1of2_t(gT: torch.Tensor, seed: int = 0, stream_id: int = 0, vals=None, meta=None):
    """MVUE 1:2 prune + compress of a gradient stored transposed, gT[O x T] (tokens contiguous).  Returns (vals, meta)."""
    lib = load()
    T, O, ldt, vals, meta = _prune_transposed(gT, vals, meta)
    _check(lib.mvue_prune_1of2_t(_ptr(gT), T, O, ldt, _dtype_code(gT), seed, stream_id, _ptr(vals), _ptr(meta), _stream(gT)))
    return vals, meta


def nm_compress(dense: torch.Tensor, n: int, m: int, vals=None, meta=None, bad_blocks: Optional[torch.Tensor] = None):
    """Compress an n:m-sparse dense tensor into the group format.  Returns (vals, meta)."""
    lib = load()
    T, O = dense.shape
    ld = _rowmajor(dense, "dense")
    if vals is None or meta is None:
        vals, meta = alloc_compressed(T - T % 16, O, dense.dtype, dense.device)
    _check(lib.nm_compress(_ptr(dense), T, O, ld, _dtype_code(dense), n, m, _ptr(vals), _ptr(meta),
                           _ptr(bad_blocks), _stream(dense)))
    return vals, meta


def _gemm_mode(dtype: torch.dtype, f32_as_bf16x3: bool) -> int:
    if dtype == torch.float32:
        return NM_F32_BF16X3 if f32_as_bf16x3 else NM_F32
    return NM_BF16


def nm_update_gemm_workspace(T: int, O: int, I: int, dtype: torch.dtype, f32_as_bf16x3: bool = False) -> int:
    return int(load().nm_update_gemm_workspace(T, O, I, _gemm_mode(dtype, f32_as_bf16x3)))


def nm_update_gemm(vals: torch.Tensor, meta: torch.Tensor, h: torch.Tensor, dW: Optional[torch.Tensor] = None,
                   beta: float = 0.0, workspace: Optional[torch.Tensor] = None, f32_as_bf16x3: bool = False) -> torch.Tensor:
    """dW[O x I] = beta*dW + decompress(vals, meta)^T h  (binary32 output).

    f32_as_bf16x3 (binary32 tensors only): multiply through three bf16 terms per value on the sparse 16-bit path."""
    lib = load()
    G, O, _ = vals.shape
    T, I = h.shape
    if T != G * 16:
        raise ValueError(f"h has {T} rows, the compressed operand covers {G * 16}")
    ldh = _rowmajor(h, "h")
    if dW is None:
        dW = torch.empty((O, I), dtype=torch.float32, device=h.device)
    lddw = _rowmajor(dW, "dW")
    if vals.dtype != h.dtype:
        raise TypeError("vals and h must have the same dtype")
    need = nm_update_gemm_workspace(T, O, I, h.dtype, f32_as_bf16x3)
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device=h.device)
    wbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib.nm_update_gemm(_ptr(vals), _ptr(meta), _ptr(h), ldh, _ptr(dW), lddw, T, O, I, _gemm_mode(h.dtype, f32_as_bf16x3),
                              float(beta), _ptr(workspace), wbytes, _stream(h)))
    return dW


def nm_update_gemm_static(vals: torch.Tensor, meta: torch.Tensor, h: torch.Tensor, dW: torch.Tensor, beta: float = 0.0,
                          f32_as_bf16x3: bool = False) -> torch.Tensor:
    """nm_update_gemm without a workspace: split-K partial sums go to the library's static device array.  The caller
    passes dW; nothing is allocated."""
    lib = load()
    G, O, _ = vals.shape
    T, I = h.shape
    if T != G * 16:
        raise ValueError(f"h has {T} rows, the compressed operand covers {G * 16}")
    if vals.dtype != h.dtype:
        raise TypeError("vals and h must have the same dtype")
    _check(lib.nm_update_gemm_static(_ptr(vals), _ptr(meta), _ptr(h), _rowmajor(h, "h"), _ptr(dW), _rowmajor(dW, "dW"), T, O, I,
                                     _gemm_mode(h.dtype, f32_as_bf16x3), float(beta), _stream(h)))
    return dW


def nm_update_gemm_static_max() -> int:
    return int(load().nm_update_gemm_static_max())


# ---- 8-bit neural gradients (e5m2, stochastic rounding) on top of 2:4 sparsity

def alloc_compressed_q8(T: int, O: int, device) -> Tuple[torch.Tensor, torch.Tensor]:
    """Buffers of the 8-bit group format: vals8[T/32, O, 16] (uint8 e5m2 codes) and meta32[T/32, O] (int32 holds the words)."""
    return (torch.empty((T // 32, O, 16), dtype=torch.uint8, device=device),
            torch.empty((T // 32, O), dtype=torch.int32, device=device))


def mvue_prune_2of4_q8(g: torch.Tensor, seed: int = 0, stream_id: int = 0, mode: int = 0, scale=1.0,
                       vals8=None, meta32=None):
    """MVUE 2:4 prune of g[T x O] along T with kept values scaled and rounded stochastically to e5m2.  Returns (vals8, meta32)."""
    lib = load()
    if not g.is_cuda:
        raise ValueError("g must live on the GPU")
    T, O = g.shape
    ldg = _rowmajor(g, "g")
    if vals8 is None or meta32 is None:
        vals8, meta32 = alloc_compressed_q8(T - T % 32, O, g.device)
    if isinstance(scale, torch.Tensor):          # a scale record in device memory (nm_q8_scale)
        _check(lib.mvue_prune_2of4_q8_ds(_ptr(g), T, O, ldg, _dtype_code(g), seed, stream_id, mode, _ptr(scale),
                                         _ptr(vals8), _ptr(meta32), _stream(g)))
    else:
        _check(lib.mvue_prune_2of4_q8(_ptr(g), T, O, ldg, _dtype_code(g), seed, stream_id, mode, float(scale),
                                      _ptr(vals8), _ptr(meta32), _stream(g)))
    return vals8, meta32


def mvue_prune_1of2_q8(g: torch.Tensor, seed: int = 0, stream_id: int = 0, scale=1.0, vals8=None, meta32=None):
    """MVUE 1:2 prune of g[T x O] along T with kept values scaled and rounded stochastically to e5m2.  Returns (vals8, meta32)."""
    lib = load()
    if not g.is_cuda:
        raise ValueError("g must live on the GPU")
    T, O = g.shape
    ldg = _rowmajor(g, "g")
    if vals8 is None or meta32 is None:
        vals8, meta32 = alloc_compressed_q8(T - T % 32, O, g.device)
    if isinstance(scale, torch.Tensor):
        _check(lib.mvue_prune_1of2_q8_ds(_ptr(g), T, O, ldg, _dtype_code(g), seed, stream_id, _ptr(scale),
                                         _ptr(vals8), _ptr(meta32), _stream(g)))
    else:
        _check(lib.mvue_prune_1of2_q8(_ptr(g), T, O, ldg, _dtype_code(g), seed, stream_id, float(scale),
                                      _ptr(vals8), _ptr(meta32), _stream(g)))
    return vals8, meta32


def _prune_q8_transposed(gT: torch.Tensor, vals8, meta32, scale):
    if not gT.is_cuda:
        raise ValueError("gT must live on the GPU")
    O, T = gT.shape
    ldt = _rowmajor(gT, "gT")
    if vals8 is None or meta32 is None:
        vals8, meta32 = alloc_compressed_q8(T - T % 32, O, gT.device)
    rec = scale if isinstance(scale, torch.Tensor) else None          # a scale record in device memory (nm_q8_scale)
    return O, T, ldt, vals8, meta32, (1.0 if rec is not None else float(scale)), rec


def mvue_prune_2of4_q8_t(gT: torch.Tensor, seed: int = 0, stream_id: int = 0, mode: int = 0, scale=1.0, vals8=None, meta32=None):
    """mvue_prune_2of4_q8 for a gradient stored transposed: gT is [O x T], tokens contiguous.  Returns (vals8, meta32), equal to
    mvue_prune_2of4_q8(gT.t().contiguous(), ...) bit for bit."""
    lib = load()
    O, T, ldt, vals8, meta32, s, rec = _prune_q8_transposed(gT, vals8, meta32, scale)
    _check(lib.mvue_prune_2of4_q8_t(_ptr(gT), T, O, ldt, _dtype_code(gT), seed, stream_id, mode, s, _ptr(rec), _ptr(vals8),
                                    _ptr(meta32), _stream(gT)))
    return vals8, meta32


def mvue_prune_1of2_q8_t(gT: torch.Tensor, seed: int = 0, stream_id: int = 0, scale=1.0, vals8=None, meta32=None):
    """mvue_prune_1of2_q8 for a gradient stored transposed (gT [O x T])."""
    lib = load()
    O, T, ldt, vals8, meta32, s, rec = _prune_q8_transposed(gT, vals8, meta32, scale)
    _check(lib.mvue_prune_1of2_q8_t(_ptr(gT), T, O, ldt, _dtype_code(gT), seed, stream_id, s, _ptr(rec), _ptr(vals8), _ptr(meta32),
                                    _stream(gT)))
    return vals8, meta32


def nm_update_gemm_q8_workspace(T: int, O: int, I: int) -> int:
    return int(load().nm_update_gemm_q8_workspace(T, O, I))


def nm_update_gemm_q8(vals8: torch.Tensor, meta32: torch.Tensor, h8: torch.Tensor, dW: Optional[torch.Tensor] = None,
                      alpha: float = 1.0, beta: float = 0.0, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """dW[O x I] = beta*dW + alpha * decompress(vals8, meta32)^T h8; h8 holds e4m3 codes (uint8 or float8_e4m3fn)."""
    lib = load()
    G, O, _ = vals8.shape
    T, I = h8.shape
    if T != G * 32:
        raise ValueError(f"h8 has {T} rows, the compressed operand covers {G * 32}")
    if h8.element_size() != 1:
        raise TypeError("h8 must be an 8-bit tensor of e4m3 codes")
    ldh = _rowmajor(h8, "h8")
    if dW is None:
        dW = torch.empty((O, I), dtype=torch.float32, device=h8.device)
    lddw = _rowmajor(dW, "dW")
    need = nm_update_gemm_q8_workspace(T, O, I)
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device=h8.device)
    wbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    if isinstance(alpha, tuple):                 # two scale records in device memory: alpha = rec_g[1] * rec_h[1]
        _check(lib.nm_update_gemm_q8_ds(_ptr(vals8), _ptr(meta32), _ptr(h8), ldh, _ptr(dW), lddw, T, O, I, _ptr(alpha[0]),
                                        _ptr(alpha[1]), float(beta), _ptr(workspace), wbytes, _stream(h8)))
    else:
        _check(lib.nm_update_gemm_q8(_ptr(vals8), _ptr(meta32), _ptr(h8), ldh, _ptr(dW), lddw, T, O, I, float(alpha),
                                     float(beta), _ptr(workspace), wbytes, _stream(h8)))
    return dW


def nm_q8_scale(t: torch.Tensor, top: float, rec: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Scale record (device float[4] = s, 1/s, bits of max|t|, 0) of a 2-D tensor: s the largest power of two with
    s * max|t| <= top.  Nothing returns to the host."""
    lib = load()
    R, Cc = t.shape
    if rec is None:
        rec = torch.empty(4, dtype=torch.float32, device=t.device)
    _check(lib.nm_q8_scale(_ptr(t), R, Cc, _rowmajor(t, "t"), _dtype_code(t), float(top), _ptr(rec), _stream(t)))
    return rec


def nm_cast_e4m3(h: torch.Tensor, rec: torch.Tensor, h8: Optional[torch.Tensor] = None) -> torch.Tensor:
    """h8 (uint8 e4m3 codes) = e4m3(h * rec[0]), round to nearest even."""
    lib = load()
    R, Cc = h.shape
    if h8 is None:
        h8 = torch.empty((R, Cc), dtype=torch.uint8, device=h.device)
    _check(lib.nm_cast_e4m3(_ptr(h), R, Cc, _rowmajor(h, "h"), _dtype_code(h), _ptr(rec), _ptr(h8), _rowmajor(h8, "h8"), _stream(h)))
    return h8


def nm_rw_mix_probe(src: torch.Tensor, dst: torch.Tensor, n_blocks: int) -> None:
    """Measurement aid: streams n_blocks * 64 KiB from src and writes n_blocks * 36 KiB to dst (the 16:9 read:write mix of
    the 16-bit prune + compress, contiguous 4 KiB instructions).  src, dst: contiguous device tensors of any dtype."""
    lib = load()
    if src.numel() * src.element_size() < n_blocks * 65536 or dst.numel() * dst.element_size() < n_blocks * 36864:
        raise ValueError("nm_rw_mix_probe: src needs 64 KiB and dst 36 KiB per block")
    _check(lib.nm_rw_mix_probe(_ptr(src), _ptr(dst), n_blocks, _stream(src)))


def nm_update_gemm_shifted(vals: torch.Tensor, meta: torch.Tensor, x_full: torch.Tensor, margin: int, shifts,
                           dW: Optional[torch.Tensor] = None, beta: float = 0.0,
                           workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """dW[O x n*C] = beta*dW + decompress(vals, meta)^T [x shifted by shifts[0] | x shifted by shifts[1] | ...].

    x_full is [margin + T + margin, C] (bf16): row 0 of the grid sits at index ``margin``; the margin rows hold zeros.
    """
    lib = load()
    G, O, _ = vals.shape
    T = G * 16
    if x_full.dim() != 2 or x_full.shape[0] != T + 2 * margin:
        raise ValueError(f"x_full must have {T + 2 * margin} rows (T = {T}, margin = {margin})")
    if max(abs(int(v)) for v in shifts) > margin:
        raise ValueError("a row shift exceeds the margin")
    ldx = _rowmajor(x_full, "x_full")
    Cb = x_full.shape[1]
    n = len(shifts)
    I = n * Cb
    if dW is None:
        dW = torch.empty((O, I), dtype=torch.float32, device=x_full.device)
    lddw = _rowmajor(dW, "dW")
    need = int(lib.nm_update_gemm_shifted_workspace(T, O, Cb, n))
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device=x_full.device)
    wbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    sh = (C.c_int64 * n)(*[int(v) for v in shifts])
    xp = x_full.data_ptr() + margin * ldx * x_full.element_size()
    _check(lib.nm_update_gemm_shifted(_ptr(vals), _ptr(meta), xp, ldx, Cb, sh, n, _ptr(dW), lddw, T, O,
                                      _dtype_code(x_full), float(beta), _ptr(workspace), wbytes, _stream(x_full)))
    return dW


def nm_update_gemm_q8_shifted(vals8: torch.Tensor, meta32: torch.Tensor, x8_full: torch.Tensor, margin: int, shifts,
                              dW: Optional[torch.Tensor] = None, alpha: float = 1.0, beta: float = 0.0,
                              workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """8-bit form of nm_update_gemm_shifted: x8_full is [margin + T + margin, C] e4m3 codes, margin rows zero."""
    lib = load()
    G, O, _ = vals8.shape
    T = G * 32
    if x8_full.dim() != 2 or x8_full.shape[0] != T + 2 * margin or x8_full.element_size() != 1:
        raise ValueError(f"x8_full must be an 8-bit tensor with {T + 2 * margin} rows (T = {T}, margin = {margin})")
    if max(abs(int(v)) for v in shifts) > margin:
        raise ValueError("a row shift exceeds the margin")
    ldx = _rowmajor(x8_full, "x8_full")
    Cb = x8_full.shape[1]
    n = len(shifts)
    if dW is None:
        dW = torch.empty((O, n * Cb), dtype=torch.float32, device=x8_full.device)
    lddw = _rowmajor(dW, "dW")
    need = int(lib.nm_update_gemm_q8_shifted_workspace(T, O, Cb, n))
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device=x8_full.device)
    wbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    sh = (C.c_int64 * n)(*[int(v) for v in shifts])
    xp = x8_full.data_ptr() + margin * ldx
    if isinstance(alpha, tuple):
        _check(lib.nm_update_gemm_q8_shifted_ds(_ptr(vals8), _ptr(meta32), xp, ldx, Cb, sh, n, _ptr(dW), lddw, T, O, _ptr(alpha[0]),
                                                _ptr(alpha[1]), float(beta), _ptr(workspace), wbytes, _stream(x8_full)))
    else:
        _check(lib.nm_update_gemm_q8_shifted(_ptr(vals8), _ptr(meta32), xp, ldx, Cb, sh, n, _ptr(dW), lddw, T, O, float(alpha),
                                             float(beta), _ptr(workspace), wbytes, _stream(x8_full)))
    return dW

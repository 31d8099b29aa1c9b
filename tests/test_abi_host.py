"""Host-side checks of the C ABI: the library loads, exports what the header declares, and
rejects bad arguments before touching a device (these run without a GPU; no compute call)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "nm_mvue.h")

NM_OK, NM_ERR_NULL, NM_ERR_SHAPE, NM_ERR_DTYPE, NM_ERR_ALIGN, NM_ERR_ALIAS, NM_ERR_WORKSPACE, NM_ERR_UNSUPPORTED = range(8)


@pytest.fixture(scope="module")
def lib():
    from paper_2203_10991_amd import api
    if not os.path.exists(api.LIB_PATH):
        from paper_2203_10991_amd import build
        build.build()
    return api.load()


def declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return re.findall(r"^\s*(?:int|size_t|const char \*)\s*(\w+)\s*\(", text, flags=re.M)


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert set(names) >= {"mvue_prune_1of2", "mvue_prune_2of4", "nm_compress", "nm_update_gemm",
                          "nm_update_gemm_workspace", "nm_last_error", "nm_version", "mvue_prune_2of4_q8", "mvue_prune_1of2_q8", "mvue_prune_1of4", "mvue_prune_2of4_t", "mvue_prune_1of2_t", "mvue_prune_2of4_q8_t", "mvue_prune_1of2_q8_t", "nm_update_gemm_shifted", "nm_update_gemm_shifted_workspace", "nm_update_gemm_q8_shifted",
                          "nm_update_gemm_q8_shifted_workspace",
                          "nm_update_gemm_q8", "nm_update_gemm_q8_workspace"}
    for n in names:
        assert hasattr(lib, n), n
    assert b"gfx950" in lib.nm_version()


P = 0x10000          # fake, aligned, never dereferenced: validation fails before any launch


def prune12(lib, g=P, T=32, O=16, ldg=16, dt=1, vals=P + 0x10000, meta=P + 0x20000, dense=None, ldd=0):
    return lib.mvue_prune_1of2(g, T, O, ldg, dt, 0, 0, vals, meta, dense, ldd, None)


def test_prune_argument_errors(lib):
    assert prune12(lib, T=30) == NM_ERR_SHAPE and b"multiple of 16" in lib.nm_last_error()
    assert prune12(lib, O=12) == NM_ERR_SHAPE
    assert prune12(lib, T=-16) == NM_ERR_SHAPE
    assert prune12(lib, ldg=8) == NM_ERR_SHAPE
    assert prune12(lib, dt=2) == NM_ERR_DTYPE
    assert prune12(lib, g=None) == NM_ERR_NULL
    assert prune12(lib, vals=None) == NM_ERR_NULL
    assert prune12(lib, meta=None) == NM_ERR_NULL
    assert prune12(lib, g=P + 2) == NM_ERR_ALIGN
    assert prune12(lib, ldg=20) == NM_ERR_ALIGN                 # 40-byte bf16 rows
    assert prune12(lib, vals=P) == NM_ERR_ALIAS                  # in place
    assert prune12(lib, vals=P + 0x20000) == NM_ERR_ALIAS        # vals == meta
    assert prune12(lib, dense=P + 0x10000, ldd=16) == NM_ERR_ALIAS
    assert prune12(lib, dense=P + 0x30000, ldd=8) == NM_ERR_SHAPE
    # empty problems are accepted and do nothing
    assert prune12(lib, T=0) == NM_OK and prune12(lib, O=0) == NM_OK
    assert lib.nm_last_error() == b""


def test_prune_2of4_modes(lib):
    call = lambda mode, **kw: lib.mvue_prune_2of4(P, kw.get("T", 32), 16, 16, 1, 0, 0, mode, P + 0x10000, P + 0x20000, None, 0, None)
    assert call(2) == NM_ERR_UNSUPPORTED and b"approx" in lib.nm_last_error()
    assert call(7) == NM_ERR_UNSUPPORTED and call(-1) == NM_ERR_UNSUPPORTED
    assert call(1, T=24) == NM_ERR_SHAPE
    assert call(0, T=24) == NM_ERR_SHAPE


def test_transposed_prune_argument_errors(lib):
    def call(gT=P, T=32, O=16, ldt=32, dt=1, mode=0, vals=P + 0x10000, meta=P + 0x20000):
        return lib.mvue_prune_2of4_t(gT, T, O, ldt, dt, 0, 0, mode, vals, meta, None)
    assert call(T=24) == NM_ERR_SHAPE and b"multiple of 16" in lib.nm_last_error()
    assert call(O=12) == NM_ERR_SHAPE
    assert call(ldt=16) == NM_ERR_SHAPE
    assert call(dt=3) == NM_ERR_DTYPE
    assert call(mode=2) == NM_ERR_UNSUPPORTED
    assert call(gT=None) == NM_ERR_NULL and call(vals=None) == NM_ERR_NULL and call(meta=None) == NM_ERR_NULL
    assert call(gT=P + 4) == NM_ERR_ALIGN
    assert call(ldt=36) == NM_ERR_ALIGN                           # 72-byte bf16 rows
    assert call(vals=P) == NM_ERR_ALIAS and call(meta=P + 0x10000) == NM_ERR_ALIAS
    assert call(T=0) == NM_OK and call(O=0) == NM_OK
    call12 = lambda T=32, O=16, ldt=32, vals=P + 0x10000: lib.mvue_prune_1of2_t(P, T, O, ldt, 1, 0, 0, vals, P + 0x20000, None)
    assert call12(T=8) == NM_ERR_SHAPE and b"mvue_prune_1of2_t" in lib.nm_last_error()
    assert call12(O=4) == NM_ERR_SHAPE and call12(ldt=24) == NM_ERR_SHAPE and call12(vals=None) == NM_ERR_NULL
    assert call12(T=0) == NM_OK


def test_compress_argument_errors(lib):
    call = lambda n, m, T=32: lib.nm_compress(P, T, 16, 16, 0, n, m, P + 0x10000, P + 0x20000, None, None)
    assert call(2, 3) == NM_ERR_UNSUPPORTED
    assert call(4, 8) == NM_ERR_UNSUPPORTED
    assert call(2, 4, T=8) == NM_ERR_SHAPE


def test_gemm_argument_errors(lib):
    def gemm(vals=P, meta=P + 0x10000, h=P + 0x20000, ldh=64, dW=P + 0x40000, lddw=64, T=64, O=32, I=64, dt=1, beta=0.0):
        return lib.nm_update_gemm(vals, meta, h, ldh, dW, lddw, T, O, I, dt, beta, None, 0, None)
    assert gemm(T=40) == NM_ERR_SHAPE
    assert gemm(O=30) == NM_ERR_SHAPE
    assert gemm(I=60) == NM_ERR_SHAPE
    assert gemm(ldh=32) == NM_ERR_SHAPE
    assert gemm(lddw=32) == NM_ERR_SHAPE
    assert gemm(dt=5) == NM_ERR_DTYPE
    assert gemm(beta=0.5) == NM_ERR_UNSUPPORTED
    assert gemm(dW=None) == NM_ERR_NULL
    assert gemm(h=None) == NM_ERR_NULL
    assert gemm(h=P + 0x20004) == NM_ERR_ALIGN
    assert gemm(dW=P + 0x20000) == NM_ERR_ALIAS
    assert gemm(O=0) == NM_OK
    # the kernels' 32-bit stage offsets bound O and ldh (checked before anything is launched)
    assert gemm(ldh=(1 << 21) + 8, dW=P + (1 << 40)) == NM_ERR_UNSUPPORTED and b"2^21" in lib.nm_last_error()
    assert gemm(O=(1 << 21) + 8, dW=P + (1 << 40)) == NM_ERR_UNSUPPORTED
    assert lib.nm_update_gemm_workspace(-1, 8, 8, 1) == 0
    # binary32 problems with few output tiles split the reduction axis as well
    assert lib.nm_update_gemm_workspace(1024, 1024, 1024, 0) == 8 * 1024 * 1024 * 4
    assert gemm(T=1024, O=1024, I=1024, ldh=1024, lddw=1024, dt=0, dW=P + (1 << 40)) == NM_ERR_WORKSPACE
    # mode 2 (binary32 tensors as three bf16 terms): six bf16 planes live in the workspace, so it is never optional
    need = lib.nm_update_gemm_workspace(64, 32, 64, 2)
    assert need >= 3 * (32 * 32 * 2) + 3 * (64 * 64 * 2)
    assert gemm(dt=2, ldh=64, dW=P + (1 << 40)) == NM_ERR_WORKSPACE
    assert lib.nm_update_gemm(P, P + 0x10000, P + 0x20000, 64, P + (1 << 40), 64, 64, 32, 64, 2, 0.0, P + 0x10000, need, None) == NM_ERR_ALIAS
    assert lib.nm_update_gemm_workspace(64, 32, 64, 3) == 0


def test_q8_argument_errors(lib):
    f32, sz = C.c_float, C.c_size_t
    lib.mvue_prune_2of4_q8.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_int, C.c_uint64, C.c_uint32, C.c_int,
                                       f32, C.c_void_p, C.c_void_p, C.c_void_p]

    def prune8(g=P, T=64, O=16, ldg=16, dt=1, mode=0, scale=1.0, vals=P + 0x10000, meta=P + 0x20000):
        return lib.mvue_prune_2of4_q8(g, T, O, ldg, dt, 0, 0, mode, scale, vals, meta, None)

    assert prune8(T=48) == NM_ERR_SHAPE and b"multiple of 32" in lib.nm_last_error()
    p12 = lambda T=64, O=16, scale=1.0, vals=P + 0x10000: lib.mvue_prune_1of2_q8(P, T, O, 16, 1, 0, 0, f32(scale), vals, P + 0x20000, None)
    assert p12(T=48) == NM_ERR_SHAPE and b"mvue_prune_1of2_q8" in lib.nm_last_error()
    assert p12(scale=-1.0) == NM_ERR_SHAPE and p12(vals=None) == NM_ERR_NULL and p12(vals=P) == NM_ERR_ALIAS and p12(T=0) == NM_OK
    assert prune8(O=12) == NM_ERR_SHAPE
    assert prune8(mode=2) == NM_ERR_UNSUPPORTED
    assert prune8(scale=0.0) == NM_ERR_SHAPE and prune8(scale=float("inf")) == NM_ERR_SHAPE and prune8(scale=float("nan")) == NM_ERR_SHAPE
    assert prune8(dt=3) == NM_ERR_DTYPE
    assert prune8(vals=None) == NM_ERR_NULL and prune8(meta=None) == NM_ERR_NULL and prune8(g=None) == NM_ERR_NULL
    assert prune8(vals=P + 8) == NM_ERR_ALIGN
    assert prune8(vals=P) == NM_ERR_ALIAS and prune8(meta=P + 0x10000) == NM_ERR_ALIAS
    assert prune8(T=0) == NM_OK and prune8(O=0, ldg=0) == NM_OK

    lib.nm_update_gemm_q8.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int64, C.c_int64,
                                      C.c_int64, f32, f32, C.c_void_p, sz, C.c_void_p]
    lib.nm_update_gemm_q8_workspace.argtypes = [C.c_int64] * 3
    lib.nm_update_gemm_q8_workspace.restype = sz

    def gemm8(vals=P, meta=P + 0x100000, h=P + 0x200000, ldh=64, dW=P + 0x300000, lddw=64, T=64, O=64, I=64, alpha=1.0, beta=0.0,
              ws=None, wsb=0):
        return lib.nm_update_gemm_q8(vals, meta, h, ldh, dW, lddw, T, O, I, alpha, beta, ws, wsb, None)

    assert gemm8(T=48) == NM_ERR_SHAPE
    assert gemm8(I=24, ldh=32) == NM_ERR_SHAPE and b"of 16" in lib.nm_last_error()
    assert gemm8(O=12) == NM_ERR_SHAPE
    assert gemm8(beta=0.5) == NM_ERR_UNSUPPORTED
    assert gemm8(dW=None) == NM_ERR_NULL and gemm8(h=None) == NM_ERR_NULL
    assert gemm8(ldh=48) == NM_ERR_SHAPE and gemm8(ldh=72) == NM_ERR_ALIGN
    assert gemm8(lddw=32) == NM_ERR_SHAPE
    assert gemm8(dW=P) == NM_ERR_ALIAS
    assert gemm8(O=(1 << 21) + 8) == NM_ERR_UNSUPPORTED
    # a problem with few tiles is split along T and needs the workspace it asks for
    need = lib.nm_update_gemm_q8_workspace(4096, 64, 256)
    assert need > 0 and need % (64 * 256 * 4) == 0
    assert gemm8(T=4096, I=256, ldh=256, lddw=256) == NM_ERR_WORKSPACE
    assert lib.nm_update_gemm_q8_workspace(32768, 28672, 8192) == 0
    assert gemm8(O=0) == NM_OK


def test_autograd_layers_have_no_cpu_fallback():
    import torch
    from paper_2203_10991_amd.autograd import NMConv2d, NMLinear
    layer = NMLinear(16, 8)
    x = torch.randn(16, 16, requires_grad=True)
    with pytest.raises(RuntimeError, match="GPU only"):
        layer(x).sum().backward()
    conv = NMConv2d(8, 8, 3, padding=1)
    with pytest.raises(RuntimeError, match="GPU only"):
        conv(torch.randn(2, 8, 4, 4)).sum().backward()
    with pytest.raises(ValueError):
        NMConv2d(8, 8, 3, groups=2)


def test_shifted_gemm_argument_errors(lib):
    i64 = C.c_int64
    lib.nm_update_gemm_shifted.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, i64, i64, C.c_void_p, C.c_int, C.c_void_p, i64, i64, i64,
                                           C.c_int, C.c_float, C.c_void_p, C.c_size_t, C.c_void_p]
    sh = (i64 * 9)(-11, -10, -9, -1, 0, 1, 9, 10, 11)

    def call(vals=P, meta=P + 0x100000, x=P + 0x200000, ldx=16, cb=16, shifts=sh, n=9, dW=P + 0x400000, lddw=144, T=64, O=64, dt=1,
             beta=0.0):
        return lib.nm_update_gemm_shifted(vals, meta, x, ldx, cb, shifts, n, dW, lddw, T, O, dt, beta, None, 0, None)

    assert call(dt=0) == NM_ERR_UNSUPPORTED and call(dt=5) == NM_ERR_DTYPE
    assert call(n=0) == NM_ERR_SHAPE and call(n=33) == NM_ERR_SHAPE
    assert call(shifts=None) == NM_ERR_NULL
    assert call(cb=12) == NM_ERR_SHAPE and call(T=40) == NM_ERR_SHAPE and call(O=12) == NM_ERR_SHAPE
    assert call(ldx=8) == NM_ERR_SHAPE and call(lddw=128) == NM_ERR_SHAPE
    assert call(x=None) == NM_ERR_NULL and call(dW=None) == NM_ERR_NULL
    assert call(ldx=20) == NM_ERR_ALIGN
    assert call(beta=2.0) == NM_ERR_UNSUPPORTED
    assert call(dW=P + 0x200000 - 64) == NM_ERR_ALIAS          # dW inside the margin rows of x
    big = (i64 * 1)(1 << 21)
    assert call(shifts=big, n=1, lddw=16) == NM_ERR_UNSUPPORTED
    assert call(O=0) == NM_OK
    # few rows, many tokens: split along T with its own plan, and the call insists on that much workspace
    lib.nm_update_gemm_shifted_workspace.argtypes = [i64, i64, i64, C.c_int]
    lib.nm_update_gemm_shifted_workspace.restype = C.c_size_t
    need = lib.nm_update_gemm_shifted_workspace(65536, 64, 64, 9)
    assert need > 0 and need % (64 * 576 * 4) == 0
    assert call(T=65536, cb=64, ldx=64, lddw=576, meta=P + 0x10000000, x=P + 0x20000000, dW=P + 0x40000000) == NM_ERR_WORKSPACE


def test_workspace_queries_over_random_shapes(lib):
    """The workspace a plan asks for is a whole number of partial dW slabs (or nothing), for every kernel family;
    a plan never asks for more slabs than there are token groups."""
    import random
    rnd = random.Random(5)
    for _ in range(400):
        T = 32 * rnd.randint(1, 4000)
        O = 8 * rnd.randint(1, 600)
        I = 16 * rnd.randint(1, 300)
        slab = O * I * 4
        for need, groups in ((lib.nm_update_gemm_workspace(T, O, I, 1), T // 16),
                             (lib.nm_update_gemm_workspace(T, O, I, 0), T // 16),
                             (lib.nm_update_gemm_q8_workspace(T, O, I), T // 32)):
            assert need % slab == 0, (T, O, I, need)
            assert need // slab <= groups, (T, O, I, need)
            assert need // slab != 1                      # one slab needs no second pass
        cb = 8 * rnd.randint(1, 64)
        n = rnd.choice([1, 9, 25])
        need = lib.nm_update_gemm_shifted_workspace(T, O, cb, n)
        assert need % (O * cb * n * 4) == 0 and need // (O * cb * n * 4) <= T // 16
        # the three-term mode holds six bf16 planes besides the 16-bit kernel's own workspace
        need3 = lib.nm_update_gemm_workspace(T, O, I, 2)
        assert need3 >= 3 * (T // 2 * O * 2) + 3 * (T * I * 2) + lib.nm_update_gemm_workspace(T, O, I, 1)

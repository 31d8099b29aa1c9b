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
                          "nm_update_gemm_workspace", "nm_last_error", "nm_version"}
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

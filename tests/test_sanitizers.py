"""Host-side sanitizer runs (AddressSanitizer + UndefinedBehaviorSanitizer, CPU only; no GPU code is sanitized):

  * the C oracle, compiled together with tests/san_oracle_driver.c, on exactly-sized buffers with ragged shapes, padded
    strides and edge values -- an access past an end, a signed overflow or a misaligned access aborts the run;
  * the host side of the C ABI: csrc/nm_abi.hip compiled for the host only and linked with stub launchers
    (tests/san_abi_driver.cpp), walking every validation path, including absurdly large sizes whose byte ranges must
    not overflow.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-O1", "-g"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0:abort_on_error=0",
           UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1", OMP_NUM_THREADS="4")


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, f"{' '.join(cmd)}\n{r.stdout}\n{r.stderr}"
    return r


def test_oracle_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "san_oracle")
    _run(["gcc", "-std=c11", *SAN, "-ffp-contract=off", "-fopenmp", "-Wall", "-Wextra",
          os.path.join(ROOT, "tests", "san_oracle_driver.c"), os.path.join(ROOT, "oracle", "mvue_oracle.c"), "-o", exe, "-lm"])
    r = _run([exe], env=ENV, timeout=600)
    assert "oracle sanitizer driver ok" in r.stdout


def test_abi_validation_under_asan_and_ubsan(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc) or shutil.which("g++") is None:
        pytest.skip("needs hipcc (host-only compile of the ABI layer) and g++")
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    obj, exe = str(tmp_path / "nm_abi_san.o"), str(tmp_path / "san_abi")
    # sanitizer flags go to the host compilation only
    host_san = []
    for f in ("-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all"):
        host_san += ["-Xarch_host", f]
    _run([hipcc, "--offload-arch=gfx950", "--offload-host-only", "-O1", "-g", "-std=c++17", "-fPIC", *host_san, "-c",
          os.path.join(ROOT, "paper_2203_10991_amd", "csrc", "nm_abi.hip"), "-o", obj], cwd=str(tmp_path))
    _run(["g++", "-std=c++17", *SAN, "-D__HIP_PLATFORM_AMD__", f"-I{rocm}/include", f"-I{ROOT}/include",
          os.path.join(ROOT, "tests", "san_abi_driver.cpp"), obj, "-o", exe, f"-L{rocm}/lib", "-lamdhip64", f"-Wl,-rpath,{rocm}/lib"])
    r = _run([exe], env=ENV, timeout=300)
    assert "abi sanitizer driver ok" in r.stdout

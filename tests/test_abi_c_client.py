"""The C ABI from plain C: the header is valid C11 on its own, and tests/abi_client.c -- a C program that uses
only the HIP runtime and include/nm_mvue.h -- builds, and on a GPU runs one pass of the hot path and agrees with
the C oracle (it links it: test code)."""
import os
import subprocess

import pytest

import build_abi_client

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_header_is_valid_c11_and_cxx():
    hdr = os.path.join(ROOT, "include", "nm_mvue.h")
    for cmd in (["gcc", "-std=c11", "-x", "c"], ["g++", "-std=c++17", "-x", "c++"]):
        r = subprocess.run(cmd + ["-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only", hdr], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr


def test_c_client_builds():
    from paper_2203_10991_amd import api
    if not os.path.exists(api.LIB_PATH):
        pytest.skip("library not built")
    from oracle import cwrap
    cwrap.lib()                                   # makes sure the oracle library exists
    assert os.access(build_abi_client.build(), os.X_OK)


@pytest.mark.gpu
def test_c_client_runs_the_hot_path_against_the_oracle():
    exe = build_abi_client.OUT
    if not os.path.exists(exe):
        build_abi_client.build()
    print("running", exe, flush=True)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    print(r.stdout, r.stderr, flush=True)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr)
    assert "abi client ok" in r.stdout

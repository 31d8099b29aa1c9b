"""Builds tests/abi_client (a plain C user of the C ABI, checked against the C oracle) with gcc.
``python tests/build_abi_client.py``; __graft_entry__.build() calls it after the two libraries are built."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
OUT = os.path.join(HERE, "abi_client")


def build() -> str:
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    if os.path.exists(OUT):
        os.remove(OUT)
    cmd = ["gcc", "-std=c11", "-O1", "-Wall", "-Werror", "-D__HIP_PLATFORM_AMD__", f"-I{rocm}/include",
           f"-I{ROOT}/include", os.path.join(HERE, "abi_client.c"), "-o", OUT,
           f"-L{ROOT}/paper_2203_10991_amd", "-lnm_mvue", f"-L{ROOT}/oracle", "-lmvue_oracle",
           f"-L{rocm}/lib", "-lamdhip64", "-lm",
           "-Wl,-rpath,$ORIGIN/../paper_2203_10991_amd", "-Wl,-rpath,$ORIGIN/../oracle", f"-Wl,-rpath,{rocm}/lib"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("gcc failed on abi_client.c:\n" + r.stdout + r.stderr)
    return OUT


if __name__ == "__main__":
    print(build())

"""Builds the plain-C test program that drives libgs.so through its C ABI (step_demo.c, C99, gcc):
HIP runtime C API for memory, libgs.so for the step, the C oracle (linked in) for the expected
values.  Test infrastructure: the binary lands in tests/c_abi/_build/ and a GPU test runs it."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
PKG = os.path.join(ROOT, "paper_2512_17570_amd")
OUT_DIR = os.path.join(HERE, "_build")
C_DEMO = os.path.join(OUT_DIR, "gs_c_demo")


def build_c_demo(verbose: bool = True) -> str:
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    os.makedirs(OUT_DIR, exist_ok=True)
    cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-Wextra", "-Wno-unused-parameter", "-ffp-contract=off",
           "-I", os.path.join(rocm, "include"), "-I", os.path.join(ROOT, "include"),
           os.path.join(HERE, "step_demo.c"), os.path.join(ROOT, "oracle", "gs_oracle.c"),
           "-L", PKG, "-lgs", "-L", os.path.join(rocm, "lib"), "-lamdhip64", "-lm",
           "-Wl,-rpath," + PKG, "-Wl,-rpath,$ORIGIN/../../../paper_2512_17570_amd", "-Wl,-rpath," + os.path.join(rocm, "lib"),
           "-o", C_DEMO]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return C_DEMO


if __name__ == "__main__":
    build_c_demo()

"""Builds tests/host_c/des_host_step: a plain C11 host program (no Python in its process) that drives one DES
step through include/des.h with hipMalloc'd buffers and checks it against the C oracle, which is linked in.
Test infrastructure; called by __graft_entry__.build().  Usage: python tests/host_c/build.py"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
BIN = os.path.join(HERE, "des_host_step")


def build(verbose: bool = False) -> str:
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    pkg = os.path.join(ROOT, "paper_1909_04823_amd")
    cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-Wall", "-D__HIP_PLATFORM_AMD__",
           "-I", os.path.join(rocm, "include"), "-I", os.path.join(ROOT, "include"),
           os.path.join(HERE, "des_host_step.c"), os.path.join(ROOT, "oracle", "des_oracle.c"),
           "-o", BIN, "-L", pkg, "-ldes", "-L", os.path.join(rocm, "lib"), "-lamdhip64", "-lm",
           "-Wl,-rpath,$ORIGIN/../../paper_1909_04823_amd", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return BIN


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)

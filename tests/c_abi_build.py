"""Builds tests/c_abi_parity.cpp: a host-only C++ program that drives libfp8lm.so through include/fp8lm.h and
compares it with the oracle library it loads at run time.  Built ahead of the tests (by ``__graft_entry__.build``),
never inside a GPU run."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "c_abi_parity.cpp")
EXE = os.path.join(HERE, "_build", "c_abi_parity")
LIBDIR = os.path.join(ROOT, "paper_2310_18313_amd")


def build(force: bool = False) -> str:
    deps = [SRC, os.path.join(ROOT, "include", "fp8lm.h"), os.path.join(LIBDIR, "libfp8lm.so")]
    if not force and os.path.exists(EXE) and all(os.path.getmtime(EXE) >= os.path.getmtime(d) for d in deps):
        return EXE
    os.makedirs(os.path.dirname(EXE), exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    subprocess.check_call([
        hipcc, "-O2", "-std=c++17", "-Wall", "-Wextra", "-I", os.path.join(ROOT, "include"), "-o", EXE, SRC,
        "-L", LIBDIR, "-lfp8lm", "-Wl,-rpath,$ORIGIN/../../paper_2310_18313_amd", "-ldl"])
    return EXE


if __name__ == "__main__":
    print(build(force=True))

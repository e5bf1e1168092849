"""Builds the plain-C client of libmoev's C ABI (test infrastructure) next to this file."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
EXE = os.path.join(HERE, "moev_c_client")
LIBDIR = os.path.join(ROOT, "paper_2412_15411_amd")


def build(verbose: bool = False) -> str:
    """Compiles moev_c_client.c as C99 with the ROCm clang and links it against libmoev.so (found at run time through an
    $ORIGIN-relative rpath) and the HIP runtime."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cc = os.path.join(rocm, "llvm", "bin", "clang")
    cmd = [cc, "-std=c99", "-O2", "-Wall", "-Wextra", "-pedantic", "-I" + os.path.join(ROOT, "include"),
           "-isystem", os.path.join(rocm, "include"), os.path.join(HERE, "moev_c_client.c"), "-o", EXE,
           "-L" + LIBDIR, "-lmoev", "-L" + os.path.join(rocm, "lib"), "-lamdhip64",
           "-Wl,-rpath,$ORIGIN/../../paper_2412_15411_amd", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("building the C client failed:\n" + res.stderr)
    if verbose and res.stderr.strip():
        print(res.stderr)
    return EXE


if __name__ == "__main__":
    print(build(verbose=True))

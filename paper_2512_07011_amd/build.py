"""Builds libbsfa.so (the HIP kernels and their C ABI) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libbsfa.so")
SOURCES = ["bsfa_fwd.hip", "bsfa_select.hip", "bsfa_probe.hip", "bsfa_api.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         # packed-fp32 VALU forms are kept out of the generated code on this target
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # the tile copies set M0 in inline asm and list it as clobbered, which clang notes for every
         # instantiation (thousands of identical lines): that one diagnostic is switched off
         "-Wall", "-Wno-unused-function", "-Wno-inline-asm"]


def build_lib(verbose: bool = False, extra_flags=()) -> str:
    """Compile every kernel source into paper_2512_07011_amd/libbsfa.so and return its path."""
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [HIPCC, *FLAGS, *extra_flags, "-o", tmp] + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    try:
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        out = "\n".join(l for l in r.stdout.splitlines() if "is not a recognized feature for this target" not in l)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + out)
        if verbose and out.strip():
            print(out)
        os.replace(tmp, LIB)
    finally:                      # an interrupted or failed build leaves no partial library behind
        if os.path.exists(tmp):
            os.remove(tmp)
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose=True))

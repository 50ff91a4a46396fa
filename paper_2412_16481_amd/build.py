"""Build step: compiles csrc/*.hip into paper_2412_16481_amd/libflash3d.so for gfx950 with hipcc, and the
issue-rate microbenchmark csrc/microbench/*.hip into libf3d_microbench.so (measurement aid of bench.py --ceilings)."""
from __future__ import annotations

import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libflash3d.so")
MICRO_LIB = os.path.join(HERE, "libf3d_microbench.so")


def hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


def _compile(srcs, out, verbose, extra) -> None:
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(HERE, "csrc"),
           # packed fp32 VALU forms are kept out of the generated code on purpose
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           # MFMA accumulators live in ordinary VGPRs (no AGPR copies around the softmax)
           "-mllvm", "--amdgpu-mfma-vgpr-form",
           # the global->LDS loads of attn.hip name M0 as clobbered, which clang reports as a reserved register
           "-Wno-inline-asm",
           *extra, *srcs, "-o", out]
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if verbose or res.returncode != 0:
        sys.stderr.write(err + "\n")
    if res.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(cmd))


def build(verbose: bool = False, extra=()) -> str:
    """Compile every HIP source (always recompiles): the library, then the microbenchmark."""
    _compile(sorted(glob.glob(os.path.join(HERE, "csrc", "*.hip"))), LIB, verbose, extra)
    _compile(sorted(glob.glob(os.path.join(HERE, "csrc", "microbench", "*.hip"))), MICRO_LIB, verbose, ())
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, extra=sys.argv[1:]))

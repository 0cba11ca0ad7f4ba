"""Compile the HIP sources in ``csrc/`` for gfx950 into ``liboptimus_attn.so`` (in-tree)."""
from __future__ import annotations

import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "liboptimus_attn.so")


def sources() -> list[str]:
    return sorted(glob.glob(os.path.join(HERE, "csrc", "*.hip")) +
                  glob.glob(os.path.join(HERE, "csrc", "*.cpp")))


def build(verbose: bool = False) -> str:
    """Always recompiles.  Returns the path of the in-tree shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           # Lets max() drop its signalling-NaN quieting moves.  What the kernels rely on: a
           # key outside the item's range may hold NaN and does enter the score MFMA, but its
           # score is replaced by -inf with an integer-compared select before any max / exp
           # sees it, and its V bits are cleared before the second MFMA; (-inf) - (-inf) in
           # the lazy running-max test may be NaN, and either outcome of that compare keeps
           # -inf.  NaN in a visible input gives an undefined output, as in any attention kernel.
           "-fno-honor-nans",
           # host code: SSE4.1 gives the planner's ceil() as one instruction instead of a
           # library call (the work-list fit evaluates it a few thousand times per plan)
           "-Xarch_host", "-msse4.1",
           "-Wall", "-Wno-unused-function",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc")]
    if verbose:
        cmd += ["-Rpass-analysis=kernel-resource-usage"]
    lib = LIB
    cmd += sources() + ["-o", lib]
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass warns that it does not know the packed-fp32 target feature: harmless
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        sys.stderr.write(err + "\n")
        raise RuntimeError("hipcc failed building liboptimus_attn.so")
    if verbose and err.strip():
        sys.stderr.write(err + "\n")
    return lib


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))

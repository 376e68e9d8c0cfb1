"""Build libstrads_lasso.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libstrads_lasso.so")
LIB_DEBUG = os.path.join(HERE, "libstrads_lasso_debug.so")   # -DSTRADS_DEBUG_SYNC: see strads_lasso_debug_build
SOURCES = ["api.hip", "sampler.hip", "gram.hip", "filter.hip", "update.hip", "csc.hip", "geno.hip", "noalloc.hip"]


def build(verbose: bool = False, debug: bool = False) -> str:
    """debug: the variant that waits and checks for errors after every kernel launch and checks the
    unit-norm precondition at create (libstrads_lasso_debug.so, loaded when STRADS_LASSO_DEBUG=1)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = LIB_DEBUG if debug else LIB
    cmd = [hipcc, "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
           "-I", INCLUDE, "-I", CSRC,
           # packed fp32 instructions are not to be generated on this target
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           # the sampling key is specified operation by operation: no contraction
           "-ffp-contract=off",
           # (-Wno-inline-asm: the global -> LDS loads of gram.hip are assembly statements that set M0 themselves)
           "-Wall", "-Wno-unused-function", "-Wno-pass-failed", "-Wno-inline-asm"] + (["-DSTRADS_DEBUG_SYNC"] if debug else []) + [
           "-o", out] + [os.path.join(CSRC, s) for s in SOURCES]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(" ".join(cmd))
        print(res.stdout)
        print("\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l))
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed building {os.path.basename(out)}")
    return out


if __name__ == "__main__":
    import sys
    print(build(verbose=True, debug="--debug" in sys.argv))

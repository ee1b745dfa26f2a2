"""Build libpex.so (HIP, gfx950) in-tree with hipcc.  Run as ``python -m paper_2510_00236_amd.build``."""
from __future__ import annotations

import glob
import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libpex.so")
_OBJ = os.path.join(_HERE, "_build")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wextra", "-Wno-inline-asm",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(_ROOT, "include"), "-I", CSRC]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build(verbose: bool = False, extra_flags=()) -> str:
    """Compile every translation unit and link libpex.so.  Always recompiles."""
    os.makedirs(_OBJ, exist_ok=True)
    objs = []
    procs = []
    for src in sources():
        obj = os.path.join(_OBJ, os.path.basename(src)[:-4] + ".o")
        cmd = [HIPCC, *FLAGS, *extra_flags, "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    # what the four-wave kernel and the Gram kernel assume about their own machine code, checked while the objects compile
    from . import isa_check
    isa_error = None
    try:
        isa_check.check_all(HIPCC, [*FLAGS, *extra_flags], os.path.join(CSRC, "pex_stat_bf16.hip"), os.path.join(CSRC, "pex_gram.hip"),
                            os.path.join(CSRC, "pex_gram_wide.hip"))
    except (isa_check.IsaCheckError, subprocess.CalledProcessError) as e:
        isa_error = e
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        # hipcc's host pass does not know the packed-fp32 target feature and says so; that is harmless
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if out.strip() and (verbose or p.returncode != 0):
            print(out, flush=True)
        if p.returncode != 0:
            print(f"hipcc failed on {src}", file=sys.stderr)
            failed = True
    if failed:
        raise RuntimeError("libpex build failed")
    if isa_error is not None:
        raise RuntimeError(f"libpex build failed: {isa_error}")
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))

"""Build the C-ABI library ``libvecinfer.so`` for gfx950 with hipcc (in-tree)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libvecinfer.so")
SOURCES = ["api.hip", "merge.hip", "encode.hip", "calibrate.hip", "probe.hip", "decode_lut.hip", "decode_mfma.hip", "decode_mfma_wide.hip", "decode_mfma_wide64.hip", "decode_mfma_tiled.hip", "decode_roles.hip"]

# Packed-fp32 VALU forms are switched off for the device pass: hipcc otherwise forms them
# from plain float code.
#
# Kernel-argument preloading: the leading scalar arguments of a kernel (up to 14 dwords) are placed
# in scalar registers by the command processor before a wavefront starts, so the attention and
# merge kernels issue their first memory requests without a trip to the argument buffer (1.4 us
# per kernel when that buffer is cold).  Code built this way still runs where the firmware does
# not preload: the kernel then enters through a short compatibility prologue that loads the same
# registers itself.
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-mllvm", "-amdgpu-kernarg-preload-count=16"]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def build(verbose: bool = False, extra_flags=()) -> str:
    """Compile every kernel source and link the shared library.  Always recompiles."""
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        cmd = [hipcc(), *FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for src, pr in procs:
        out, _ = pr.communicate()
        # the host pass warns that it does not know the packed-fp32 feature: harmless
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l and l.strip())
        if pr.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and out:
            print(out, flush=True)
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))

"""Build libdualkv.so (gfx950) in-tree with hipcc.  Usage: python -m paper_2605_15422_amd.build"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdualkv.so")
SOURCES = ["api.hip", "qstat.hip", "fwd2.hip", "dq2.hip", "dkdv4.hip", "fwd256.hip", "dq256.hip", "dkdv256.hip", "dkdv512.hip", "dq512.hip", "fwd512.hip", "kvstat.hip", "aux.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-munsafe-fp-atomics",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-Wno-inline-asm"]


# The generic kernels run four waves of up to 512 registers at some head dims.  There the compiler's default puts MFMA
# results in the accumulation half of the register file and copies them back and forth for the vector ALU (256 copies
# per tile in the d = 256 dQ kernel); with the MFMAs in their VGPR form it allocates the two halves itself (8 % faster).
PER_FILE_FLAGS = {"qstat.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"], "kvstat.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


def build(verbose: bool = True, extra_flags=()) -> str:
    extra_flags = tuple(extra_flags) + tuple(os.environ.get("DUALKV_EXTRA_HIPCC_FLAGS", "").split())
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    hipcc = _hipcc()

    def compile_one(src):
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        cmd = [hipcc, *FLAGS, *PER_FILE_FLAGS.get(src, []), *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, r.stdout, r.stderr))
        if verbose and r.stderr.strip():
            lines = [ln for ln in r.stderr.splitlines() if "packed-fp32-ops" not in ln and ln.strip()]
            if lines:
                print("\n".join(lines), file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s\n%s" % (r.stdout, r.stderr))
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build()

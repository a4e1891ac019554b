"""Compile the HIP/C++ sources in csrc/ into libsig_mi355x.so (in-tree) for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsig_mi355x.so")
SOURCES = ["api.cpp", "wordset.cpp", "jit.cpp", "jit_lanes.cpp", "kernels_generic.hip", "kernels_trunc.hip", "kernels_chunk.hip", "kernels_words.hip"]
# -packed-fp32-ops is switched off on purpose: the packed FP32 forms are not used by this library.
HIPCC_FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
               "-packed-fp32-ops", "-Wall", "-Wno-unused-command-line-argument",
               # matrix-instruction results stay in ordinary vector registers: the vector ALU reads them without
               # v_accvgpr_read copies (a quarter of the instructions of the backward kernels otherwise)
               "-mllvm", "-amdgpu-mfma-vgpr-form",
               # instruction scheduling for latency hiding inside a wavefront rather than for occupancy, which launch
               # bounds fix anyway (two wavefronts per SIMD at most in the main kernels): measured 3-7 % on them
               "-mllvm", "-amdgpu-sched-strategy=max-ilp"]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def build(verbose: bool = False) -> str:
    objs = []
    bdir = os.path.join(HERE, "_build")
    os.makedirs(bdir, exist_ok=True)
    procs = []
    for src in SOURCES:
        obj = os.path.join(bdir, src + ".o")
        cmd = [hipcc(), *HIPCC_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and out.strip():
            print(out)
    tmp = LIB + f".{os.getpid()}.tmp"
    cmd = [hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp, *objs, "-L/opt/rocm/lib", "-lhiprtc"]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))

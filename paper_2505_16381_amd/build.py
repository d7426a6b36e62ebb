"""Builds libpath_attn.so (hipcc, gfx950) in-tree.  Usage: python -m paper_2505_16381_amd.build"""
from __future__ import annotations

import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libpath_attn.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-fno-honor-nans", "-mno-amdgpu-ieee",      # infinities are used, NaNs never: no canonicalisation of max operands
         "-Wno-unused-command-line-argument"]
# per-file extras: the sweep keeps MFMA results in architectural VGPRs (two waves per SIMD, 256 registers each)
PER_FILE = {"attn_fwd2.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"]}


def build(verbose: bool = True, extra=()) -> str:
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    objs = []
    procs = []
    os.makedirs(os.path.join(HERE, "_build"), exist_ok=True)
    for s in srcs:
        o = os.path.join(HERE, "_build", os.path.basename(s) + ".o")
        objs.append(o)
        cmd = [HIPCC, *FLAGS, *PER_FILE.get(os.path.basename(s), []), *extra, "-c", s, "-o", o]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append(subprocess.Popen(cmd, stderr=subprocess.PIPE, text=True))
    for pr in procs:
        _, err = pr.communicate()
        err = "\n".join(l for l in err.splitlines() if "packed-fp32-ops" not in l)
        if pr.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + err)
        if verbose and err.strip():
            print(err, file=sys.stderr)
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", OUT, *objs]
    subprocess.run(cmd, check=True)
    return OUT


if __name__ == "__main__":
    build(extra=sys.argv[1:])
    print("built", OUT)

"""Builds libdash_attn.so (gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdash_attn.so")
# bench.py's yardstick kernels (streaming read, register-fed MFMA loop): their own small library
MICROBENCH_LIB = os.path.join(HERE, "libdash_microbench.so")
# (source, extra defines, object name); stage1_regs.hip is compiled once per GQA group size
SOURCES = [(s, [], s.replace(".hip", ".o")) for s in
           ["api.hip", "compress.hip", "stage1.hip", "stage2.hip", "stage2_decode.hip", "stage2_f32.hip", "backward.hip"]]
SOURCES += [("stage1_regs.hip", [f"-DDASH_S1R_G={g}"], f"stage1_regs_g{g}.o") for g in (1, 2, 4, 8, 16)]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-w",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(verbose: bool = True, lib: str = LIB, extra=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    extra = list(extra) + os.environ.get("DASH_EXTRA_FLAGS", "").split()
    objs, procs = [], []
    for s, defs, oname in SOURCES:   # one compiler process per object file, all at once
        o = os.path.join(CSRC, oname)
        cmd = [hipcc, *[f for f in FLAGS if f != "-shared"], *extra, *defs, "-c", os.path.join(CSRC, s), "-o", o]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((cmd, subprocess.Popen(cmd)))
        objs.append(o)
    for cmd, pr in procs:
        if pr.wait() != 0:
            raise subprocess.CalledProcessError(pr.returncode, cmd)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", lib]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    if lib == LIB:
        cmd = [hipcc, *FLAGS, *extra, os.path.join(CSRC, "microbench.hip"), "-o", MICROBENCH_LIB]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
    return lib


if __name__ == "__main__":
    build()
    sys.exit(0)

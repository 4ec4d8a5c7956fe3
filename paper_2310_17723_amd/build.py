"""Builds libhero.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2310_17723_amd.build

-ffp-contract=off keeps the epilogue's fp32 operation order exactly as written (explicit
fmaf where a fused multiply-add is meant); packed-fp32 instruction selection is disabled;
the attention kernels keep MFMA results in VGPRs (their scores go straight into vector ALU code;
for the GEMMs the AGPR form measured faster).
"""
from __future__ import annotations

import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libhero.so")
PROBE_SRC = os.path.join(HERE, "probe", "probe_ops.hip")      # bench-side measuring instruments: a library of their own
PROBE_LIB = os.path.join(HERE, "libhero_probe.so")

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-Wno-inline-asm",      # (the m0 clobber of the direct-load asm is intended)
         "-DHERO_BUILD_ARCH=\"gfx950\""]


# extra per-file flags
EXTRA = {"int8_attn.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
         "bf16_ops.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build_lib(verbose: bool = True, jobs: int = 8) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    for src in sources():
        obj = os.path.join(objdir, os.path.basename(src) + ".o")
        objs.append(obj)
        cmd = [hipcc, *FLAGS, *EXTRA.get(os.path.basename(src), []), "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        if len(procs) >= jobs:
            _drain(procs)
    _drain(procs)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    cmd = [hipcc, *FLAGS, "-shared", "-o", PROBE_LIB, PROBE_SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + "\n")
        raise RuntimeError("hipcc failed on the probe library")
    return LIB


def _drain(procs):
    while procs:
        src, p = procs.pop(0)
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            sys.stderr.write(out + "\n")
            raise RuntimeError(f"hipcc failed on {src}")
        if out.strip():
            print(out)


if __name__ == "__main__":
    build_lib()

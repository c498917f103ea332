"""Builds libs2attn.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libs2attn.so")
PROBES_LIB = os.path.join(HERE, "libs2attn_probes.so")
SOURCES = ["s2attn_api.hip", "s2attn_prepost.hip", "s2attn_f32.hip", "s2attn_bf16_fwd.hip", "s2attn_bf16_bwd.hip",
           "s2attn_bf16_dkdv_split.hip", "s2attn_bf16_dq_spill.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-fno-honor-nans", "-mno-amdgpu-ieee",
         "-Wno-unused-command-line-argument", "-Wno-inline-asm"]


def build(verbose: bool = True, extra_flags=(), out_path: str | None = None) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build" if out_path is None else "_build_" + os.path.basename(out_path))
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [hipcc, *FLAGS, *extra_flags, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
               "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            failed = True
            sys.stderr.write(f"[build] {src} FAILED\n{out}\n")
        elif verbose and out.strip():
            sys.stderr.write(f"[build] {src}:\n{out}\n")
    if failed:
        raise RuntimeError("hipcc failed")
    lib = LIB if out_path is None else out_path
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs]
    subprocess.run(link, check=True)
    if verbose:
        sys.stderr.write(f"[build] wrote {lib}\n")
    if out_path is None:
        build_probes(hipcc, verbose)
    return lib


def build_probes(hipcc: str, verbose: bool) -> str:
    """libs2attn_probes.so: the hardware probes of bench.py --probes (MFMA rate against operand
    data, L2 atomic rate).  Separate from the attention library, which does not depend on it."""
    cmd = [hipcc, *FLAGS, "-munsafe-fp-atomics", "-shared", "-o", PROBES_LIB, os.path.join(CSRC, "s2attn_probes.hip")]
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if p.returncode != 0:
        sys.stderr.write(p.stdout)
        raise RuntimeError("hipcc failed on s2attn_probes.hip")
    if verbose:
        sys.stderr.write(f"[build] wrote {PROBES_LIB}\n")
    return PROBES_LIB


if __name__ == "__main__":
    build()

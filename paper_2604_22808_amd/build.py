"""Builds libfreqattn.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libfreqattn.so")
SOURCES = ["mfma_dct_plain.hip", "mfma_dct_plain_tot.hip", "mfma_dct_scatter.hip", "mfma_dct_scatter_en.hip",
           "mfma_dct_gather.hip", "mfma_attn.hip", "mfma_vsum.hip", "mfma_gemm.hip", "api.cpp", "tables.cpp", "generic_kernels.hip", "mfma_dct.hip"]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def build(verbose: bool = False, jobs: int = 6) -> str:
    """Compiles every source to an object (in parallel) and links the shared library.  Always recompiles."""
    objdir = os.path.join(PKG, "_build")
    os.makedirs(objdir, exist_ok=True)
    flags = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-x", "hip",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-Wno-unused-value", "-Wno-inline-asm"]   # (m0 named as clobbered by the LDS-copy assembly)
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(objdir, os.path.splitext(src)[0] + ".o")
        objs.append(obj)
        cmd = [hipcc()] + flags + ["-c", os.path.join(CSRC, src), "-o", obj]
        # compiler output goes to a file: a pipe nobody reads while the build waits would block a chatty compile
        log = open(obj + ".log", "w+")
        procs.append((src, subprocess.Popen(cmd, stdout=log, stderr=subprocess.STDOUT), log))
        while sum(p.poll() is None for _, p, _ in procs) >= jobs:
            for _, p, _ in procs:
                if p.poll() is None:
                    p.wait()
                    break
    failed = False
    for src, p, log in procs:
        p.wait()
        log.seek(0)
        out = log.read()
        log.close()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            failed = True
            sys.stderr.write(f"--- {src} failed\n{out}\n")
        elif verbose and out.strip():
            sys.stderr.write(f"--- {src}\n{out}\n")
    if failed:
        raise RuntimeError("hipcc failed")
    tmp = LIB + ".tmp"
    subprocess.check_call([hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp] + objs)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))

"""Builds libmoe_cache.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmoe_cache.so")
SOURCES = ["moe_cache.hip", "route_cache.hip", "ffn_rowmajor.hip", "ffn_tiled.hip", "ffn_fused.hip", "ffn_gemm.hip", "stream_probe.hip",
           "cache_sim.hip", "ffn_fused_q4.hip", "ffn_gemm_q4.hip", "noalloc.hip", "ffn_tiles.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function"]


def build_library(verbose: bool = False) -> str:
    """Compile every HIP source and link the shared library; always rebuilds."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs, objs = [], []
    for src in SOURCES:
        obj = os.path.join(objdir, src + ".o")
        objs.append(obj)
        cmd = [hipcc, *FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
               "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for cmd, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError("hipcc failed: %s\n%s" % (" ".join(cmd), out))
        if verbose and out.strip():
            print(out)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    subprocess.check_call(cmd)
    return LIB


def _stale() -> bool:
    """True if a source or header is newer than the built library."""
    if not os.path.exists(LIB):
        return True
    built = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, n) for n in os.listdir(CSRC)] + [os.path.join(ROOT, "include", "moe_cache.h")]
    return any(os.path.getmtime(d) > built for d in deps if os.path.isfile(d))


def ensure_built() -> str:
    """Tests, smoke and the benchmark load what is built; build if nothing is there.  A library older than its
    sources is rebuilt when a compiler is at hand, and refused otherwise: running stale kernels would test or
    time something other than the sources say."""
    if not _stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if os.path.exists(LIB) and not os.path.exists(hipcc):
        raise RuntimeError("libmoe_cache.so is older than its sources and no hipcc is available to rebuild it")
    return build_library()


if __name__ == "__main__":
    print(build_library(verbose=True))

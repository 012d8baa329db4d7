"""Builds libcalvo.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcalvo.so")
SOURCES = ["calvo_api.hip", "kernels_ingest.hip", "attn_simple.hip", "attn_mfma.hip", "attn_pipe.hip", "attn_duo.hip", "attn_plan.cpp", "ingest_plan.cpp", "calvo_sched.cpp", "calvo_pool.cpp"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-result", "-fno-gpu-rdc"]


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *FLAGS, *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass warns that it does not know the packed-fp32 feature; that is harmless
    out = "\n".join(ln for ln in res.stdout.splitlines() if "packed-fp32-ops" not in ln)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return LIB


PROBES = ["probe_coissue.hip", "probe_valu_issue.hip"]      # stand-alone microbenchmarks, not part of the library


def build_probes(outdir: str) -> list:
    """Compiles the microbenchmarks into outdir (they are run by hand on a GPU machine)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(outdir, exist_ok=True)
    made = []
    for src in PROBES:
        exe = os.path.join(outdir, os.path.splitext(src)[0])
        cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
               "-packed-fp32-ops", os.path.join(CSRC, src), "-o", exe]
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n" + res.stdout)
        made.append(exe)
    return made


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)

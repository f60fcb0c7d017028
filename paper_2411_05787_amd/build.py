"""Builds librefreshkv.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librefreshkv.so")
SOURCES = ["rk_api.hip", "rk_attn.hip", "rk_topk.hip", "rk_gather.hip", "rk_query_sim.hip", "rk_step.hip",
           "rk_window.hip", "rk_h2o.hip"]
# Packed fp32 VALU forms are switched off for every device compilation of this library.
HIPCC_FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               # the first scalar kernel arguments arrive in registers (see attn_split_kernel)
               "-mllvm", "-amdgpu-kernarg-preload-count=16",
               "-Wall", "-Wno-unused-function"]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found: the HIP library cannot be built")


def build(verbose: bool = False, jobs: int = 6) -> str:
    """Compile every source for gfx950 and link the shared library; returns its path."""
    cc = hipcc()
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [cc, *HIPCC_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        if len([p for p in procs if p[2].poll() is None]) >= jobs:
            procs[0][2].wait()
    for src, cmd, pr in procs:
        out, _ = pr.communicate()
        lines = [ln for ln in out.splitlines() if "packed-fp32-ops" not in ln]
        if pr.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s\n%s" % (src, " ".join(cmd), "\n".join(lines)))
        if verbose and lines:
            print("\n".join(lines))
    cmd = [cc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))

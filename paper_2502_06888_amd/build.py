"""Build the HIP library (gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libklotski_moe.so")
OBJ_DIR = os.path.join(HERE, "_build")
SOURCES = ["moe_api.hip", "k_router.hip", "k_plan.hip", "k_misc.hip", "k_ffn_f32.hip",
           "k_ffn_bf16.hip", "attn_api.hip", "k_attn.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _newer(src: str, dst: str) -> bool:
    return not os.path.exists(dst) or os.path.getmtime(dst) < os.path.getmtime(src)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every source and link the shared library.  ``force`` recompiles everything."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    headers = [os.path.join(CSRC, "kernels.h"), os.path.join(CSRC, "attn_kernels.h"),
               os.path.join(HERE, "..", "include", "moe.h"), os.path.join(HERE, "..", "include", "moe_attn.h")]
    jobs = []
    for name in SOURCES:
        src = os.path.join(CSRC, name)
        obj = os.path.join(OBJ_DIR, name.replace(".hip", ".o"))
        stale = force or _newer(src, obj) or any(_newer(h, obj) for h in headers)
        if stale:
            jobs.append((src, obj))

    def compile_one(job):
        src, obj = job
        cmd = [hipcc, *FLAGS, "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        return src, r

    with ThreadPoolExecutor(max_workers=min(6, max(1, len(jobs)))) as pool:
        for src, r in pool.map(compile_one, jobs):
            warn = "\n".join(l for l in r.stderr.splitlines()
                             if "packed-fp32-ops" not in l and l.strip())
            if r.returncode != 0:
                raise RuntimeError(f"hipcc failed on {src}:\n{r.stderr}")
            if verbose and warn:
                print(warn, file=sys.stderr)
    objs = [os.path.join(OBJ_DIR, n.replace(".hip", ".o")) for n in SOURCES]
    if jobs or not os.path.exists(LIB):
        cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"link failed:\n{r.stderr}")
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, verbose=True))

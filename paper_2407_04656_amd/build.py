"""Build liblazarus_moe.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblazarus_moe.so")
SOURCES = ["route.hip", "plan.hip", "permute_combine.hip", "ffn.hip", "backward.hip", "misc.hip", "planner.cpp"]

FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fno-gpu-rdc", "-Wall", "-Wno-unused-function",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]
OBJ_DIR = os.path.join(HERE, "_build")  # git-ignored


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
    return proc.returncode, out


def build(verbose: bool = True) -> str:
    """Compile every translation unit (in parallel: the two GEMM files take a minute each) and link."""
    from concurrent.futures import ThreadPoolExecutor

    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    objs = [os.path.join(OBJ_DIR, os.path.splitext(s)[0] + ".o") for s in SOURCES]
    cmds = [[hipcc, *FLAGS, "-x", "hip", "-c", os.path.join(CSRC, s), "-o", o] for s, o in zip(SOURCES, objs)]
    jobs = max(1, min(len(cmds), int(os.environ.get("MAX_JOBS", os.cpu_count() or 1))))
    with ThreadPoolExecutor(jobs) as pool:
        results = list(pool.map(lambda c: _run(c, verbose), cmds))
    results.append(_run([hipcc, "--offload-arch=gfx950", "-fno-gpu-rdc", "-shared", "-fPIC", *objs, "-o", LIB], verbose)
                   if all(rc == 0 for rc, _ in results) else (1, "not linked"))
    out = "\n".join(o for _, o in results if o.strip())
    if verbose and out.strip():
        print(out, flush=True)
    if any(rc != 0 for rc, _ in results):
        raise RuntimeError("hipcc failed:\n" + out)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)

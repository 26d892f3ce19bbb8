"""Compile the HIP library in-tree: paper_2306_02272_amd/libowq.so (gfx950 only).

Every source is compiled to an object of its own (in parallel), then linked.  `defines` and
`out` let a developer build a variant beside the product library for A/B timing."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SOURCES = ["owq_api.cpp", "owq_pack.cpp", "owq_kernels.hip", "owq_gemv_multi.hip", "owq_tile.hip", "owq_tile_small.hip",
           "owq_search.hip", "owq_backward.hip", "owq_probe.hip"]
LIB = os.path.join(HERE, "libowq.so")
NOISE = "is not a recognized feature for this target"


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _run(cmd, cwd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, cwd=cwd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if NOISE not in l)
    if res.returncode != 0:
        sys.stderr.write(err + "\n")
        raise RuntimeError("hipcc failed: " + " ".join(cmd))
    if verbose and err.strip():
        print(err)


def build(verbose: bool = True, keep_asm: bool = False, defines=(), out: str = LIB, tag: str = "") -> str:
    out_dir = os.path.join(ROOT, "_build", tag) if tag else os.path.join(ROOT, "_build")
    os.makedirs(out_dir, exist_ok=True)
    flags = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
             "-I" + os.path.join(ROOT, "include"),
             # no packed-fp32 instructions: some of their forms misbehave on these machines
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wall", "-Wno-unused-command-line-argument"] + ["-D" + d for d in defines]
    if keep_asm:
        flags += ["-save-temps=obj"]
    objs = [os.path.join(out_dir, os.path.splitext(s)[0] + ".o") for s in SOURCES]
    jobs = [[hipcc()] + flags + ["-c", os.path.join(HERE, "csrc", s), "-o", o] for s, o in zip(SOURCES, objs)]
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
        list(pool.map(lambda c: _run(c, out_dir, verbose), jobs))
    tmp_lib = os.path.join(out_dir, "libowq.so")
    _run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp_lib] + objs, out_dir, verbose)
    os.replace(tmp_lib, out)
    return out


if __name__ == "__main__":
    build(keep_asm="--asm" in sys.argv)

"""In-tree build of the gfx950 library: hipcc compiles every csrc/*.hip into
libsolar.so next to this file.  No JIT, no cache outside the tree."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libsolar.so")
SOURCES = ["api", "gram", "eig", "project", "rsvd", "attention", "attention_x32", "linear", "backward", "dense_ref"]
FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build_library(verbose: bool = False) -> str:
    os.makedirs(BUILD, exist_ok=True)

    def compile_one(name: str) -> str:
        obj = os.path.join(BUILD, name + ".o")
        cmd = ["hipcc", *FLAGS, "-c", os.path.join(CSRC, name + ".hip"), "-o", obj]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc failed for {name}:\n{res.stderr}")
        if verbose and res.stderr.strip():
            print(res.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=6) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed:\n{res.stderr}")
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))

"""Compile the HIP sources into paper_2111_10672_amd/libspb.so for gfx950 (in-tree, no JIT cache)."""
from __future__ import annotations

import glob
import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libspb.so")


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
         # hipcc -O3 would otherwise form packed float32 instructions from scalar code
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I" + os.path.join(ROOT, "include")]


def _compile(src: str, obj: str):
    return subprocess.run([hipcc(), *FLAGS, "-c", src, "-o", obj], capture_output=True, text=True)


def build_library(verbose: bool = False) -> str:
    """Compile every csrc/*.hip (one process per file, side by side) and link libspb.so."""
    from concurrent.futures import ThreadPoolExecutor
    sources = sorted(glob.glob(os.path.join(HERE, "csrc", "*.hip")))
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    objs = [os.path.join(objdir, os.path.basename(s)[:-4] + ".o") for s in sources]
    with ThreadPoolExecutor(max_workers=min(8, len(sources))) as pool:
        results = list(pool.map(_compile, sources, objs))
    for src, res in zip(sources, results):
        if verbose or res.returncode:
            print(src, res.stdout, res.stderr)
        if res.returncode:
            raise RuntimeError(f"hipcc failed on {src}:\n" + res.stderr[-4000:])
    res = subprocess.run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB + ".tmp"], capture_output=True, text=True)
    if res.returncode:
        raise RuntimeError("link failed:\n" + res.stderr[-4000:])
    os.replace(LIB + ".tmp", LIB)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=False))

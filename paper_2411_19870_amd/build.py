"""Build libdemo.so (HIP kernels + C ABI) for gfx950, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "libdemo.so")
SOURCES = [os.path.join(PKG, "csrc", f) for f in ("demo_kernels.hip", "demo_enc64.hip", "demo_enc64d.hip", "demo_dec64.hip", "demo_dec32.hip", "demo_wg128.hip", "demo_noalloc.hip", "demo_api.cpp")]


def build(verbose: bool = True, out: str = LIB, defines=(), extra_flags=()) -> str:
    """Compile every source to an object (in parallel, one hipcc per file) and link the shared library.
    `extra_flags` go to every compile and to the link (e.g. host-side sanitizers)."""
    from concurrent.futures import ThreadPoolExecutor

    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(PKG, "_build", os.path.splitext(os.path.basename(out))[0])
    os.makedirs(objdir, exist_ok=True)
    flags = [
        "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
        # packed-fp32 VALU forms are kept out of the generated code on this target
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
        "-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG, "csrc"),
    ] + [f"-D{d}" for d in defines] + list(extra_flags)

    def compile_one(src: str) -> str:
        obj = os.path.join(objdir, os.path.basename(src) + ".o")
        cmd = [hipcc, "-c"] + flags + ["-o", obj, src]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        return obj

    jobs = max(1, min(len(SOURCES), os.cpu_count() or 1, 8))
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    link = [hipcc, "-shared", "-fPIC", "--offload-arch=gfx950"] + list(extra_flags) + ["-o", out] + objs
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.run(link, check=True)
    return out


if __name__ == "__main__":
    build()
    sys.exit(0)

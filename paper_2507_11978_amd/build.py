"""Build libnt.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

Each source is compiled to an object file in parallel (the kernel instantiations are
spread over several translation units for that purpose), then linked."""
from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libnt.so")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # the epilogues unroll 256 accumulator elements with address arithmetic, masks and format switches per
         # element: above LLVM's default size limit for "#pragma unroll", and a loop left rolled would index
         # the accumulator registers dynamically, i.e. move them to scratch memory
         "-mllvm", "-pragma-unroll-threshold=100000",
         "-Wall", "-Wno-unused-function"]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.cpp")) + glob.glob(os.path.join(CSRC, "*.hip")))


def _headers():
    return glob.glob(os.path.join(CSRC, "*.h")) + [os.path.join(HERE, "..", "include", "nt.h")]


def _quiet(text: str) -> str:
    # the host pass does not know the device-only target feature and says so; harmless
    return "\n".join(ln for ln in text.splitlines() if "packed-fp32-ops" not in ln)


def _compile(src: str, force: bool) -> str:
    obj = os.path.join(OBJ, os.path.basename(src) + ".o")
    newest = max(os.path.getmtime(p) for p in [src] + _headers())
    if not force and os.path.exists(obj) and os.path.getmtime(obj) >= newest:
        return obj
    res = subprocess.run(["hipcc"] + FLAGS + ["-c", src, "-o", obj], capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n" + _quiet(res.stdout + res.stderr))
    msg = _quiet(res.stdout + res.stderr).strip()
    if msg:
        print(msg, flush=True)
    return obj


def build(force: bool = True, jobs: int = 8) -> str:
    """Compile every HIP/C++ source into paper_2507_11978_amd/libnt.so.
    force=False recompiles only what is older than its source or a header."""
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(lambda s: _compile(s, force), sources()))
    res = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs,
                         capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + _quiet(res.stdout + res.stderr))
    return LIB


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv))

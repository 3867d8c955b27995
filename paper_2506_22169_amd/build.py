"""Builds libmcf.so (HIP kernels for gfx950 + the C ABI) in-tree with hipcc.

hipcc cross-compiles without a GPU.  Objects go to _build/ at the repository root (ignored
by git); the shared library is written next to this file so that it travels with the tree.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(ROOT, "_build", "mcf")
LIB = os.path.join(HERE, "libmcf.so")

# -packed-fp32-ops is switched off on purpose: hipcc must not form packed fp32 instructions.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function", "-Wno-inline-asm",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def sources():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hip", ".cpp")))


def _headers_mtime():
    hs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".h", ".hpp"))]
    hs.append(os.path.join(ROOT, "include", "mcf.h"))
    return max(os.path.getmtime(h) for h in hs)


def _compile(src, force, hdr_mtime):
    obj = os.path.join(OBJ_DIR, os.path.basename(src) + ".o")
    if (not force and os.path.exists(obj) and os.path.getmtime(obj) >= os.path.getmtime(src)
            and os.path.getmtime(obj) >= hdr_mtime):
        return obj
    cmd = ["hipcc"] + HIPCC_FLAGS + (["-x", "hip"] if src.endswith(".cpp") else []) + ["-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("hipcc failed on " + src)
    return obj


def build_library(force=True, jobs=8, verbose=False):
    """Compile every source and link libmcf.so.  force=False reuses up-to-date objects."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    hdr = _headers_mtime()
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force, hdr), sources()))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("link of libmcf.so failed")
    if verbose:
        print("built", LIB, "from", len(objs), "objects")
    return LIB


if __name__ == "__main__":
    build_library(force="--force" in sys.argv, verbose=True)

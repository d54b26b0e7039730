"""Compile the HIP sources under csrc/ into libbppsa.so for gfx950 (in-tree)."""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
INCLUDE = os.path.join(os.path.dirname(PKG_DIR), "include")
LIB_PATH = os.path.join(PKG_DIR, "libbppsa.so")
OBJ_DIR = os.path.join(PKG_DIR, "_build")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-munsafe-fp-atomics",
    "-I", INCLUDE, "-I", CSRC,
]


# Options of single files.  scan_h128.hip: MFMA results go to ordinary vector registers, because the
# reduce kernel feeds the accumulators of one step to the next step as the B operand, which the
# accumulation registers cannot be without a copy of all 64 per step (and twice the registers).
FILE_FLAGS = {
    "scan_h128.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
}


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


def _compile(src: str, force: bool) -> str:
    obj = os.path.join(OBJ_DIR, src[:-4] + ".o")
    src_path = os.path.join(CSRC, src)
    if not force and os.path.exists(obj):
        newest = max(os.path.getmtime(os.path.join(CSRC, f)) for f in os.listdir(CSRC))
        newest = max(newest, os.path.getmtime(os.path.join(INCLUDE, "bppsa.h")))
        if os.path.getmtime(obj) > newest:
            return obj
    cmd = [HIPCC, *FLAGS, *FILE_FLAGS.get(src, []), "-c", src_path, "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s\n%s" % (src, res.stdout, res.stderr))
    return obj


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every .hip file and link libbppsa.so.  Returns the library path."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    srcs = sources()
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), srcs))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n%s\n%s" % (res.stdout, res.stderr))
    if verbose:
        print("built", LIB_PATH, file=sys.stderr)
    return LIB_PATH


if __name__ == "__main__":
    build(force="--incremental" not in sys.argv, verbose=True)

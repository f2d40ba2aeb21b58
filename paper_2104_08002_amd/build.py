"""Compile the HIP sources under ``csrc/`` into ``libconv1d_mi355x.so`` for gfx950.

hipcc cross-compiles without a GPU.  Each translation unit is compiled to an object
(in parallel) and linked into one shared library that sits next to this file.
"""
from __future__ import annotations

import concurrent.futures
import hashlib
import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libconv1d_mi355x.so")
STAMP = LIB + ".srchash"   # hash of the sources the library was built from (travels with the library)
OBJ_DIR = os.path.join(HERE, "_build")

# packed FP32 VALU forms are switched off for all device code on this machine pool
HIP_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc", "-Wall", "-Wno-unused-function",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the fully unrolled MFMA schedules are long: with the default threshold the larger instantiations are left
    # as loops, their register arrays go to scratch memory and they run two orders of magnitude slower
    "-mllvm", "-pragma-unroll-threshold=262144",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def sources():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))


def source_hash() -> str:
    """SHA-256 over every file the library is compiled from (csrc/*.hip, csrc/*.h, include/conv1d.h) and the flags."""
    h = hashlib.sha256(" ".join(HIP_FLAGS).encode())
    deps = sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hip", ".h")))
    deps.append(os.path.join(os.path.dirname(HERE), "include", "conv1d.h"))
    for d in deps:
        h.update(os.path.basename(d).encode())
        with open(d, "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ_DIR, os.path.basename(src) + ".o")
    cmd = [hipcc(), *HIP_FLAGS, "-Rpass-analysis=kernel-resource-usage", "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    lines = (r.stdout + r.stderr).splitlines()
    # a kernel that keeps an array in scratch memory runs orders of magnitude slower than intended: say so loudly
    name = None
    for l in lines:
        if "Function Name:" in l:
            name = l.split("Function Name:")[1].strip()
        elif "ScratchSize [bytes/lane]:" in l and name is not None:
            nbytes = int(l.split("ScratchSize [bytes/lane]:")[1].split()[0])
            if nbytes > 128:
                print(f"WARNING: {os.path.basename(src)}: kernel {name} uses {nbytes} bytes of scratch per lane", file=sys.stderr)
            name = None
    msgs = "\n".join(l for l in lines if "packed-fp32-ops" not in l and "remark:" not in l and "[-Rpass-analysis" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{msgs}")
    if msgs.strip():
        print(msgs, file=sys.stderr)
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    srcs = sources()
    stamp = source_hash()
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(_compile, srcs))
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout + r.stderr)
    with open(STAMP, "w") as f:
        f.write(stamp + "\n")
    if verbose:
        print(f"built {LIB} from sources {stamp}")
    return LIB


def built_hash():
    """Hash of the sources the existing library was built from; None when there is no library or no record."""
    if not os.path.exists(LIB) or not os.path.exists(STAMP):
        return None
    with open(STAMP) as f:
        return f.read().strip()


def needs_build() -> bool:
    """True when the library is missing or was built from other sources than the ones in the tree (by content,
    not by time stamps: copies of the tree do not keep those)."""
    return built_hash() != source_hash()


if __name__ == "__main__":
    build()

"""Builds libconv1d_hostmodel.so: the library's HIP sources compiled as plain host C++ against hip_cpu_shim.h.

The sources are used as they are, with one textual change: `extern __shared__ T name[];` (the dynamic LDS of a
kernel) becomes a pointer to the model's guard-paged LDS block.  Compiler: the clang++ that ships with ROCm (the
kernels use clang's vector extensions and __bf16); no GPU and no hipcc pass is involved.
"""
from __future__ import annotations

import concurrent.futures
import hashlib
import os
import re
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
CSRC = os.path.join(ROOT, "paper_2104_08002_amd", "csrc")
OUT = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libconv1d_hostmodel.so")
CLANG = "/opt/rocm/lib/llvm/bin/clang++"
FLAGS = ["-std=c++17", "-O1", "-fPIC", "-w", "-fbracket-depth=1024", "-fmax-type-align=2", "-I", OUT, "-I", HERE]
SHARED = re.compile(r"extern\s+__shared__\s+(\w+)\s+(\w+)\[\];")


def _hash() -> str:
    h = hashlib.sha256()
    for d in (CSRC, HERE):
        for f in sorted(os.listdir(d)):
            if f.endswith((".hip", ".h", ".cpp", ".py")):
                h.update(f.encode())
                h.update(open(os.path.join(d, f), "rb").read())
    h.update(open(os.path.join(ROOT, "include", "conv1d.h"), "rb").read())
    return h.hexdigest()[:16]


def _compile(src: str, flags) -> str:
    obj = src[:-4] + ".o"
    r = subprocess.run([CLANG, *flags, "-c", src, "-o", obj], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"host model: {os.path.basename(src)} does not compile:\n{r.stderr[-4000:]}")
    return obj


def build(force: bool = False, mutate=None, tag: str = "") -> str:
    """mutate: {file name: function(text) -> text} applied to the model's COPY of a source (a test plants a known
    mistake this way and expects the model to find it); tag names that build and its library."""
    out, lib = (OUT, LIB) if not tag else (OUT + "_" + tag, LIB[:-3] + "_" + tag + ".so")
    stamp = os.path.join(out, "stamp")
    h = _hash()
    if not force and os.path.exists(lib) and os.path.exists(stamp) and open(stamp).read() == h:
        return lib
    if not os.path.exists(CLANG):
        raise RuntimeError("clang++ of ROCm not found")
    shutil.rmtree(out, ignore_errors=True)
    os.makedirs(os.path.join(out, "include"))
    # conv1d_internal.h reaches the public header as ../../include/conv1d.h
    os.makedirs(os.path.join(out, "sub", "csrc"))
    shutil.copy(os.path.join(ROOT, "include", "conv1d.h"), os.path.join(out, "include", "conv1d.h"))
    work = os.path.join(out, "sub", "csrc")
    os.makedirs(os.path.join(out, "hip"))
    open(os.path.join(out, "hip", "hip_runtime.h"), "w").write("// replaced by hip_cpu_shim.h in the host model\n")
    flags = [f if f != OUT else out for f in FLAGS]
    srcs = []
    for f in sorted(os.listdir(CSRC)):
        text = open(os.path.join(CSRC, f)).read()
        if mutate and f in mutate:
            changed = mutate[f](text)
            if changed == text:
                raise RuntimeError(f"the planted change did not apply to {f}")
            text = changed
        text = SHARED.sub(r"\1* \2 = static_cast<\1*>(hostmodel::dynamic_lds());", text)
        if f.endswith(".hip"):
            dst = os.path.join(work, f[:-4] + ".cpp")
            text = '#include "hip_cpu_shim.h"\n' + text
            srcs.append(dst)
        else:
            dst = os.path.join(work, f)
        open(dst, "w").write(text)
    shutil.copy(os.path.join(HERE, "model.cpp"), os.path.join(work, "model_runtime.cpp"))
    srcs.append(os.path.join(work, "model_runtime.cpp"))
    with concurrent.futures.ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(lambda src: _compile(src, flags), srcs))
    r = subprocess.run([CLANG, "-shared", "-fPIC", "-o", lib, *objs], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("host model: link failed:\n" + r.stderr[-4000:])
    open(stamp, "w").write(h)
    return lib


if __name__ == "__main__":
    print(build(force=True))

"""Measured roofline denominators: MFMA-only loops (bf16, fp32) and a plain device copy.

``python -m paper_2104_08002_amd.ubench`` prints them; ``measure()`` returns them as a dict for the benchmark
driver.  The kernels live in ``peaks.hip`` (built into ``libconv1d_ubench.so`` next to it by ``build()``).
"""
from __future__ import annotations

import ctypes
import os
import shutil
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(_HERE, "peaks.hip")
LIB = os.path.join(_HERE, "libconv1d_ubench.so")

MFMA_SHAPES = {0: "bf16_32x32x16", 1: "fp32_32x32x2", 2: "fp32_16x16x4", 3: "fp32_16x16x4_1wave_4acc",
               4: "fp32_16x16x4_1wave_8acc", 5: "fp32_32x32x2_1wave_4acc", 6: "bf16_16x16x32",
               7: "bf16_16x16x32_1wave_8acc", 8: "bf16_16x16x32_1wave_13acc"}
COPY_SIZES_MB = (64, 256, 1024)


def build() -> str:
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", SRC, "-o", LIB]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for peaks.hip:\n" + r.stdout + r.stderr)
    return LIB


def measure() -> dict:
    """Run every microbenchmark once on the current GPU (about a second in total)."""
    if not os.path.exists(LIB):
        build()
    lib = ctypes.CDLL(LIB)
    lib.conv1d_ubench_mfma_tflops.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_double)]
    lib.conv1d_ubench_copy_gbps.argtypes = [ctypes.c_size_t, ctypes.POINTER(ctypes.c_double)]
    lib.conv1d_ubench_stream_gbps.argtypes = [ctypes.c_int, ctypes.c_size_t, ctypes.POINTER(ctypes.c_double)]
    lib.conv1d_ubench_device.argtypes = [ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
    out = {}
    cu, mhz = ctypes.c_int(), ctypes.c_int()
    if lib.conv1d_ubench_device(ctypes.byref(cu), ctypes.byref(mhz)) == 0:
        out["compute_units"], out["nominal_clock_mhz"] = cu.value, mhz.value
    v = ctypes.c_double()
    for shape, name in MFMA_SHAPES.items():
        if lib.conv1d_ubench_mfma_tflops(shape, ctypes.byref(v)) != 0:
            raise RuntimeError(f"MFMA microbenchmark {name} failed")
        out["mfma_" + name + "_tflops"] = round(v.value, 1)
    for mb in COPY_SIZES_MB:
        if lib.conv1d_ubench_copy_gbps(mb << 20, ctypes.byref(v)) != 0:
            raise RuntimeError(f"copy microbenchmark {mb} MB failed")
        out[f"copy_{mb}MB_gbps"] = round(v.value, 1)
    for mode, name in ((0, "fill"), (1, "read")):
        for mb in COPY_SIZES_MB:
            if lib.conv1d_ubench_stream_gbps(mode, mb << 20, ctypes.byref(v)) != 0:
                raise RuntimeError(f"{name} microbenchmark {mb} MB failed")
            out[f"{name}_{mb}MB_gbps"] = round(v.value, 1)
    out["mfma_bf16_tflops"] = out["mfma_bf16_32x32x16_tflops"]
    out["mfma_fp32_tflops"] = out["mfma_fp32_32x32x2_tflops"]
    out["hbm_copy_gbps"] = out["copy_1024MB_gbps"]
    # the dense bf16 peak of 2.5 PFLOP/s is quoted at 2.4 GHz: the MFMA-only rate bounds the sustained clock from below
    out["implied_clock_ghz_at_least"] = round(2.4 * out["mfma_bf16_tflops"] / 2516.6, 2)
    return out

"""Helpers shared by the GPU parity tests: run one pass through the C ABI, run the oracle
on the same numbers, and reduce to the parity metric  max |gpu - oracle| / sum|products|."""
from __future__ import annotations

import json
import os

import numpy as np

# The bar of the parity metric: 1e-5 for fp32 inputs, 1e-2 for bf16 inputs.
TOL = {"fp32": 1e-5, "bf16": 1e-2}
# What the arithmetic supports, and what every test asserts: bf16 products are exact in FP32 and are
# accumulated in FP32, so a bf16 pass has the same rounding error as an fp32 pass (n terms: at most
# n * 2^-24 of the summed magnitudes, ~sqrt(n) * 2^-24 typically; n <= 2304 here).  A wrongly masked channel,
# tap or column shows up at 1e-3 .. 1e-2, far above this bound and below the 1e-2 bar.
REGRESSION_TOL = {"fp32": 1e-5, "bf16": 1e-5}

_ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
_ERR_TABLE = os.path.join(_ROOT, "gpurun_out", "parity_errors.jsonl")


def record(case: str, variant: str, errs: dict) -> None:
    """Append one line per compared case to the per-case error table (a JSON-lines file in the run's output folder)."""
    try:
        os.makedirs(os.path.dirname(_ERR_TABLE), exist_ok=True)
        with open(_ERR_TABLE, "a") as f:
            f.write(json.dumps({"case": case, "variant": variant, "max_rel_err": errs}) + "\n")
    except OSError:
        pass


def assert_parity(case: str, variant: str, dtype: str, errs: dict) -> None:
    record(case, variant, errs)
    print(case, variant, errs, flush=True)
    for p, e in errs.items():
        assert e <= TOL[dtype], (case, variant, p, e, "above the parity bar")
        assert e <= REGRESSION_TOL[dtype], (case, variant, p, e, "above the bound FP32 accumulation supports")


def to_device(wl, data):
    """Move a workload's tensors to the GPU in their storage dtype."""
    import torch

    out = {}
    for k in ("x", "w", "dy"):
        if wl.dtype == "bf16":
            out[k] = torch.from_numpy(data[k + "_bits"].view(np.int16)).cuda().view(torch.bfloat16)
        else:
            out[k] = torch.from_numpy(data[k]).cuda()
    return out


def rel_err(gpu: np.ndarray, ref: np.ndarray, scale: np.ndarray) -> float:
    """max over elements of |gpu-ref|/scale; an element whose scale is 0 must be exactly 0."""
    gpu = np.asarray(gpu, dtype=np.float64)
    assert gpu.shape == ref.shape == scale.shape, (gpu.shape, ref.shape, scale.shape)
    assert np.isfinite(gpu).all(), "non-finite value in GPU output"
    zero = scale == 0
    if zero.any():
        assert not gpu[zero].any(), "nonzero output where every product is zero"
    if zero.all():
        return 0.0
    return float(np.max(np.abs(gpu - ref)[~zero] / scale[~zero]))


def gpu_passes(wl, dev, passes=("fwd", "bwd_data", "bwd_weight")):
    """Run the requested passes through the binding; returns {pass: numpy float32 array}."""
    import torch

    from paper_2104_08002_amd import binding

    res = {}
    if "fwd" in passes:
        res["fwd"] = binding.conv1d_fwd(dev["x"], dev["w"], wl.d, wl.P)
    if "bwd_data" in passes:
        res["bwd_data"] = binding.conv1d_bwd_data(dev["dy"], dev["w"], wl.W, wl.d, wl.P)
    if "bwd_weight" in passes:
        res["bwd_weight"] = binding.conv1d_bwd_weight(dev["x"], dev["dy"], wl.S, wl.d, wl.P)
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in res.items()}


def check_full(oracle, wl, data, got, passes=("fwd", "bwd_data", "bwd_weight")):
    """Element-by-element comparison with the full oracle output; returns {pass: max rel err}."""
    x, w, dy = (data[k].astype(np.float64) for k in ("x", "w", "dy"))
    errs = {}
    if "fwd" in passes:
        ref, sc = oracle.fwd(x, w, wl.d, wl.P, with_abs=True)
        errs["fwd"] = rel_err(got["fwd"], ref, sc)
    if "bwd_data" in passes:
        ref, sc = oracle.bwd_data(dy, w, wl.W, wl.d, wl.P, with_abs=True)
        errs["bwd_data"] = rel_err(got["bwd_data"], ref, sc)
    if "bwd_weight" in passes:
        ref, sc = oracle.bwd_weight(x, dy, wl.S, wl.d, wl.P, with_abs=True)
        errs["bwd_weight"] = rel_err(got["bwd_weight"], ref, sc)
    return errs


def sample_coords(rng, dims, count, edge):
    """`count` random coordinates in a (a, b, width) box, a third of them within `edge`
    columns of either end of the width axis (where padding and tile tails live)."""
    a = rng.integers(0, dims[0], count)
    b = rng.integers(0, dims[1], count)
    col = rng.integers(0, dims[2], count)
    e = max(1, min(edge, dims[2]))
    third = count // 3
    col[:third // 2] = rng.integers(0, e, third // 2)
    col[third // 2:third] = dims[2] - 1 - rng.integers(0, e, third - third // 2)
    return np.stack([a, b, col], axis=1).astype(np.int64)


def check_sampled(oracle, wl, data, got, rng, count=3000, wcount=300, passes=("fwd", "bwd_data", "bwd_weight")):
    """Comparison on sampled outputs, each evaluated one by one by the oracle."""
    x, w, dy = (data[k].astype(np.float64) for k in ("x", "w", "dy"))
    halo = (wl.S - 1) * wl.d + 64
    errs = {}
    if "fwd" in passes:
        idx = sample_coords(rng, (wl.N, wl.K, wl.Q), count, halo)
        ref, sc = oracle.fwd_at(x, w, idx, wl.d, wl.P)
        errs["fwd"] = rel_err(got["fwd"][idx[:, 0], idx[:, 1], idx[:, 2]], ref, sc)
    if "bwd_data" in passes:
        idx = sample_coords(rng, (wl.N, wl.C, wl.W), count, halo)
        ref, sc = oracle.bwd_data_at(dy, w, idx, wl.W, wl.d, wl.P)
        errs["bwd_data"] = rel_err(got["bwd_data"][idx[:, 0], idx[:, 1], idx[:, 2]], ref, sc)
    if "bwd_weight" in passes:
        n = min(wcount, wl.K * wl.C * wl.S)
        flat = rng.choice(wl.K * wl.C * wl.S, size=n, replace=False)
        idx = np.stack(np.unravel_index(flat, (wl.K, wl.C, wl.S)), axis=1).astype(np.int64)
        ref, sc = oracle.bwd_weight_at(x, dy, idx, wl.S, wl.d, wl.P)
        errs["bwd_weight"] = rel_err(got["bwd_weight"][idx[:, 0], idx[:, 1], idx[:, 2]], ref, sc)
    return errs

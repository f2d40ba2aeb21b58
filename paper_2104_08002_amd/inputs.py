"""Seeded synthetic workloads for the 1D dilated convolution layer.

This module holds no arithmetic of the method: it only names the layer
geometries that are measured and draws their tensors.  Both the FP64 oracle's
tests and the HIP path's tests/benchmark take their inputs from here, so the
two sides always see the same numbers.  It imports nothing else from this
package.

Shapes follow the paper's experiments: the AtacWorks layer (15 channels, 15
filters, filter width 51, dilation 8, segments of 50000 padded to 60000;
Section 4.2) and the efficiency sweep over filter width and dilation with 64
channels/filters (Section 4.3).  The ATAC-seq data itself is not available;
a sparse non-negative track (80 % exact zeros, the rest exponential) stands in
for a coverage signal.

Draw order is always x, w, dy from one ``numpy.random.Generator(PCG64(seed))``
in float32.  BF16 workloads round those float32 draws to bfloat16 once, here
(round-to-nearest-even), and both sides consume the rounded values.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Iterator, Tuple

import numpy as np

BASE_SEED = 20210408


@dataclass(frozen=True)
class Workload:
    name: str
    N: int
    C: int
    K: int
    W: int
    S: int
    d: int
    P: int
    dtype: str          # "fp32" or "bf16": storage type of x, w, dy (outputs are fp32)
    x_dist: str         # "uniform" | "normal" | "sparse_exp"
    w_dist: str         # "uniform" | "normal_fan" (variance 1/(C*S))
    dy_dist: str        # "uniform" | "normal"
    seed: int

    @property
    def Q(self) -> int:
        return self.W + 2 * self.P - (self.S - 1) * self.d

    @property
    def flops(self) -> int:
        """Nominal FLOPs of one pass: 2*N*C*K*S*Q."""
        return 2 * self.N * self.C * self.K * self.S * self.Q

    def geometry(self) -> Tuple[int, int, int, int, int, int, int]:
        return (self.N, self.C, self.K, self.W, self.S, self.d, self.P)


def same_padding(S: int, d: int) -> int:
    """Zeros per side that keep Q == W for odd S (Fig. 1: S=3, d=3 -> 3 per side)."""
    return (S - 1) * d // 2


TINY = Workload("tiny_fp32", 2, 4, 4, 256, 5, 2, 0, "fp32", "uniform", "uniform", "normal",
                BASE_SEED + 0)
GENOMICS_FP32 = Workload("genomics_fp32", 16, 15, 15, 60000, 51, 8, same_padding(51, 8), "fp32",
                         "sparse_exp", "normal_fan", "normal", BASE_SEED + 1)
GENOMICS_BF16 = replace(GENOMICS_FP32, name="genomics_bf16", dtype="bf16", seed=BASE_SEED + 2)
WIDE_BF16 = Workload("wide_bf16", 32, 256, 256, 8192, 9, 4, same_padding(9, 4), "bf16",
                     "normal", "normal_fan", "normal", BASE_SEED + 4)

SWEEP_S = (5, 9, 17, 33, 51)
SWEEP_D = (1, 2, 4, 8, 16)


def sweep_point(S: int, d: int, dtype: str) -> Workload:
    i_s, i_d = SWEEP_S.index(S), SWEEP_D.index(d)
    return Workload(f"sweep_{dtype}_S{S}_d{d}", 8, 64, 64, 20000, S, d, same_padding(S, d), dtype,
                    "uniform", "uniform", "uniform", BASE_SEED + 3 + 100 * i_s + i_d)


def sweep(dtype: str) -> Iterator[Workload]:
    for S in SWEEP_S:
        for d in SWEEP_D:
            yield sweep_point(S, d, dtype)


# The paper's own single-layer grid (Section 4.3, the axes of Figs. 4-6): batch 56, output widths 1000 ... 60000,
# for 15 channels and filters at dilation 8 (FP32, Fig. 4), 64 at dilation 1 (FP32, Fig. 5), and 32 and 16 at
# dilation 4 in BF16 (Fig. 6 and the BF16 training shape of Section 4.4).  Same padding, all tensors U[-1,1].
Q_SWEEP_Q = (1000, 2000, 5000, 10000, 20000, 60000)
Q_SWEEP_S = (1, 5, 9, 15, 21, 25, 31, 49, 51)
Q_SWEEP_FAMILIES = {
    "c15_d8_fp32": (15, 8, "fp32"),
    "c64_d1_fp32": (64, 1, "fp32"),
    "c32_d4_bf16": (32, 4, "bf16"),
    "c16_d4_bf16": (16, 4, "bf16"),
}
Q_SWEEP_N = 56


def q_sweep_point(family: str, Q: int, S: int) -> Workload:
    ch, d, dtype = Q_SWEEP_FAMILIES[family]
    i_f = list(Q_SWEEP_FAMILIES).index(family)
    return Workload(f"q_{family}_S{S}_Q{Q}", Q_SWEEP_N, ch, ch, Q, S, d, same_padding(S, d), dtype,
                    "uniform", "uniform", "uniform",
                    BASE_SEED + 10000 + 1000 * i_f + 10 * Q_SWEEP_S.index(S) + Q_SWEEP_Q.index(Q))


WORKLOADS: Dict[str, Workload] = {w.name: w for w in (TINY, GENOMICS_FP32, GENOMICS_BF16, WIDE_BF16)}
WORKLOADS.update({w.name: w for dt in ("fp32", "bf16") for w in sweep(dt)})
for _dt in ("fp32", "bf16"):
    for _w in sweep(_dt):
        WORKLOADS[_w.name] = _w


def scaled(wl: Workload, **kw) -> Workload:
    """Same distributions and seed family with some dimensions changed (for small parity cases)."""
    return replace(wl, **kw)


# ---------------------------------------------------------------------------
# bfloat16 storage helpers (bit manipulation only)
# ---------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest even) and return the uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns to float32 exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _draw(rng: np.random.Generator, dist: str, shape, fan: int) -> np.ndarray:
    if dist == "uniform":
        return rng.uniform(-1.0, 1.0, size=shape).astype(np.float32)
    if dist == "normal":
        return rng.standard_normal(size=shape, dtype=np.float32)
    if dist == "normal_fan":
        return (rng.standard_normal(size=shape, dtype=np.float32) / np.float32(np.sqrt(fan))).astype(np.float32)
    if dist == "sparse_exp":
        keep = rng.random(size=shape, dtype=np.float32) < np.float32(0.2)
        vals = rng.standard_exponential(size=shape, dtype=np.float32)
        return np.where(keep, vals, np.float32(0.0)).astype(np.float32)
    raise ValueError(dist)


def make_inputs(wl: Workload) -> Dict[str, np.ndarray]:
    """Draw x (N,C,W), w (K,C,S), dy (N,K,Q) as float32 arrays.

    For a bf16 workload the float32 arrays hold bfloat16-representable values
    and ``x_bits`` / ``w_bits`` / ``dy_bits`` hold the matching uint16 patterns.
    """
    rng = np.random.Generator(np.random.PCG64(wl.seed))
    x = _draw(rng, wl.x_dist, (wl.N, wl.C, wl.W), 1)
    w = _draw(rng, wl.w_dist, (wl.K, wl.C, wl.S), wl.C * wl.S)
    dy = _draw(rng, wl.dy_dist, (wl.N, wl.K, wl.Q), 1)
    out = {"x": x, "w": w, "dy": dy}
    if wl.dtype == "bf16":
        for k in ("x", "w", "dy"):
            bits = f32_to_bf16_bits(out[k])
            out[k + "_bits"] = bits
            out[k] = bf16_bits_to_f32(bits)
    elif wl.dtype != "fp32":
        raise ValueError(wl.dtype)
    return out

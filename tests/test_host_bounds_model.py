"""Host-side bounds model: every kernel of the library, compiled as CPU code (tests/hostmodel), is run thread by
thread on seeded geometries with each tensor of the call surrounded by inaccessible address space; any global-memory
address outside its tensor (a wrong sample index, an unclamped halo, a tail that is not masked) stops the run and is
reported with the workgroup and thread that formed it.  No GPU is involved: this is how an off-by-one in the
producers' request arithmetic is found without a memory fault on the device.
"""
import ctypes
import os
import sys

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.join(HERE, "hostmodel"))

PASS_NAMES = ("fwd", "bwd_data", "bwd_weight", "bwd", "fwd_ex", "bwd_data_ex")


def _load(path):
    lib = ctypes.CDLL(path)
    lib.hostmodel_run.argtypes = [ctypes.c_int] * 11 + [ctypes.c_char_p, ctypes.c_int]
    lib.hostmodel_run.restype = ctypes.c_int
    return lib


@pytest.fixture(scope="module")
def model():
    import build as hostmodel_build

    return _load(hostmodel_build.build())


def _run(lib, ps, geom, dtype, variant=0, placement=0):
    msg = ctypes.create_string_buffer(512)
    rc = lib.hostmodel_run(ps, *geom, dtype, variant, placement, msg, 512)
    return rc, msg.value.decode()


def _check(lib, geom, dtype, passes=range(6), placements=(0, 1), variant=0):
    ran = 0
    for ps in passes:
        for pl in placements:
            rc, msg = _run(lib, ps, geom, dtype, variant, pl)
            if rc == 102:        # CONV1D_EUNSUPPORTED: a forced family that cannot run this geometry
                continue
            assert rc == 0, f"{PASS_NAMES[ps]} {geom} dtype {dtype} placement {pl} variant {variant}: rc {rc} {msg}"
            ran += 1
    return ran


def _curated():
    sys.path.insert(0, HERE)
    import test_gpu_parity as t

    cases = [c[1:] for c in t.SMALL] + [c[1:] for c in t.UNALIGNED]
    cases += [(2, 4, 4, 256, 5, 2, 0), (3, 15, 15, 5000, 51, 8, 200), (2, 15, 15, 4096 + 37, 51, 8, 200),
              (2, 64, 64, 3007, 51, 8, 200), (2, 64, 64, 3007, 5, 1, 2), (2, 256, 256, 1000, 9, 4, 16)]
    return cases


@pytest.mark.parametrize("dtype", [0, 1], ids=["fp32", "bf16"])
def test_curated_geometries_stay_inside_their_tensors(model, dtype):
    """The geometries of the GPU parity suite (every kernel family, odd sizes, halos wider than the row, the shape of
    the one memory fault this library ever had), every entry point, tensors flush against the guard on either side."""
    n = 0
    for geom in _curated():
        if max(geom[1], geom[2]) > 600:      # the streamed-weight shapes: forward and backward-data only (seconds each)
            n += _check(model, geom, dtype, passes=(0, 1), placements=(0, 1))
        else:
            n += _check(model, geom, dtype)
    assert n > 300


def test_element_aligned_tensors(model):
    """Every tensor shifted by one element inside its allocation: the kernels' unaligned paths."""
    for geom in [(2, 15, 15, 3000, 51, 8, 200), (1, 64, 64, 1536, 51, 8, 200), (2, 64, 64, 1200, 9, 2, 8),
                 (2, 40, 24, 2000, 33, 4, 64), (2, 9, 13, 1777, 25, 3, 36), (1, 256, 256, 600, 9, 4, 16)]:
        for dtype in (0, 1):
            _check(model, geom, dtype, placements=(2,))


def test_forced_kernel_families(model):
    for variant in (1, 2, 3):
        for geom in [(2, 4, 4, 256, 5, 2, 0), (2, 15, 13, 2500, 25, 3, 36), (2, 17, 33, 1200, 9, 2, 8), (1, 64, 64, 2500, 33, 16, 256)]:
            for dtype in (0, 1):
                _check(model, geom, dtype, passes=(0, 1, 2), placements=(0,), variant=variant)


def _random_geometry(rng):
    d = int(rng.choice([1, 1, 2, 2, 3, 4, 4, 5, 7, 8, 8, 8, 16, 16]))
    S = int(rng.choice([1, 2, 3, 4, 5, 7, 9, 12, 15, 17, 20, 21, 25, 31, 33, 49, 51, 52, 53, 70]))
    kind = rng.integers(0, 10)
    if kind < 4:
        C, K = int(rng.integers(1, 17)), int(rng.integers(1, 17))
    elif kind < 8:
        C, K = int(rng.integers(17, 97)), int(rng.integers(17, 97))
    else:
        C, K = int(rng.integers(100, 300)), int(rng.integers(100, 300))
    if S > 52:  # the plain-FMA kernels start one workgroup per weight-gradient element: keep that count small
        C, K = min(C, 24), min(K, 24)
    span = (S - 1) * d
    W = int(rng.choice([rng.integers(1, 64), rng.integers(64, 700), rng.integers(700, 2600), 8 * rng.integers(8, 300)]))
    P = int(rng.choice([0, span // 2, rng.integers(0, span + 1), span + int(rng.integers(0, 9)), 8 * (span // 16)]))
    N = int(rng.integers(1, 4))
    if W + 2 * P - span < 1:
        W = span - 2 * P + int(rng.integers(1, 40))
    # the model runs every thread of every workgroup on one core: bound the work of a geometry
    while N * C * K * S * (W + 2 * P - span) > 3e7 and W - (W + 2 * P - span) // 2 >= 1:
        W -= (W + 2 * P - span) // 2
    return (N, C, K, W, S, d, P)


def test_seeded_random_geometries(model):
    rng = np.random.default_rng(20210408)
    ran = 0
    for i in range(800):
        geom = _random_geometry(rng)
        dtype = i & 1
        # forward, backward-data and backward-weight always; the combined and fused entry points on every fourth one
        passes = range(6) if i % 4 == 0 else (0, 1, 2)
        ran += _check(model, geom, dtype, passes=passes, placements=(i // 2 % 2,))
    assert ran >= 2400


def test_seeded_random_few_tap_small_dilation(model):
    """The corner of the register-shift backward-weight kernel and the light prologue paths of the resident-weight
    kernel: bfloat16, 2-17 taps at dilations 1, 2, 4, any padding up to a little beyond the span."""
    rng = np.random.default_rng(20210409)
    ran = 0
    for i in range(150):
        N, C, K, W, S, d, P = _random_geometry(rng)
        d = int(rng.choice([1, 2, 4]))
        S = int(rng.integers(2, 18))
        if (S - 1) * d > 32:
            S = 32 // d + 1
        P = int(rng.integers(0, (S - 1) * d + 9))
        if W + 2 * P - (S - 1) * d < 1:
            W = (S - 1) * d + 5
        ran += _check(model, (N, C, K, W, S, d, P), 1, passes=(0, 1, 2), placements=(i % 2,))
    assert ran >= 450


def test_the_model_finds_a_planted_off_by_one():
    """The one GPU memory fault in this library's history: the streamed-weight kernel asked for a stage behind its
    counters and took its sample index one past the batch.  With that repair removed from the model's copy of the
    source, the geometry that faulted must be reported (and the unchanged source must pass it)."""
    import build as hostmodel_build

    repair = """            while (cc < 0) {
                cc += a.ncc;
                if (tc-- == 0) {
                    tc = a.tiles_per_row - 1;
                    --n;
                }
            }
"""
    lib = _load(hostmodel_build.build(mutate={"conv1d_igemm_stream_bf16.hip": lambda t: t.replace(repair, "")},
                                      tag="planted_stream"))
    geom = (4, 232, 1056, 200, 17, 2, 16)
    rc, msg = _run(lib, 0, geom, 1)
    assert rc == 1 and "outside x" in msg, (rc, msg)
    assert _run(_load(hostmodel_build.build()), 0, geom, 1)[0] == 0


def test_multiply_high_division_is_exact(model):
    """The kernels divide small indices by launch constants with one multiply-high; the host accepts a divisor only with
    the largest dividend it was checked for.  Every accepted (divisor, bound) pair is compared with the plain quotient
    over its whole range; pairs the host refuses are counted, not trusted."""
    import ctypes as ct

    model.hostmodel_fastdiv_mismatch.argtypes = [ct.c_long, ct.c_long]
    model.hostmodel_fastdiv_mismatch.restype = ct.c_long
    rng = np.random.default_rng(7)
    divisors = list(range(1, 70)) + [95, 117, 118, 188, 255, 256, 257, 626, 641, 1000, 1023, 4097, 65535, 65537] + \
        [int(v) for v in rng.integers(2, 200000, 40)]
    accepted = refused = 0
    for d in divisors:
        for nmax in (d - 1, 5 * d + 3, 70000, 1 << 20):
            r = model.hostmodel_fastdiv_mismatch(d, nmax)
            assert r in (-1, -2), f"fast_div({r}, {d}) differs from {r} // {d} although the bound {nmax} was accepted"
            accepted += r == -1
            refused += r == -2
    assert accepted > 300 and refused < accepted

"""conv1d_fwd_ex / conv1d_bwd_data_ex (fused bias, ReLU, bfloat16 storage) against the oracle's epilogue, through
the C ABI, for every kernel family.

Float output: |gpu - oracle| <= tol * (sum|products| + |bias|), the bar of the plain passes (ReLU is 1-Lipschitz).
bfloat16 output: rounding is a decision, and the two sides round values that differ by FP32 summation error, so the
test asks for what is unique: rounding and ReLU are monotone, hence the GPU value must lie between the oracle's
epilogue applied to (z - tol*A) and to (z + tol*A), z the oracle's pre-activation in FP64.  Away from rounding
boundaries that interval is a single bfloat16 value.
"""
import numpy as np
import pytest

from paper_2104_08002_amd import inputs
from parity_util import REGRESSION_TOL, record, rel_err, to_device

pytestmark = pytest.mark.gpu

VARIANTS = {"auto": 0, "generic": 1}


@pytest.fixture(scope="module")
def binding():
    import torch

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2104_08002_amd import binding as b

    b.load()
    yield b
    b.conv1d_set_variant(0)


CASES = [
    # name               N  C    K    W     S   d   P     kernel the auto choice lands on
    ("epi_genomics",     2, 15,  15,  5000, 51, 8,  200),   # small-channel MFMA
    ("epi_genomics_k9",  3, 12,  9,   4104, 51, 8,  200),   # small-channel MFMA, fewer than 15 filters: general output flush
    ("epi_smallc_d3",    2, 9,   13,  1777, 25, 3,  36),  # small-channel, no operand sharing, odd width
    ("epi_ring_S51",     1, 64,  64,  2100, 51, 8,  200), # resident weights
    ("epi_ring_k40",     2, 72,  40,  1000, 7,  4,  12),
    ("epi_stream",       4, 200, 1056, 1100, 9, 4,  16),  # streamed weights
    ("epi_staged_d3",    2, 40,  24,  2500, 9,  3,  12),  # staged many-channel kernel
    ("epi_c64_S9",       2, 64,  64,  1100, 9,  1,  4),   # fp32: one launch, channel blocks in the accumulators
    ("epi_c64_S51",      1, 64,  64,  1536, 51, 8,  200), # fp32: one launch per channel block, epilogue kernel at the end
    ("epi_pairs_oddW",   2, 40,  24,  901,  7,  3,  9),   # odd width: 16 x 16 block launches
    ("epi_tiny",         2, 4,   4,   256,  5,  2,  0),
]
EPILOGUES = [
    # bias, relu, out_bf16
    (True, False, False),
    (False, True, False),
    (True, True, False),
    (True, True, True),
    (False, False, True),
]


def _wl(case, dtype):
    name, N, C, K, W, S, d, P = case
    return inputs.scaled(inputs.TINY, name=f"{name}_{dtype}", N=N, C=C, K=K, W=W, S=S, d=d, P=P, dtype=dtype,
                         x_dist="normal", w_dist="normal_fan", dy_dist="normal", seed=inputs.BASE_SEED + 5000 + len(name))


def _bias(wl):
    # seeded like the tensors; large enough to flip signs of many outputs under ReLU
    return np.random.default_rng(wl.seed + 1).standard_normal(wl.K).astype(np.float32)


def _check(oracle, z, A, got, relu, out_bf16, tol, what):
    got = np.asarray(got, dtype=np.float64)
    assert np.isfinite(got).all(), what
    if not out_bf16:
        ref = oracle.epilogue(z.copy(), None, relu, False)
        return rel_err(got, ref, A)
    lo = oracle.epilogue(z - tol * A, None, relu, True)
    hi = oracle.epilogue(z + tol * A, None, relu, True)
    bad = (got < lo) | (got > hi)
    assert not bad.any(), (what, int(bad.sum()), "values outside the rounding interval")
    exact = oracle.epilogue(z.copy(), None, relu, True)
    return float(np.mean(got != exact))      # fraction that sits on the other side of a rounding boundary


@pytest.mark.parametrize("variant", list(VARIANTS))
@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_fused_epilogue(binding, oracle, case, dtype, variant):
    import torch

    wl = _wl(case, dtype)
    data = inputs.make_inputs(wl)
    dev = to_device(wl, data)
    b32 = _bias(wl)
    bias = torch.from_numpy(b32).cuda()
    x, w, dy = (data[k].astype(np.float64) for k in ("x", "w", "dy"))
    tol = REGRESSION_TOL[dtype]
    z0, A0 = oracle.fwd(x, w, wl.d, wl.P, with_abs=True)
    errs = {}
    binding.conv1d_set_variant(VARIANTS[variant])
    try:
        for use_bias, relu, out_bf16 in EPILOGUES:
            if out_bf16 and dtype != "bf16":
                with pytest.raises(binding.Conv1dError):
                    binding.conv1d_fwd_ex(dev["x"], dev["w"], wl.d, wl.P, relu=relu, out_bf16=True)
                continue
            y = binding.conv1d_fwd_ex(dev["x"], dev["w"], wl.d, wl.P, bias=bias if use_bias else None, relu=relu,
                                      out_bf16=out_bf16)
            torch.cuda.synchronize()
            z, A = z0.copy(), A0.copy()
            if use_bias:
                oracle.epilogue(z, b32.astype(np.float64), False, False, A)
            key = f"fwd{'+bias' if use_bias else ''}{'+relu' if relu else ''}{'+bf16' if out_bf16 else ''}"
            errs[key] = _check(oracle, z, A, y.float().cpu().numpy(), relu, out_bf16, tol, (wl.name, key))
            if not out_bf16:
                assert errs[key] <= tol, (wl.name, variant, key, errs[key])
        if dtype == "bf16":
            dx = binding.conv1d_bwd_data_ex(dev["dy"], dev["w"], wl.W, wl.d, wl.P, out_bf16=True)
            torch.cuda.synchronize()
            z, A = oracle.bwd_data(dy, w, wl.W, wl.d, wl.P, with_abs=True)
            errs["bwd_data+bf16"] = _check(oracle, z, A, dx.float().cpu().numpy(), False, True, tol, (wl.name, "bwd_data+bf16"))
    finally:
        binding.conv1d_set_variant(0)
    record(wl.name, f"epilogue_{variant}", errs)
    print(wl.name, variant, errs, flush=True)


def test_fused_epilogue_genomics_full_size(binding, oracle):
    """The benchmarked shape, bf16 in and out with bias and ReLU: whole-output comparison."""
    import torch

    wl = inputs.GENOMICS_BF16
    data = inputs.make_inputs(wl)
    dev = to_device(wl, data)
    b32 = _bias(wl)
    y = binding.conv1d_fwd_ex(dev["x"], dev["w"], wl.d, wl.P, bias=torch.from_numpy(b32).cuda(), relu=True, out_bf16=True)
    dx = binding.conv1d_bwd_data_ex(dev["dy"], dev["w"], wl.W, wl.d, wl.P, out_bf16=True)
    torch.cuda.synchronize()
    x, w, dy = (data[k].astype(np.float64) for k in ("x", "w", "dy"))
    tol = REGRESSION_TOL["bf16"]
    z, A = oracle.fwd_ex(x, w, wl.d, wl.P, bias=b32.astype(np.float64), with_abs=True)
    f1 = _check(oracle, z, A, y.float().cpu().numpy(), True, True, tol, "genomics fwd+bias+relu+bf16")
    z, A = oracle.bwd_data(dy, w, wl.W, wl.d, wl.P, with_abs=True)
    f2 = _check(oracle, z, A, dx.float().cpu().numpy(), False, True, tol, "genomics bwd_data+bf16")
    record(wl.name, "epilogue_full", {"fwd_other_side_of_a_tie": f1, "bwd_data_other_side_of_a_tie": f2})
    assert f1 < 1e-3 and f2 < 1e-3      # such values are rare: FP32 summation error is ~1e-7 of a bfloat16 step of 4e-3

"""conv1d_bwd (both backward passes in one call) and the autograd wrapper, against the oracle and against the
separate entry points, through the C ABI."""
import numpy as np
import pytest

from paper_2104_08002_amd import inputs
from parity_util import REGRESSION_TOL, assert_parity, check_full, rel_err, to_device

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def binding():
    import torch

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2104_08002_amd import binding as b

    b.load()
    return b


CASES = [
    inputs.GENOMICS_BF16,                                                       # fused second stage (full size, 256 workgroups)
    inputs.scaled(inputs.GENOMICS_BF16, N=3, W=30000 + 8, name="bwd_genomics_bf16_mid"),   # 177 tiles: too few workgroups for the side job
    inputs.scaled(inputs.GENOMICS_BF16, N=7, W=20000, C=9, K=13, name="bwd_bf16_c9_k13"),
    inputs.scaled(inputs.GENOMICS_BF16, N=16, W=60000, S=33, P=128, name="bwd_bf16_S33"),
    inputs.scaled(inputs.GENOMICS_FP32, N=4, W=9000, name="bwd_genomics_fp32"),
    inputs.scaled(inputs.sweep_point(17, 4, "bf16"), N=2, W=5000, name="bwd_c64_bf16"),
    inputs.scaled(inputs.sweep_point(9, 2, "fp32"), N=2, W=3000, name="bwd_c64_fp32"),
    inputs.scaled(inputs.TINY, name="bwd_tiny"),
]


@pytest.mark.parametrize("wl", CASES, ids=lambda w: w.name)
def test_conv1d_bwd_matches_the_separate_passes_and_the_oracle(binding, oracle, wl):
    import torch

    data = inputs.make_inputs(wl)
    dev = to_device(wl, data)
    dx_ref = binding.conv1d_bwd_data(dev["dy"], dev["w"], wl.W, wl.d, wl.P)
    dw_ref = binding.conv1d_bwd_weight(dev["x"], dev["dy"], wl.S, wl.d, wl.P)
    dx = torch.full((wl.N, wl.C, wl.W), float("nan"), device="cuda")
    dw = torch.full((wl.K, wl.C, wl.S), float("nan"), device="cuda")
    for _ in range(2):      # twice: the second call finds the first one's partial sums in the workspace
        binding.conv1d_bwd(dev["x"], dev["dy"], dev["w"], wl.d, wl.P, out_dx=dx, out_dw=dw)
    torch.cuda.synchronize()
    assert torch.equal(dx, dx_ref) and torch.equal(dw, dw_ref), wl.name
    errs = check_full(oracle, wl, data, {"bwd_data": dx.cpu().numpy(), "bwd_weight": dw.cpu().numpy()},
                      passes=("bwd_data", "bwd_weight"))
    assert_parity(wl.name, "conv1d_bwd", wl.dtype, errs)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_autograd_wrapper(binding, oracle, dtype):
    """forward() and sum().backward() (the measurement protocol of Section 4.3), then a random upstream gradient."""
    import torch

    from paper_2104_08002_amd import autograd

    wl = inputs.scaled(inputs.GENOMICS_FP32, N=3, W=6000, dtype=dtype, name=f"autograd_{dtype}")
    data = inputs.make_inputs(wl)
    dev = to_device(wl, data)
    x, w = dev["x"].clone().requires_grad_(True), dev["w"].clone().requires_grad_(True)
    y = autograd.conv1d(x, w, None, wl.d, wl.P)
    y.sum().backward()
    torch.cuda.synchronize()
    xs, ws = data["x"].astype(np.float64), data["w"].astype(np.float64)
    ones = np.ones((wl.N, wl.K, wl.Q))
    tol = REGRESSION_TOL[dtype]
    ref, sc = oracle.fwd(xs, ws, wl.d, wl.P, with_abs=True)
    assert rel_err(y.detach().cpu().numpy(), ref, sc) <= tol
    # gradients come back in the parameter's dtype: for bf16 that is one rounding of the FP32 result
    slack = 2.0 ** -8 if dtype == "bf16" else 0.0
    ref, sc = oracle.bwd_data(ones, ws, wl.W, wl.d, wl.P, with_abs=True)
    assert rel_err(x.grad.float().cpu().numpy(), ref, sc + slack * np.abs(ref) / tol if slack else sc) <= tol
    ref, sc = oracle.bwd_weight(xs, ones, wl.S, wl.d, wl.P, with_abs=True)
    assert rel_err(w.grad.float().cpu().numpy(), ref, sc + slack * np.abs(ref) / tol if slack else sc) <= tol
    # module with a bias and a fused ReLU against the oracle's epilogue and torch's rule for the bias gradient
    layer = autograd.Conv1d(wl.C, wl.K, wl.S, dilation=wl.d, padding=wl.P, bias=True, relu=True,
                            dtype=torch.bfloat16 if dtype == "bf16" else torch.float32)
    with torch.no_grad():
        layer.weight.copy_(dev["w"])
        layer.bias.copy_(torch.linspace(-1, 1, wl.K))
    out = layer(dev["x"])
    g = dev["dy"].float()
    out.backward(g)
    torch.cuda.synchronize()
    b = np.linspace(-1, 1, wl.K).astype(np.float32).astype(np.float64)
    z, A = oracle.fwd_ex(xs, ws, wl.d, wl.P, bias=b, with_abs=True)
    assert rel_err(out.detach().cpu().numpy(), np.maximum(z, 0), A) <= tol
    # upstream gradient masked where the GPU's own output is zero (the decision is the kernel's, taken in FP32)
    mask = out.detach().cpu().numpy() > 0
    gm = data["dy"].astype(np.float64) * mask
    if dtype == "bf16":
        gm = inputs.bf16_bits_to_f32(inputs.f32_to_bf16_bits(gm.astype(np.float32))).astype(np.float64)
    ref, sc = oracle.bwd_weight(xs, gm, wl.S, wl.d, wl.P, with_abs=True)
    assert rel_err(layer.weight.grad.float().cpu().numpy(), ref, sc + slack * np.abs(ref) / tol if slack else sc) <= tol
    np.testing.assert_allclose(layer.bias.grad.cpu().numpy(), (data["dy"].astype(np.float64) * mask).sum(axis=(0, 2)), rtol=1e-4, atol=1e-3)

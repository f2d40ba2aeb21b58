"""conv1d_bwd_weight_noalloc (partial sums in the library's built-in device buffer) against conv1d_bwd_weight
(caller's workspace), through the C ABI: bit-identical weight gradients, on two calls in a row, the second one on a
smaller input, and both within the parity bar of the FP64 oracle."""
import ctypes

import numpy as np
import pytest

from paper_2104_08002_amd import inputs
from parity_util import REGRESSION_TOL, check_full, record, to_device

pytestmark = pytest.mark.gpu

CASES = [
    # first call, then a smaller one that leaves most of the buffer's old contents in place
    (inputs.GENOMICS_BF16, inputs.scaled(inputs.GENOMICS_BF16, N=3, W=7000 + 8, name="genomics_bf16_smaller")),
    (inputs.scaled(inputs.sweep_point(33, 4, "bf16"), N=4, W=12000), inputs.scaled(inputs.sweep_point(33, 4, "bf16"), N=1, W=3001)),
    (inputs.scaled(inputs.GENOMICS_FP32, N=8, W=30000), inputs.scaled(inputs.GENOMICS_FP32, N=2, W=2999)),
    (inputs.scaled(inputs.sweep_point(9, 2, "fp32"), N=2, W=9000), inputs.scaled(inputs.TINY)),
    (inputs.scaled(inputs.WIDE_BF16, N=4), inputs.scaled(inputs.WIDE_BF16, N=1, W=1000, name="wide_bf16_smaller")),
]


@pytest.fixture(scope="module")
def binding():
    import torch

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2104_08002_amd import binding as b

    b.load()
    return b


@pytest.mark.parametrize("pair", CASES, ids=[a.name for a, _ in CASES])
def test_noalloc_matches_workspace_entry_point(binding, oracle, pair):
    import torch

    lib = binding.load()
    for wl in pair:
        code = 1 if wl.dtype == "bf16" else 0
        need = binding.conv1d_bwd_weight_workspace_bytes(*wl.geometry(), code)
        assert 0 < need <= binding.NOALLOC_SCRATCH_BYTES, (wl.name, need)
        data = inputs.make_inputs(wl)
        dev = to_device(wl, data)
        ref = binding.conv1d_bwd_weight(dev["x"], dev["dy"], wl.S, wl.d, wl.P)
        dw = torch.full((wl.K, wl.C, wl.S), float("nan"), dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        st = lib.conv1d_bwd_weight_noalloc(dev["x"].data_ptr(), dev["dy"].data_ptr(), dw.data_ptr(), *wl.geometry(), code,
                                           ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
        assert st == 0, binding.conv1d_status_string(st)
        torch.cuda.synchronize()
        assert torch.equal(ref, dw), f"{wl.name}: the two entry points disagree"
        errs = check_full(oracle, wl, data, {"bwd_weight": dw.cpu().numpy()}, passes=("bwd_weight",))
        record(wl.name, "noalloc", errs)
        assert errs["bwd_weight"] <= REGRESSION_TOL[wl.dtype], (wl.name, errs)


def test_noalloc_rejects_what_does_not_fit(binding):
    import torch

    wl = inputs.scaled(inputs.sweep_point(51, 8, "bf16"), C=256, K=256)
    assert binding.conv1d_bwd_weight_workspace_bytes(*wl.geometry(), 1) > binding.NOALLOC_SCRATCH_BYTES
    x = torch.zeros((wl.N, wl.C, wl.W), dtype=torch.bfloat16, device="cuda")
    dy = torch.zeros((wl.N, wl.K, wl.Q), dtype=torch.bfloat16, device="cuda")
    dw = torch.full((wl.K, wl.C, wl.S), 7.0, dtype=torch.float32, device="cuda")
    with pytest.raises(binding.Conv1dError) as ei:
        binding.conv1d_bwd_weight_noalloc(x, dy, wl.S, wl.d, wl.P, out=dw)
    assert ei.value.status == -5 and "scratch" in str(ei.value)
    torch.cuda.synchronize()
    assert bool((dw == 7.0).all()), "a rejected call must not launch anything"

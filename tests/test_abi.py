"""The C-ABI library loads, exports what the header declares, and rejects bad arguments
before touching a GPU.  No kernel is launched here."""
import ctypes
import os
import re

import pytest

from paper_2104_08002_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return binding.load()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "conv1d.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(conv1d_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_out_width():
    assert binding.conv1d_out_width(17, 3, 3, 3) == 17          # Fig. 1 geometry
    assert binding.conv1d_out_width(256, 5, 2, 0) == 248
    assert binding.conv1d_out_width(60000, 51, 8, 200) == 60000
    assert binding.conv1d_out_width(5, 4, 3, 0) <= 0
    assert binding.conv1d_out_width(0, 1, 1, 0) <= 0
    assert binding.conv1d_out_width(10, 3, 0, 0) <= 0
    assert binding.conv1d_out_width(10, 3, 1, -1) <= 0


def test_status_strings(lib):
    seen = {binding.conv1d_status_string(s) for s in (0, -1, -2, -3, -4, -5)}
    assert len(seen) == 6 and binding.conv1d_status_string(0) == "ok"
    assert "unknown" in binding.conv1d_status_string(-99)


def test_argument_validation_without_gpu(lib):
    fake = ctypes.c_void_p(0x1000)          # never dereferenced: every call below fails validation
    g = (2, 4, 4, 256, 5, 2, 0)
    assert lib.conv1d_fwd(None, fake, fake, *g, 0, None) == -1
    assert lib.conv1d_fwd(fake, None, fake, *g, 0, None) == -1
    assert lib.conv1d_fwd(fake, fake, None, *g, 0, None) == -1
    assert lib.conv1d_fwd(fake, fake, fake, *g, 7, None) == -1                      # dtype
    assert lib.conv1d_fwd(fake, fake, fake, 0, 4, 4, 256, 5, 2, 0, 0, None) == -1   # N
    assert lib.conv1d_fwd(fake, fake, fake, 2, 4, 4, 256, 5, 0, 0, 0, None) == -1   # dilation
    assert lib.conv1d_fwd(fake, fake, fake, 2, 4, 4, 256, 5, 2, -1, 0, None) == -1  # padding
    assert lib.conv1d_fwd(fake, fake, fake, 2, 4, 4, 8, 5, 2, 0, 0, None) == -1     # Q <= 0
    assert lib.conv1d_fwd(ctypes.c_void_p(0x1002), fake, fake, *g, 0, None) == -1   # misaligned float
    assert lib.conv1d_fwd(ctypes.c_void_p(0x1001), fake, fake, *g, 1, None) == -1   # misaligned bf16
    assert lib.conv1d_bwd_data(None, fake, fake, *g, 0, None) == -1
    assert lib.conv1d_bwd_data(fake, fake, fake, 2, 4, 4, 8, 5, 2, 0, 1, None) == -1
    assert lib.conv1d_bwd_weight(fake, fake, fake, None, 0, *g, 0, None) == -3
    assert lib.conv1d_bwd_weight(fake, fake, fake, fake, 16, *g, 0, None) == -3
    assert lib.conv1d_bwd_weight(None, fake, fake, fake, 1 << 20, *g, 0, None) == -1
    assert lib.conv1d_bwd_weight(fake, fake, fake, ctypes.c_void_p(0x1010), 1 << 20, *g, 0, None) == -1  # ws alignment
    assert lib.conv1d_set_variant(99) == -1 and lib.conv1d_set_variant(0) == 0
    # fused epilogues: unknown flag bits, bfloat16 output for float inputs, ReLU on a gradient
    assert lib.conv1d_fwd_ex(fake, fake, None, fake, *g, 0, 4, None) == -1
    assert lib.conv1d_fwd_ex(fake, fake, None, fake, *g, 0, 2, None) == -1
    assert lib.conv1d_fwd_ex(fake, fake, ctypes.c_void_p(0x1002), fake, *g, 0, 0, None) == -1      # misaligned bias
    assert lib.conv1d_fwd_ex(fake, fake, None, None, *g, 1, 3, None) == -1
    assert lib.conv1d_bwd_data_ex(fake, fake, fake, *g, 1, 1, None) == -1
    assert lib.conv1d_bwd_data_ex(fake, fake, fake, *g, 0, 2, None) == -1
    # the entry point without a workspace: same argument checks, and a geometry beyond its built-in buffer is
    # rejected before any HIP call
    assert lib.conv1d_bwd_weight_noalloc(None, fake, fake, *g, 0, None) == -1
    assert lib.conv1d_bwd_weight_noalloc(fake, fake, fake, 2, 4, 4, 8, 5, 2, 0, 0, None) == -1
    big = (8, 256, 256, 20000, 51, 8, 200)
    assert binding.conv1d_bwd_weight_workspace_bytes(*big, 1) > binding.NOALLOC_SCRATCH_BYTES
    assert lib.conv1d_bwd_weight_noalloc(fake, fake, fake, *big, 1, None) == -5


def test_workspace_query_and_kernel_names():
    assert binding.conv1d_bwd_weight_workspace_bytes(2, 4, 4, 8, 5, 2, 0, 0) == 0   # invalid geometry
    for dt in (0, 1):
        b = binding.conv1d_bwd_weight_workspace_bytes(16, 15, 15, 60000, 51, 8, 200, dt)
        assert b >= 15 * 15 * 51 * 4 and b % 256 == 0
    assert binding.conv1d_kernel_name(0, 2, 4, 4, 8, 5, 2, 0, 0) == "invalid"
    binding.conv1d_set_variant(binding.VARIANT_GENERIC)
    try:
        assert binding.conv1d_kernel_name(binding.PASS_FWD, 2, 4, 4, 256, 5, 2, 0, 0) == "generic_fma_fp32"
        assert binding.conv1d_kernel_name(binding.PASS_BWD_WEIGHT, 2, 4, 4, 256, 5, 2, 0, 1) == "generic_wgrad_bf16"
    finally:
        binding.conv1d_set_variant(binding.VARIANT_AUTO)


def test_headline_workloads_dispatch_to_mfma_kernels():
    """The benchmarked genomics shapes must not silently run on the plain-FMA fallback."""
    from paper_2104_08002_amd import inputs

    binding.conv1d_set_variant(binding.VARIANT_AUTO)
    for wl in (inputs.GENOMICS_FP32, inputs.GENOMICS_BF16):
        code = 1 if wl.dtype == "bf16" else 0
        names = [binding.conv1d_kernel_name(i, *wl.geometry(), code) for i in range(3)]
        assert all("mfma" in n for n in names), names


def test_wide_layers_dispatch_to_blocked_mfma_kernels():
    """More than 16 channels or filters: the channel-blocked family, not the plain-FMA fallback."""
    from paper_2104_08002_amd import inputs

    binding.conv1d_set_variant(binding.VARIANT_AUTO)
    wls = [inputs.WIDE_BF16] + [inputs.sweep_point(S, d, dt) for S in inputs.SWEEP_S for d in inputs.SWEEP_D for dt in ("fp32", "bf16")]
    for wl in wls:
        code = 1 if wl.dtype == "bf16" else 0
        names = [binding.conv1d_kernel_name(i, *wl.geometry(), code) for i in range(3)]
        assert all(n.startswith("igemm_") and "mfma" in n for n in names), (wl.name, names)
    # small channel counts at a dilation other than 8: bf16 backward-weight still runs on MFMA
    for d in (1, 2, 3, 4, 16):
        assert "mfma" in binding.conv1d_kernel_name(binding.PASS_BWD_WEIGHT, 4, 15, 15, 5000, 51, d, 25 * d, 1)
    # fp32 backward-weight runs all 16 x 16 block pairs in one launch, one workgroup per CU in total: the
    # partial sums of all pairs together take what a single pair's 256 workgroups take
    wl = inputs.sweep_point(51, 8, "fp32")
    g = wl.geometry()
    small = (g[0], 16, 16) + tuple(g[3:])
    assert binding.conv1d_bwd_weight_workspace_bytes(*g, 0) == binding.conv1d_bwd_weight_workspace_bytes(*small, 0)
    assert binding.conv1d_bwd_weight_workspace_bytes(*g, 0) == 256 * 51 * 256 * 4


def test_plan_queries_survive_arbitrary_geometries():
    """Host logic only: the kernel-family decision and the workspace size of every pass for a few hundred seeded
    geometries (tiny and large channel counts, widths below one tile, dilations the fast families do not take).
    Every answer is a known family name; a valid geometry never reports 'invalid', and its workspace is a multiple
    of 256 bytes that a single MI355X can hold."""
    import random

    rnd = random.Random(20210408)
    families = ("smallc_", "igemm_", "generic_")
    binding.conv1d_set_variant(binding.VARIANT_AUTO)
    for _ in range(400):
        N = rnd.choice([1, 2, 3, 5, 16, 64])
        C = rnd.choice([1, 3, 15, 16, 17, 40, 64, 200, 256, 1040])
        K = rnd.choice([1, 2, 15, 16, 24, 64, 72, 256, 288, 1056])
        S = rnd.choice([1, 2, 4, 5, 9, 12, 13, 17, 20, 33, 51, 52, 53, 70])
        d = rnd.choice([1, 2, 3, 4, 6, 8, 16, 32])
        W = rnd.choice([(S - 1) * d + 1, 8, 63, 200, 1024, 4097, 60000])
        P = rnd.choice([0, 1, 3, (S - 1) * d // 2, (S - 1) * d])
        if W + 2 * P - (S - 1) * d < 1:
            continue
        for dt in (0, 1):
            for i in range(3):
                name = binding.conv1d_kernel_name(i, N, C, K, W, S, d, P, dt)
                assert name.startswith(families), (name, N, C, K, W, S, d, P, dt)
            b = binding.conv1d_bwd_weight_workspace_bytes(N, C, K, W, S, d, P, dt)
            assert b % 256 == 0 and 0 < b < (64 << 30), (b, N, C, K, W, S, d, P, dt)

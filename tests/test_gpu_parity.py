"""Parity of the HIP path against the FP64 oracle, through the C ABI, on a real MI355X.

Bar (per output element e, A[e] = sum of |products| feeding it):
    |gpu[e] - oracle[e]| / A[e] <= 1e-5 for fp32 inputs, <= 1e-2 for bf16 inputs,
and gpu[e] == 0 exactly where A[e] == 0.
"""
import numpy as np
import pytest

from paper_2104_08002_amd import inputs
from parity_util import assert_parity, check_full, check_sampled, gpu_passes, to_device

pytestmark = pytest.mark.gpu

VARIANTS = {"auto": 0, "generic": 1, "smallc": 2, "igemm": 3}
PASS_ID = {"fwd": 0, "bwd_data": 1, "bwd_weight": 2}


@pytest.fixture(scope="module")
def binding():
    import torch

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2104_08002_amd import binding as b

    b.load()
    yield b
    b.conv1d_set_variant(b.VARIANT_AUTO)


def _supported_passes(binding, wl):
    code = 1 if wl.dtype == "bf16" else 0
    return tuple(p for p, i in PASS_ID.items()
                 if binding.conv1d_kernel_name(i, *wl.geometry(), code) != "unsupported")


def _run_full(binding, oracle, wl, variant):
    binding.conv1d_set_variant(VARIANTS[variant])
    try:
        passes = _supported_passes(binding, wl)
        if not passes:
            pytest.skip(f"variant {variant} does not run this geometry")
        data = inputs.make_inputs(wl)
        got = gpu_passes(wl, to_device(wl, data), passes)
    finally:
        binding.conv1d_set_variant(0)
    errs = check_full(oracle, wl, data, got, passes)
    assert_parity(wl.name, variant, wl.dtype, errs)
    return passes


def _mk(name, N, C, K, W, S, d, P, dtype, base=inputs.TINY, **kw):
    return inputs.scaled(base, name=name, N=N, C=C, K=K, W=W, S=S, d=d, P=P, dtype=dtype, **kw)


# ---- the tiny configuration under every kernel family -------------------------------------------
@pytest.mark.parametrize("variant", list(VARIANTS))
@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_tiny_every_variant(binding, oracle, variant, dtype):
    wl = inputs.scaled(inputs.TINY, dtype=dtype, name=f"tiny_{dtype}")
    _run_full(binding, oracle, wl, variant)


# ---- small geometries: several tiles, ragged tails, odd channel counts, every dilation ----------
SMALL = [
    # name                N  C   K   W     S   d   P
    ("one_of_each",       1, 1,  1,  1,    1,  1,  0),
    ("single_column",     2, 3,  2,  9,    3,  4,  0),     # Q = 1
    ("pad_gt_span",       2, 3,  4,  40,   3,  2,  9),     # P > (S-1)d: bwd_data sees a negative shift
    ("valid_ragged",      3, 5,  7,  1000, 5,  3,  0),
    ("same_d1",           2, 15, 15, 1333, 51, 1,  25),
    ("same_d2",           2, 15, 15, 1500, 51, 2,  50),
    ("same_d4",           2, 16, 16, 2049, 51, 4,  100),
    ("genomics_small",    3, 15, 15, 5000, 51, 8,  200),
    ("same_d16",          2, 15, 15, 3001, 51, 16, 400),
    ("d3_odd",            2, 15, 13, 2500, 25, 3,  36),
    ("d5_asym",           2, 9,  16, 1777, 31, 5,  7),
    ("narrow_S9",         4, 10, 8,  777,  9,  8,  32),
    ("S1_gemm",           2, 15, 15, 4100, 1,  1,  0),
    ("even_S",            2, 8,  4,  900,  6,  8,  20),
    ("c17_k33",           2, 17, 33, 1200, 9,  2,  8),
    ("c32_k32_d4",        2, 32, 32, 2100, 17, 4,  32),
    ("c64_k64_d1",        2, 64, 64, 1100, 9,  1,  4),
    ("c64_k64_d16",       1, 64, 64, 2500, 33, 16, 256),
    ("c48_k80",           2, 48, 80, 700,  5,  8,  16),
    ("c256_k256",         1, 256, 256, 600, 9, 4,  16),
    ("c40_k24_odd_W",     2, 40, 24, 901,  7,  3,  9),     # odd width: no dword-aligned rows
    ("c20_k20_S3",        2, 20, 20, 500,  3,  2,  2),     # fewer taps than one MFMA step of the many-channel kernel
    ("c64_k64_odd_P",     2, 64, 64, 1536, 9,  2,  7),     # odd padding: window origin one column early
    ("halo_gt_width",     2, 15, 15, 300,  51, 8,  200),   # halo (S-1)d = 400 exceeds W
    ("long_halo_short_W", 4, 4,  4,  64,   33, 16, 256),
    # many taps at dilations 1, 2, 4, 8, 16: bf16 backward-weight keeps the shared x operands in a register ring
    ("ring_two_tap_groups", 1, 20, 20, 3000, 100, 4, 13),  # S > 52: two tap groups
    ("ring_S33_d1_c40",   3, 40, 24, 5000, 33, 1,  16),
    ("ring_S33_d2_odd_P", 3, 40, 24, 5000, 33, 2,  31),
    ("ring_S17_d8_odd_W", 2, 33, 17, 4001, 17, 8,  64),
    ("ring_S27_d4_short", 1, 16, 16, 300,  27, 4,  0),     # a strip shorter than one unit of k-steps
    ("ring_S70_d16",      1, 20, 20, 5000, 70, 16, 5),
    # forward / backward-data with resident weights: few taps, odd padding, a filter count that is no multiple of 32
    ("res_S12_d16",       3, 40, 24, 5000, 12, 16, 43),
    ("res_S7_d4",         2, 72, 40, 1000, 7,  4,  12),
    ("res_S45_d8_c128",   1, 128, 48, 2000, 45, 8, 77),
    # many filters and channels, few taps, few tiles: the staged kernel
    ("wide_S7_d8",        1, 128, 200, 3000, 7, 8,  21),    # filter count no multiple of 32
    ("wide_S12_d2",       2, 136, 72, 2500, 12, 2,  11),    # odd padding, channel count no multiple of 16
    ("wide_S5_d16",       1, 256, 256, 1024, 5, 16, 32),    # one column tile per sample
    ("wide_S9_d1_odd",    3, 160, 96, 2100, 9,  1,  4),
    ("wide_c200_fwd",     1, 200, 72, 1500, 9, 2,  7),
    ("wide_k200_bwd",     2, 72, 200, 1100, 12, 4, 0),     # no padding
    ("wide_c264_short",   1, 264, 40, 70,  5,  1,  2),     # one short tile; 33 planes of channels
    # forward / backward-data with streamed weights: weights too large for LDS and more than 128 (tile, filter
    # group) pairs; 2, 3 and 5 tap groups, in the forward and in the backward-data pass
    ("str2_fwd",          4, 288, 1056, 200, 7, 1,  3),
    ("str2_bwd",          5, 1040, 288, 190, 5, 16, 32),    # ragged filter groups
    ("str3_fwd",          4, 200, 1056, 1100, 9, 4, 16),    # a second tile of a few columns per sample
    ("str3_bwd",          4, 1056, 200, 200, 12, 2, 11),    # odd padding
    ("str5_fwd",          4, 232, 1056, 200, 17, 2, 16),    # an odd number of stages, the last tile of the last sample
    ("str5_bwd",          4, 1056, 232, 210, 15, 8, 3),
    # small-channel bf16 forward / backward-data with block staging (d = 8 or 16; width and padding multiples of 8)
    ("blk_d16_S25",       2, 15, 15, 3000, 25, 16, 192),
    ("blk_d8_S9",         3, 10, 8,  4000, 9,  8,  32),
    ("blk_short",         2, 15, 15, 64,   51, 8,  200),   # both row edges inside one window
    ("blk_P_gt_span",     2, 7,  16, 2048, 5,  8,  40),    # backward-data shift -8: window starts beyond column 0
    ("blk_one_block",     1, 16, 16, 8,    3,  8,  8),
    # bf16 backward-weight with the tap shift applied in registers: d = 1, 2 and (S - 1) d <= 16
    ("shift_S5_d1_odd_W", 2, 40, 24, 901,  5,  1,  2),     # odd width: element-wise staging
    ("shift_S17_d1",      2, 64, 40, 1500, 17, 1,  8),     # three x slots per lane and k-step
    ("shift_S2_d2",       3, 33, 17, 700,  2,  2,  1),     # odd padding: dy rows staged from odd columns
    ("shift_S5_d2_P0",    2, 70, 64, 1000, 5,  2,  0),     # two channel groups
    ("shift_S9_d2_big_P", 1, 64, 64, 300,  9,  2,  37),    # padding beyond the span: x slots left of the row
    ("shift_tiny_W",      2, 20, 20, 9,    5,  1,  2),     # less than one k-step
    ("shift_k300",        1, 24, 300, 2000, 3, 1,  1),     # many filter groups
    ("shift_d4_c96",      2, 96, 96, 900,  5,  4,  7),     # dilation 4, many channel blocks, odd padding; four filter blocks
    ("shift_d4_S9_c300",  1, 300, 40, 1000, 9, 4,  16),    # five x slots per lane; ragged channel and filter groups
    ("c40_halo_gt_width", 2, 40, 24, 200,  51, 8,  200),   # many channels, halo (S-1)d = 400 exceeds W
    ("c40_tiny_Q",        3, 40, 24, 420,  51, 8,  0),     # Q = 20: less than one k-step / one position block pair
]


@pytest.mark.parametrize("variant", list(VARIANTS))
@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("case", SMALL, ids=[c[0] for c in SMALL])
def test_small_geometries(binding, oracle, case, dtype, variant):
    name, N, C, K, W, S, d, P = case
    dists = dict(x_dist="sparse_exp", w_dist="normal_fan", dy_dist="normal") if "genomics" in name else {}
    wl = _mk(f"{name}_{dtype}", N, C, K, W, S, d, P, dtype, seed=inputs.BASE_SEED + 1000 + len(name), **dists)
    _run_full(binding, oracle, wl, variant)


# ---- seeded random geometries in the many-channel, few-tap corner (bf16): the resident-weight kernel's two prologue
# ---- paths and filter-block counts, the register-shift backward-weight kernel's slot counts, masks and edge units ----
def _random_few_tap_cases(count=36, seed=20210408):
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < count:
        d = int(rng.choice([1, 2, 4, 8, 16]))
        S = int(rng.integers(2, 13)) if d <= 4 else int(rng.integers(5, 13))
        C = int(rng.choice([17, 24, 32, 40, 64, 72, 96, 130]))
        K = int(rng.choice([17, 24, 33, 48, 64, 80, 100, 144]))
        W = int(rng.integers(40, 2600))
        P = int(rng.integers(0, (S - 1) * d + 3))
        N = int(rng.integers(1, 4))
        if W + 2 * P - (S - 1) * d < 1:
            continue
        cases.append((f"rnd{len(cases)}_c{C}_k{K}_S{S}_d{d}", N, C, K, W, S, d, P))
    return cases


RANDOM_FEW_TAP = _random_few_tap_cases()


@pytest.mark.parametrize("case", RANDOM_FEW_TAP, ids=[c[0] for c in RANDOM_FEW_TAP])
def test_random_many_channel_few_taps(binding, oracle, case):
    name, N, C, K, W, S, d, P = case
    wl = _mk(f"{name}_bf16", N, C, K, W, S, d, P, "bf16", seed=inputs.BASE_SEED + 3000 + len(name) + W)
    _run_full(binding, oracle, wl, "auto")


# ---- base pointers that are only element-aligned: every kernel's unaligned path --------------------
UNALIGNED = [
    # name             N  C   K   W     S   d  P
    ("una_genomics",   2, 15, 15, 3000, 51, 8, 200),
    ("una_c64_S51",    1, 64, 64, 1536, 51, 8, 200),
    ("una_c64_S9",     2, 64, 64, 1200, 9,  2, 8),
    ("una_c40_S33_d4", 2, 40, 24, 2000, 33, 4, 64),
]


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("case", UNALIGNED, ids=[c[0] for c in UNALIGNED])
def test_element_aligned_pointers(binding, oracle, case, dtype):
    """The ABI asks for element alignment only: shift every tensor by one element inside a larger allocation."""
    import torch

    name, N, C, K, W, S, d, P = case
    wl = _mk(f"{name}_{dtype}", N, C, K, W, S, d, P, dtype, seed=inputs.BASE_SEED + 2000 + len(name))
    data = inputs.make_inputs(wl)
    dev = to_device(wl, data)

    def shifted(t):
        big = torch.empty(t.numel() + 1, dtype=t.dtype, device=t.device)
        view = big[1:].view(t.shape)
        view.copy_(t)
        assert view.data_ptr() % 16 != 0 and view.is_contiguous()
        return view

    x, w, dy = shifted(dev["x"]), shifted(dev["w"]), shifted(dev["dy"])
    y = shifted(torch.empty((N, K, wl.Q), dtype=torch.float32, device="cuda"))
    dx = shifted(torch.empty((N, C, W), dtype=torch.float32, device="cuda"))
    dw = shifted(torch.empty((K, C, S), dtype=torch.float32, device="cuda"))
    binding.conv1d_fwd(x, w, d, P, out=y)
    binding.conv1d_bwd_data(dy, w, W, d, P, out=dx)
    binding.conv1d_bwd_weight(x, dy, S, d, P, out=dw)
    torch.cuda.synchronize()
    got = {"fwd": y.cpu().numpy(), "bwd_data": dx.cpu().numpy(), "bwd_weight": dw.cpu().numpy()}
    errs = check_full(oracle, wl, data, got)
    assert_parity(wl.name, "unaligned", wl.dtype, errs)


# ---- genomics at full size, the configuration the benchmark times: whole-output comparison ------
@pytest.mark.parametrize("wl", [inputs.GENOMICS_FP32, inputs.GENOMICS_BF16], ids=lambda w: w.name)
def test_genomics_full_size(binding, oracle, wl):
    _run_full(binding, oracle, wl, "auto")


# ---- sampled comparison: only for widths whose whole output the oracle cannot finish in seconds ----
def _run_sampled(binding, oracle, wl):
    data = inputs.make_inputs(wl)
    got = gpu_passes(wl, to_device(wl, data))
    errs = check_sampled(oracle, wl, data, got, np.random.default_rng(wl.seed))
    assert_parity(wl.name, "sampled", wl.dtype, errs)
    for k, v in got.items():
        assert np.isfinite(v).all(), (wl.name, k)


# ---- filter-width x dilation sweep and the wide configuration at full size, in the launch configuration the
# ---- benchmark times: whole-output comparison (the oracle needs 1-8 s per pass on the machine's host cores) ----
@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("S", inputs.SWEEP_S)
@pytest.mark.parametrize("d", inputs.SWEEP_D)
def test_sweep_full_size(binding, oracle, S, d, dtype):
    _run_full(binding, oracle, inputs.sweep_point(S, d, dtype), "auto")


def test_wide_full_size(binding, oracle):
    _run_full(binding, oracle, inputs.WIDE_BF16, "auto")


# ---- the paper's own grid (Section 4.3): batch 56, output widths 1000 ... 60000, four channel/dilation families ----
Q_POINTS = [(f, Q, 51) for f in inputs.Q_SWEEP_FAMILIES for Q in inputs.Q_SWEEP_Q]
Q_POINTS += [(f, 1000, S) for f in inputs.Q_SWEEP_FAMILIES for S in (1, 5, 21)]       # short rows, few taps


@pytest.mark.parametrize("family,Q,S", Q_POINTS, ids=[f"{f}_S{S}_Q{Q}" for f, Q, S in Q_POINTS])
def test_paper_grid_batch56(binding, oracle, family, Q, S):
    wl = inputs.q_sweep_point(family, Q, S)
    # whole output wherever the oracle finishes in well under a minute; sampled for the two largest 64-channel points
    if wl.flops > 3e11:
        _run_sampled(binding, oracle, wl)
    else:
        _run_full(binding, oracle, wl, "auto")


# ---- long segments (the paper's 600000-wide inputs, Section 4.5.3): one sample, sampled outputs -----
LONG = [
    # name                N  C   K   W       S   d  P
    ("long_genomics",     1, 15, 15, 600000, 51, 8, 200),
    ("long_c64_S17_d4",   1, 64, 64, 300000, 17, 4, 32),
]


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("case", LONG, ids=[c[0] for c in LONG])
def test_long_segments_sampled(binding, oracle, case, dtype):
    name, N, C, K, W, S, d, P = case
    wl = _mk(f"{name}_{dtype}", N, C, K, W, S, d, P, dtype, seed=inputs.BASE_SEED + 3000 + len(name))
    _run_sampled(binding, oracle, wl)


# ---- the sweep and wide shapes at a width the oracle finishes whole ------------------------------
@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("S,d", [(5, 1), (9, 16), (17, 2), (33, 4), (51, 8), (51, 16)])
def test_sweep_reduced_width_full_compare(binding, oracle, S, d, dtype):
    wl = inputs.scaled(inputs.sweep_point(S, d, dtype), N=2, W=3000 + 7)
    _run_full(binding, oracle, wl, "auto")


def test_wide_reduced_full_compare(binding, oracle):
    wl = inputs.scaled(inputs.WIDE_BF16, N=2, W=1000)
    _run_full(binding, oracle, wl, "auto")


# ---- backward-weight is bit-reproducible (fixed-order second stage, no float atomics) -----------
@pytest.mark.parametrize("wl", [inputs.scaled(inputs.GENOMICS_BF16, N=4, W=20000, name="det_bf16"),
                                inputs.scaled(inputs.GENOMICS_FP32, N=4, W=20000, name="det_fp32"),
                                inputs.scaled(inputs.sweep_point(17, 4, "bf16"), N=2, W=5000)],
                         ids=lambda w: w.name)
def test_bwd_weight_is_deterministic(binding, wl):
    import torch

    dev = to_device(wl, inputs.make_inputs(wl))
    runs = []
    for _ in range(3):
        runs.append(binding.conv1d_bwd_weight(dev["x"], dev["dy"], wl.S, wl.d, wl.P).clone())
        torch.cuda.synchronize()
    assert torch.equal(runs[0], runs[1]) and torch.equal(runs[0], runs[2])


# ---- outputs are overwritten, not accumulated into (beta = 0) ------------------------------------
@pytest.mark.parametrize("wl", [inputs.scaled(inputs.GENOMICS_FP32, N=2, W=3000, name="overwrite"),
                                inputs.scaled(inputs.sweep_point(9, 4, "fp32"), N=2, W=2000, name="overwrite_blocked")],
                         ids=lambda w: w.name)
def test_outputs_are_overwritten(binding, oracle, wl):
    import torch

    data = inputs.make_inputs(wl)
    dev = to_device(wl, data)
    y = torch.full((wl.N, wl.K, wl.Q), float("nan"), device="cuda")
    dx = torch.full((wl.N, wl.C, wl.W), float("nan"), device="cuda")
    dw = torch.full((wl.K, wl.C, wl.S), float("nan"), device="cuda")
    ws = torch.full((binding.conv1d_bwd_weight_workspace_bytes(*wl.geometry(), 0) // 4,), float("nan"), device="cuda")
    binding.conv1d_fwd(dev["x"], dev["w"], wl.d, wl.P, out=y)
    binding.conv1d_bwd_data(dev["dy"], dev["w"], wl.W, wl.d, wl.P, out=dx)
    binding.conv1d_bwd_weight(dev["x"], dev["dy"], wl.S, wl.d, wl.P, out=dw, workspace=ws.view(torch.uint8))
    torch.cuda.synchronize()
    got = {"fwd": y.cpu().numpy(), "bwd_data": dx.cpu().numpy(), "bwd_weight": dw.cpu().numpy()}
    assert_parity(wl.name, "nan_prefilled", "fp32", check_full(oracle, wl, data, got))


# ---- a non-default stream --------------------------------------------------------------------------
def test_runs_on_callers_stream(binding, oracle):
    import torch

    wl = inputs.scaled(inputs.GENOMICS_BF16, N=2, W=4000, name="stream")
    data = inputs.make_inputs(wl)
    dev = to_device(wl, data)
    st = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(st):
        y = binding.conv1d_fwd(dev["x"], dev["w"], wl.d, wl.P)
        dx = binding.conv1d_bwd_data(dev["dy"], dev["w"], wl.W, wl.d, wl.P)
        dw = binding.conv1d_bwd_weight(dev["x"], dev["dy"], wl.S, wl.d, wl.P)
    st.synchronize()
    got = {"fwd": y.cpu().numpy(), "bwd_data": dx.cpu().numpy(), "bwd_weight": dw.cpu().numpy()}
    assert_parity(wl.name, "side_stream", "bf16", check_full(oracle, wl, data, got))

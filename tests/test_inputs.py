"""The synthetic workloads: geometry, seeds, distributions and bf16 rounding."""
import numpy as np

from paper_2104_08002_amd import inputs


def test_workload_geometry():
    g = inputs.GENOMICS_FP32
    assert (g.N, g.C, g.K, g.W, g.S, g.d, g.P, g.Q) == (16, 15, 15, 60000, 51, 8, 200, 60000)
    assert g.flops == 2 * 16 * 15 * 15 * 51 * 60000
    t = inputs.TINY
    assert t.Q == 248 and t.P == 0
    w = inputs.WIDE_BF16
    assert (w.P, w.Q) == (16, 8192)
    pts = list(inputs.sweep("bf16"))
    assert len(pts) == 25 and all(p.Q == p.W == 20000 for p in pts)
    assert len({p.seed for p in pts}) == 25


def test_draws_are_seeded_and_distributed():
    wl = inputs.scaled(inputs.GENOMICS_FP32, N=2, W=20000, name="g_small")
    a, b = inputs.make_inputs(wl), inputs.make_inputs(wl)
    for k in ("x", "w", "dy"):
        assert np.array_equal(a[k], b[k]) and a[k].dtype == np.float32
    assert a["x"].shape == (2, 15, 20000) and a["w"].shape == (15, 15, 51) and a["dy"].shape == (2, 15, 20000)
    assert abs((a["x"] == 0).mean() - 0.8) < 0.01 and (a["x"] >= 0).all()
    assert abs(a["x"][a["x"] > 0].mean() - 1.0) < 0.02
    assert abs(a["w"].var() * 15 * 51 - 1.0) < 0.05
    assert abs(a["dy"].std() - 1.0) < 0.01
    t = inputs.make_inputs(inputs.TINY)
    assert np.abs(t["x"]).max() <= 1.0 and np.abs(t["w"]).max() <= 1.0


def test_bf16_rounding_is_nearest_even():
    f = np.array([1.0, 1.00390625, 1.01171875, -1.00390625, 3.0e38, 1e-40, 0.0], dtype=np.float32)
    bits = inputs.f32_to_bf16_bits(f)
    back = inputs.bf16_bits_to_f32(bits)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: even mantissa wins (1.0);
    # 1 + 3*2^-8 ties between 1+2^-7 and 1+2^-6: even is 1+2^-6.
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == np.float32(1.015625) and back[3] == -1.0
    rng = np.random.default_rng(0)
    a = rng.standard_normal(10000).astype(np.float32)
    r = inputs.bf16_bits_to_f32(inputs.f32_to_bf16_bits(a))
    assert np.max(np.abs(r - a) / np.abs(a)) <= 2.0 ** -8
    assert np.array_equal(inputs.f32_to_bf16_bits(r), inputs.f32_to_bf16_bits(a))
    wl = inputs.scaled(inputs.GENOMICS_BF16, N=1, W=4000)
    d = inputs.make_inputs(wl)
    for k in ("x", "w", "dy"):
        assert d[k + "_bits"].dtype == np.uint16
        assert np.array_equal(inputs.bf16_bits_to_f32(d[k + "_bits"]), d[k])

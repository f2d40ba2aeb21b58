"""Pins for the FP64 oracle against things the paper and the mathematics fix.

None of these re-type the oracle's formula: each compares with a library
routine of a special case, a closed form, an algebraic identity, or a literal
scatter-form brute force written in the opposite loop order.
"""
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(rng, *shape):
    return rng.standard_normal(shape)


# -- Section 2: d = 1 reduces Eq. 2 to the ordinary (undilated) layer, which for one
#    channel and no padding is numpy's 'valid' cross-correlation. -------------------------
def test_d1_single_channel_is_numpy_correlate(oracle):
    rng = np.random.default_rng(1)
    x, w = _rand(rng, 1, 1, 41), _rand(rng, 1, 1, 7)
    y = oracle.fwd(x, w, 1, 0)
    np.testing.assert_allclose(y[0, 0], np.correlate(x[0, 0], w[0, 0], "valid"), rtol=0, atol=1e-13)


def test_d1_multichannel_is_sum_of_correlations(oracle):
    rng = np.random.default_rng(2)
    N, C, K, W, S = 2, 3, 4, 37, 5
    x, w = _rand(rng, N, C, W), _rand(rng, K, C, S)
    y = oracle.fwd(x, w, 1, 0)
    for n in range(N):
        for k in range(K):
            ref = sum(np.correlate(x[n, c], w[k, c], "valid") for c in range(C))
            np.testing.assert_allclose(y[n, k], ref, rtol=0, atol=1e-12)


def test_dilated_is_correlation_with_zero_stuffed_filter(oracle):
    # A dilated filter is the plain filter with d-1 zeros between taps (Section 2).
    rng = np.random.default_rng(3)
    d, S, W, P = 3, 4, 50, 5
    x, w = _rand(rng, 1, 1, W), _rand(rng, 1, 1, S)
    stuffed = np.zeros((S - 1) * d + 1)
    stuffed[::d] = w[0, 0]
    xp = np.pad(x[0, 0], P)
    np.testing.assert_allclose(oracle.fwd(x, w, d, P)[0, 0], np.correlate(xp, stuffed, "valid"),
                               rtol=0, atol=1e-13)


# -- Algorithm 1 with a single tap is one GEMM. -------------------------------------------
def test_S1_is_plain_gemm(oracle):
    rng = np.random.default_rng(4)
    N, C, K, W = 3, 5, 7, 29
    x, w, g = _rand(rng, N, C, W), _rand(rng, K, C, 1), _rand(rng, N, K, W)
    y = oracle.fwd(x, w, 1, 0)
    dx = oracle.bwd_data(g, w, W, 1, 0)
    dw = oracle.bwd_weight(x, g, 1, 1, 0)
    for n in range(N):
        np.testing.assert_allclose(y[n], w[:, :, 0] @ x[n], rtol=0, atol=1e-12)
        np.testing.assert_allclose(dx[n], w[:, :, 0].T @ g[n], rtol=0, atol=1e-12)
    np.testing.assert_allclose(dw[:, :, 0], sum(g[n] @ x[n].T for n in range(N)), rtol=0, atol=1e-11)


# -- The three passes are one bilinear map and its two adjoints (Sections 3.2, 3.3). -------
@pytest.mark.parametrize("geom", [(2, 3, 4, 50, 5, 3, 4), (1, 4, 2, 33, 7, 2, 0), (3, 2, 5, 64, 3, 8, 8),
                                  (2, 5, 3, 23, 4, 5, 9)])
def test_adjoint_identities(oracle, geom):
    N, C, K, W, S, d, P = geom
    Q = W + 2 * P - (S - 1) * d
    rng = np.random.default_rng(5)
    x, w, g = _rand(rng, N, C, W), _rand(rng, K, C, S), _rand(rng, N, K, Q)
    lhs = np.sum(oracle.fwd(x, w, d, P) * g)
    via_x = np.sum(x * oracle.bwd_data(g, w, W, d, P))
    via_w = np.sum(w * oracle.bwd_weight(x, g, S, d, P))
    scale = np.sum(np.abs(oracle.fwd(np.abs(x), np.abs(w), d, P)) * np.abs(g))
    assert abs(lhs - via_x) <= 1e-13 * scale
    assert abs(lhs - via_w) <= 1e-13 * scale


# -- L(w) = <fwd(x,w), g> is linear in w and in x, so a central difference with any step
#    equals the gradient entry up to rounding. ---------------------------------------------
def test_finite_differences_of_both_gradients(oracle):
    N, C, K, W, S, d, P = 2, 3, 2, 19, 4, 2, 3
    Q = W + 2 * P - (S - 1) * d
    rng = np.random.default_rng(6)
    x, w, g = _rand(rng, N, C, W), _rand(rng, K, C, S), _rand(rng, N, K, Q)
    dw = oracle.bwd_weight(x, g, S, d, P)
    dx = oracle.bwd_data(g, w, W, d, P)
    h = 1.0
    for k in range(K):
        for c in range(C):
            for s in range(S):
                wp, wm = w.copy(), w.copy()
                wp[k, c, s] += h
                wm[k, c, s] -= h
                fd = (np.sum(oracle.fwd(x, wp, d, P) * g) - np.sum(oracle.fwd(x, wm, d, P) * g)) / (2 * h)
                assert abs(fd - dw[k, c, s]) < 1e-10
    for n, c, i in [(0, 0, 0), (1, 2, 18), (0, 1, 7), (1, 0, 3), (0, 2, 11)]:
        xp, xm = x.copy(), x.copy()
        xp[n, c, i] += h
        xm[n, c, i] -= h
        fd = (np.sum(oracle.fwd(xp, w, d, P) * g) - np.sum(oracle.fwd(xm, w, d, P) * g)) / (2 * h)
        assert abs(fd - dx[n, c, i]) < 1e-10


# -- Closed forms: impulses place the taps, reversed and d apart. --------------------------
def test_input_impulse_response(oracle):
    N, C, K, W, S, d, P = 1, 3, 2, 40, 5, 4, 6
    Q = W + 2 * P - (S - 1) * d
    rng = np.random.default_rng(7)
    w = _rand(rng, K, C, S)
    for c0, i0 in [(0, 0), (1, 17), (2, 39), (1, 3)]:
        x = np.zeros((N, C, W))
        x[0, c0, i0] = 1.0
        y = oracle.fwd(x, w, d, P)
        expect = np.zeros((K, Q))
        for s in range(S):
            q = i0 + P - s * d
            if 0 <= q < Q:
                expect[:, q] = w[:, c0, s]
        assert np.array_equal(y[0], expect)


def test_weight_impulse_is_a_shift(oracle):
    N, C, K, W, S, d, P = 2, 3, 2, 30, 4, 3, 5
    Q = W + 2 * P - (S - 1) * d
    rng = np.random.default_rng(8)
    x = _rand(rng, N, C, W)
    for k0, c0, s0 in [(0, 0, 0), (1, 2, 3), (0, 1, 2)]:
        w = np.zeros((K, C, S))
        w[k0, c0, s0] = 1.0
        y = oracle.fwd(x, w, d, P)
        xp = np.pad(x, ((0, 0), (0, 0), (P, P)))
        assert np.array_equal(y[:, k0], xp[:, c0, s0 * d: s0 * d + Q])
        assert not y[:, 1 - k0].any()


def test_grad_impulses(oracle):
    # dy = delta at (k0,q0): dx[c, q0 - P + s*d] = w[k0,c,s]; dw[k0,c,s] = x[c, q0+s*d-P].
    N, C, K, W, S, d, P = 1, 2, 3, 25, 3, 4, 2
    Q = W + 2 * P - (S - 1) * d
    rng = np.random.default_rng(9)
    x, w = _rand(rng, N, C, W), _rand(rng, K, C, S)
    for k0, q0 in [(0, 0), (2, Q - 1), (1, 9)]:
        g = np.zeros((N, K, Q))
        g[0, k0, q0] = 1.0
        dx = oracle.bwd_data(g, w, W, d, P)
        dw = oracle.bwd_weight(x, g, S, d, P)
        edx, edw = np.zeros((C, W)), np.zeros((K, C, S))
        for s in range(S):
            i = q0 - P + s * d
            if 0 <= i < W:
                edx[:, i] = w[k0, :, s]
                edw[k0, :, s] = x[0, :, i]
        assert np.array_equal(dx[0], edx)
        assert np.array_equal(dw, edw)


# -- Fig. 1 geometry with all-ones tensors: outputs count the in-range taps. ----------------
def _read_fig1():
    vals = {}
    with open(os.path.join(GOLDEN, "fig1_shape.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, *rest = line.split()
            vals[key] = [int(v) for v in rest]
    return vals


def test_fig1_shape_and_allones_counts(oracle):
    g = _read_fig1()
    C, W, K, S, d, P, Q = (g[k][0] for k in "C W K S d P Q".split())
    assert oracle.out_width(W, S, d, P) == Q
    y, ya = oracle.fwd(np.ones((1, C, W)), np.ones((K, C, S)), d, P, with_abs=True)
    expect = C * np.asarray(g["taps_in_range"], dtype=np.float64)
    for k in range(K):
        assert np.array_equal(y[0, k], expect)
    assert np.array_equal(ya, y)


# -- Algorithm 1 (S GEMMs over shifted slices of the padded input) is another schedule of
#    the same sum; so is any width blocking (Algorithm 2). ---------------------------------
def _alg1_numpy(x, w, d, P):
    N, C, W = x.shape
    K, _, S = w.shape
    Q = W + 2 * P - (S - 1) * d
    xp = np.pad(x, ((0, 0), (0, 0), (P, P)))
    y = np.zeros((N, K, Q))
    for s in range(S):
        for n in range(N):
            y[n] += w[:, :, s] @ xp[n, :, d * s: d * s + Q]
    return y


@pytest.mark.parametrize("geom", [(2, 4, 4, 256, 5, 2, 0), (2, 15, 15, 700, 51, 8, 200), (1, 7, 3, 130, 9, 16, 64),
                                  (2, 5, 4, 17, 3, 3, 3)])
def test_matches_S_gemm_schedule(oracle, geom):
    N, C, K, W, S, d, P = geom
    rng = np.random.default_rng(10)
    x, w = _rand(rng, N, C, W), _rand(rng, K, C, S)
    y, ya = oracle.fwd(x, w, d, P, with_abs=True)
    assert np.max(np.abs(y - _alg1_numpy(x, w, d, P)) / ya) < 1e-14
    np.testing.assert_allclose(ya, _alg1_numpy(np.abs(x), np.abs(w), d, P), rtol=1e-13)


# -- Literal scatter form (every input element pushes to the outputs it touches). -----------
def _scatter_bruteforce(x, w, g, d, P):
    N, C, W = x.shape
    K, _, S = w.shape
    Q = W + 2 * P - (S - 1) * d
    y, dx, dw = np.zeros((N, K, Q)), np.zeros((N, C, W)), np.zeros((K, C, S))
    for n in range(N):
        for c in range(C):
            for i in range(W):
                for k in range(K):
                    for s in range(S):
                        q = i + P - s * d
                        if 0 <= q < Q:
                            y[n, k, q] += x[n, c, i] * w[k, c, s]
                            dx[n, c, i] += g[n, k, q] * w[k, c, s]
                            dw[k, c, s] += g[n, k, q] * x[n, c, i]
    return y, dx, dw


@pytest.mark.parametrize("geom", [(2, 3, 4, 20, 3, 2, 1), (1, 2, 2, 15, 4, 3, 5), (2, 4, 3, 32, 5, 1, 0),
                                  (1, 1, 1, 9, 2, 5, 2)])
def test_scatter_bruteforce_all_passes(oracle, geom):
    N, C, K, W, S, d, P = geom
    Q = W + 2 * P - (S - 1) * d
    rng = np.random.default_rng(11)
    x, w, g = _rand(rng, N, C, W), _rand(rng, K, C, S), _rand(rng, N, K, Q)
    y, dx, dw = _scatter_bruteforce(x, w, g, d, P)
    np.testing.assert_allclose(oracle.fwd(x, w, d, P), y, rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.bwd_data(g, w, W, d, P), dx, rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.bwd_weight(x, g, S, d, P), dw, rtol=0, atol=1e-12)


# -- Independent library: torch's CPU conv1d and its autograd, in float64. ------------------
@pytest.mark.parametrize("geom", [(2, 4, 4, 256, 5, 2, 0), (2, 15, 15, 900, 51, 8, 200), (3, 6, 5, 100, 9, 4, 16),
                                  (1, 3, 2, 40, 4, 3, 1)])
def test_against_torch_cpu_conv1d(oracle, geom):
    torch = pytest.importorskip("torch")
    N, C, K, W, S, d, P = geom
    Q = W + 2 * P - (S - 1) * d
    rng = np.random.default_rng(12)
    x, w, g = _rand(rng, N, C, W), _rand(rng, K, C, S), _rand(rng, N, K, Q)
    tx = torch.tensor(x, requires_grad=True)
    tw = torch.tensor(w, requires_grad=True)
    ty = torch.nn.functional.conv1d(tx, tw, padding=P, dilation=d)
    ty.backward(torch.tensor(g))
    y, ya = oracle.fwd(x, w, d, P, with_abs=True)
    dx, dxa = oracle.bwd_data(g, w, W, d, P, with_abs=True)
    dw, dwa = oracle.bwd_weight(x, g, S, d, P, with_abs=True)
    assert np.max(np.abs(y - ty.detach().numpy()) / ya) < 1e-13
    assert np.max(np.abs(dx - tx.grad.numpy()) / np.maximum(dxa, 1e-300)) < 1e-13
    assert np.max(np.abs(dw - tw.grad.numpy()) / dwa) < 1e-13


# -- Translation equivariance in the interior (tiling seams would break it). -----------------
def test_translation_equivariance(oracle):
    rng = np.random.default_rng(13)
    N, C, K, W, S, d, P, t = 1, 3, 3, 120, 5, 4, 8, 7
    x, w = np.zeros((N, C, W)), _rand(rng, K, C, S)
    x[:, :, 30:70] = _rand(rng, N, C, 40)
    y0 = oracle.fwd(x, w, d, P)
    y1 = oracle.fwd(np.roll(x, t, axis=2), w, d, P)
    np.testing.assert_allclose(y1[:, :, t:], y0[:, :, :-t], rtol=0, atol=1e-14)


# -- The abs companion is fwd of the absolute values; sampled variants equal the full ones. --
def test_abs_companion_and_sampled_variants(oracle):
    rng = np.random.default_rng(14)
    N, C, K, W, S, d, P = 2, 5, 4, 90, 7, 3, 9
    Q = W + 2 * P - (S - 1) * d
    x, w, g = _rand(rng, N, C, W), _rand(rng, K, C, S), _rand(rng, N, K, Q)
    y, ya = oracle.fwd(x, w, d, P, with_abs=True)
    dx, dxa = oracle.bwd_data(g, w, W, d, P, with_abs=True)
    dw, dwa = oracle.bwd_weight(x, g, S, d, P, with_abs=True)
    np.testing.assert_allclose(ya, oracle.fwd(np.abs(x), np.abs(w), d, P), rtol=1e-14)
    np.testing.assert_allclose(dxa, oracle.bwd_data(np.abs(g), np.abs(w), W, d, P), rtol=1e-14)
    np.testing.assert_allclose(dwa, oracle.bwd_weight(np.abs(x), np.abs(g), S, d, P), rtol=1e-14)
    idx = np.stack([rng.integers(0, N, 50), rng.integers(0, K, 50), rng.integers(0, Q, 50)], axis=1)
    v, a = oracle.fwd_at(x, w, idx, d, P)
    assert np.array_equal(v, y[idx[:, 0], idx[:, 1], idx[:, 2]])
    assert np.array_equal(a, ya[idx[:, 0], idx[:, 1], idx[:, 2]])
    idx = np.stack([rng.integers(0, N, 50), rng.integers(0, C, 50), rng.integers(0, W, 50)], axis=1)
    v, a = oracle.bwd_data_at(g, w, idx, W, d, P)
    assert np.array_equal(v, dx[idx[:, 0], idx[:, 1], idx[:, 2]])
    assert np.array_equal(a, dxa[idx[:, 0], idx[:, 1], idx[:, 2]])
    idx = np.stack([rng.integers(0, K, 50), rng.integers(0, C, 50), rng.integers(0, S, 50)], axis=1)
    v, a = oracle.bwd_weight_at(x, g, idx, S, d, P)
    assert np.array_equal(v, dw[idx[:, 0], idx[:, 1], idx[:, 2]])
    assert np.array_equal(a, dwa[idx[:, 0], idx[:, 1], idx[:, 2]])


def test_rejects_bad_geometry(oracle):
    with pytest.raises(ValueError):
        oracle.fwd(np.zeros((1, 2, 5)), np.zeros((1, 2, 4)), 3, 0)      # Q <= 0
    with pytest.raises(ValueError):
        oracle.fwd(np.zeros((1, 2, 5)), np.zeros((1, 3, 2)), 1, 0)      # channel mismatch

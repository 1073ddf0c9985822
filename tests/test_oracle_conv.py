"""Pins for the fp64 convolution oracle: hand-computed cases, closed forms, library
routines on special cases, adjoint and finite-difference identities, micro-batch
equivalence.  None of these re-types the oracle's loops."""
import json
import os

import numpy as np
import pytest
from scipy import signal

from oracle import conv as oc
from oracle.conv import Layer

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "conv_hand_cases.json")
rng = np.random.default_rng(1234)

SHAPES = [
    Layer(2, 3, 7, 6, 4, 3, 3, 1, 1, 1, 1),
    Layer(3, 2, 8, 9, 3, 3, 2, 2, 2, 1, 0),     # R != S, stride 2, (H+2p-R)%s != 0
    Layer(2, 4, 9, 9, 5, 5, 5, 1, 1, 2, 2),
    Layer(2, 3, 11, 10, 2, 7, 7, 2, 2, 3, 3),
    Layer(1, 5, 6, 6, 7, 1, 1, 2, 2, 0, 0),     # 1x1 stride 2 projection
    Layer(2, 2, 12, 13, 3, 4, 3, 3, 2, 2, 1),   # mixed strides and pads
    Layer(2, 3, 15, 15, 2, 11, 11, 4, 4, 0, 0),
]


def rand(shape):
    return rng.uniform(-1, 1, size=shape)


@pytest.mark.parametrize("case", json.load(open(GOLDEN))["cases"], ids=lambda c: c["name"][:30])
def test_hand_computed_cases(case):
    L = Layer(*case["layer"])
    x = np.array(case["x"], float).reshape(L.x_shape)
    w = np.array(case["w"], float).reshape(L.w_shape)
    assert oc.conv_fwd(L, x, w).ravel().tolist() == case["y"]
    if "dy" in case:
        dy = np.array(case["dy"], float).reshape(L.y_shape)
        assert oc.conv_bwd_data(L, dy, w).ravel().tolist() == case["dx"]
        assert oc.conv_bwd_filter(L, x, dy).ravel().tolist() == case["dw"]


def test_identity_1x1_filter_returns_input():
    L = Layer(3, 6, 5, 7, 6, 1, 1)
    x = rand(L.x_shape)
    w = np.eye(6).reshape(L.w_shape)
    assert np.array_equal(oc.conv_fwd(L, x, w), x)


def test_all_ones_closed_form_counts_in_bounds_taps():
    # x = 1, w = 1: y[p,q] = C * (#in-bounds rows) * (#in-bounds cols)
    L = Layer(1, 5, 6, 8, 2, 3, 3, 1, 1, 1, 1)
    y = oc.conv_fwd(L, np.ones(L.x_shape), np.ones(L.w_shape))
    rows = np.array([2] + [3] * 4 + [2])
    cols = np.array([2] + [3] * 6 + [2])
    expect = 5 * rows[:, None] * cols[None, :]
    assert np.array_equal(y[0, 0], expect) and np.array_equal(y[0, 1], expect)
    assert y[0, 0, 0, 0] == 20 and y[0, 0, 0, 3] == 30 and y[0, 0, 2, 2] == 45


def test_ones_filter_gives_window_sums_via_integral_image():
    L = Layer(2, 1, 9, 8, 1, 3, 4, 1, 1, 1, 2)
    x = rng.integers(-5, 6, size=L.x_shape).astype(float)
    y = oc.conv_fwd(L, x, np.ones(L.w_shape))
    xp = np.pad(x, ((0, 0), (0, 0), (1, 1), (2, 2)))
    ii = np.pad(xp.cumsum(2).cumsum(3), ((0, 0), (0, 0), (1, 0), (1, 0)))
    win = ii[:, :, 3:, 4:] - ii[:, :, :-3, 4:] - ii[:, :, 3:, :-4] + ii[:, :, :-3, :-4]
    assert np.array_equal(y, win)


def test_1x1_conv_is_a_matrix_product():
    L = Layer(2, 7, 4, 5, 3, 1, 1)
    x, w = rand(L.x_shape), rand(L.w_shape)
    expect = np.matmul(w.reshape(3, 7), x.reshape(2, 7, 20)).reshape(L.y_shape)
    np.testing.assert_allclose(oc.conv_fwd(L, x, w), expect, rtol=0, atol=1e-14)


def test_delta_input_reads_filter_back_index_reversed():
    # x = delta at (h0, w0): y[k, p, q] = w[k, c0, h0 - p, w0 - q] (valid conv, stride 1)
    L = Layer(1, 2, 5, 5, 3, 3, 3)
    x = np.zeros(L.x_shape)
    x[0, 1, 2, 2] = 1.0
    w = rand(L.w_shape)
    y = oc.conv_fwd(L, x, w)
    assert np.array_equal(y[0], w[:, 1, ::-1, ::-1])


@pytest.mark.parametrize("L", SHAPES, ids=str)
def test_against_scipy_correlate(L):
    """Stride-1 correlation per (n,k,c) is a library routine; a strided conv subsamples it."""
    x, w, dy = rand(L.x_shape), rand(L.w_shape), rand(L.y_shape)
    xp = np.pad(x, ((0, 0), (0, 0), (L.ph, L.ph), (L.pw, L.pw)))
    y = np.zeros(L.y_shape)
    for n in range(L.N):
        for k in range(L.K):
            for c in range(L.C):
                full = signal.correlate2d(xp[n, c], w[k, c], mode="valid")
                y[n, k] += full[::L.sh, ::L.sw][:L.P, :L.Q]
    np.testing.assert_allclose(oc.conv_fwd(L, x, w), y, rtol=0, atol=1e-12)

    # BackwardData: dilate dy by the stride, true (flipped) full convolution with w, crop the pad
    dx = np.zeros((L.N, L.C, L.H + 2 * L.ph, L.W + 2 * L.pw))
    dw = np.zeros(L.w_shape)
    for n in range(L.N):
        for k in range(L.K):
            up = np.zeros(((L.P - 1) * L.sh + 1, (L.Q - 1) * L.sw + 1))
            up[::L.sh, ::L.sw] = dy[n, k]
            for c in range(L.C):
                f = signal.convolve2d(up, w[k, c], mode="full")
                dx[n, c, :f.shape[0], :f.shape[1]] += f
                # BackwardFilter: correlate padded input with the dilated dy
                g = signal.correlate2d(xp[n, c], up, mode="valid")
                dw[k, c] += g[:L.R, :L.S]
    dx = dx[:, :, L.ph:L.ph + L.H, L.pw:L.pw + L.W]
    np.testing.assert_allclose(oc.conv_bwd_data(L, dy, w), dx, rtol=0, atol=1e-12)
    np.testing.assert_allclose(oc.conv_bwd_filter(L, x, dy), dw, rtol=0, atol=1e-12)


@pytest.mark.parametrize("L", SHAPES, ids=str)
def test_adjoint_identities(L):
    x, w, dy = rand(L.x_shape), rand(L.w_shape), rand(L.y_shape)
    a = np.vdot(oc.conv_fwd(L, x, w), dy)
    b = np.vdot(x, oc.conv_bwd_data(L, dy, w))
    c = np.vdot(w, oc.conv_bwd_filter(L, x, dy))
    scale = np.abs(a) + 1.0
    assert abs(a - b) / scale < 1e-12 and abs(a - c) / scale < 1e-12


def test_finite_difference_of_the_bilinear_loss():
    L = Layer(2, 2, 6, 5, 3, 3, 3, 2, 1, 1, 1)
    x, w, dy = rand(L.x_shape), rand(L.w_shape), rand(L.y_shape)
    dx, dw = oc.conv_bwd_data(L, dy, w), oc.conv_bwd_filter(L, x, dy)
    loss = lambda xx, ww: np.vdot(oc.conv_fwd(L, xx, ww), dy)
    for _ in range(5):
        i = tuple(rng.integers(0, s) for s in L.x_shape)
        e = np.zeros(L.x_shape); e[i] = 0.5
        assert abs((loss(x + e, w) - loss(x - e, w)) - dx[i]) < 1e-12
        j = tuple(rng.integers(0, s) for s in L.w_shape)
        e = np.zeros(L.w_shape); e[j] = 0.5
        assert abs((loss(x, w + e) - loss(x, w - e)) - dw[j]) < 1e-12


def test_linearity():
    L = SHAPES[1]
    x1, x2, w = rand(L.x_shape), rand(L.x_shape), rand(L.w_shape)
    lhs = oc.conv_fwd(L, 2 * x1 - 3 * x2, w)
    rhs = 2 * oc.conv_fwd(L, x1, w) - 3 * oc.conv_fwd(L, x2, w)
    np.testing.assert_allclose(lhs, rhs, rtol=0, atol=1e-13)


def test_unused_trailing_rows_get_zero_gradient():
    # (H+2p-R) % s != 0: the last input row/col is never read by Forward
    L = Layer(1, 1, 6, 6, 1, 1, 1, 2, 2, 0, 0)
    dx = oc.conv_bwd_data(L, np.ones(L.y_shape), np.ones(L.w_shape))
    assert np.array_equal(dx[0, 0], np.kron(np.ones((3, 3)), np.array([[1, 0], [0, 0]])))


@pytest.mark.parametrize("parts", [[8], [1] * 8, [3, 5], [2, 2, 4], [7, 1]])
def test_micro_batched_equals_undivided(parts):
    L = Layer(8, 3, 7, 7, 4, 3, 3, 1, 1, 1, 1)
    x, w, dy = rand(L.x_shape), rand(L.w_shape), rand(L.y_shape)
    assert np.array_equal(oc.micro_fwd(L, x, w, parts), oc.conv_fwd(L, x, w))
    assert np.array_equal(oc.micro_bwd_data(L, dy, w, parts), oc.conv_bwd_data(L, dy, w))
    np.testing.assert_allclose(oc.micro_bwd_filter(L, x, dy, parts), oc.conv_bwd_filter(L, x, dy),
                               rtol=0, atol=1e-13)
    dw0 = rand(L.w_shape)
    np.testing.assert_allclose(oc.micro_bwd_filter(L, x, dy, parts, beta=1.0, dw=dw0),
                               dw0 + oc.conv_bwd_filter(L, x, dy), rtol=0, atol=1e-13)


def test_beta_zero_ignores_old_contents_even_nan():
    L = Layer(1, 1, 3, 3, 1, 2, 2)
    x, dy = rand(L.x_shape), rand(L.y_shape)
    junk = np.full(L.w_shape, np.nan)
    assert np.array_equal(oc.conv_bwd_filter(L, x, dy, beta=0.0, dw=junk), oc.conv_bwd_filter(L, x, dy))


def test_sampled_forms_match_full_tensors():
    L = SHAPES[3]
    x, w, dy = rand(L.x_shape), rand(L.w_shape), rand(L.y_shape)
    y, dx, dw = oc.conv_fwd(L, x, w), oc.conv_bwd_data(L, dy, w), oc.conv_bwd_filter(L, x, dy)
    for full, f, args in ((y, oc.conv_fwd_at, (x, w)), (dx, oc.conv_bwd_data_at, (dy, w)),
                          (dw, oc.conv_bwd_filter_at, (x, dy))):
        idx = rng.integers(0, full.size, size=50)
        assert np.array_equal(f(L, *args, idx), full.ravel()[idx])


def test_empty_batch():
    L = Layer(0, 2, 4, 4, 3, 3, 3, 1, 1, 1, 1)
    assert oc.conv_fwd(L, np.zeros(L.x_shape), np.zeros(L.w_shape)).shape == (0, 3, 4, 4)
    assert np.array_equal(oc.conv_bwd_filter(L, np.zeros(L.x_shape), np.zeros(L.y_shape)),
                          np.zeros(L.w_shape))

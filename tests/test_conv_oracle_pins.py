"""Pins for the CPU oracle of the convolution layer (no GPU, no HIP library).

The paper gives the layer's shape (Sec. 4.1, workload table: N=8, C=64, H=W=56, F=128, 3x3, stride
1, padding 1, FP16) and no output value, so the oracle is held by what the definition fixes: closed
forms (centre-tap identity, single-tap shifts, all-ones tap counts), reduction to a matrix product
for 1x1 filters, two independent library routines on integer-valued data (scipy's correlate2d,
torch's fp64 conv2d with strides and paddings), exact rational brute force, and linearity.
"""
from fractions import Fraction

import numpy as np
import pytest
import scipy.signal
import torch

from paper_2605_28213_amd import inputs as gen

F32, BF16, F16, E4M3 = 0, 1, 2, 3
DTYPES = [F32, BF16, F16, E4M3]


def _ints(rng, shape, lo=-2, hi=2):
    return rng.integers(lo, hi + 1, size=shape).astype(np.float32)


def _q(dt, a):
    return gen.quantise(dt, np.ascontiguousarray(a, dtype=np.float32).ravel()).reshape(a.shape)


@pytest.mark.parametrize("dt", DTYPES)
def test_centre_tap_identity_filter_returns_the_input(oracle, dt):
    rng = np.random.default_rng(1)
    N, H, W, C = 2, 5, 7, 6
    x = _ints(rng, (N, H, W, C))
    w = np.zeros((C, 3, 3, C), np.float32)
    for c in range(C):
        w[c, 1, 1, c] = 1.0
    y, d = oracle.conv2d(dt, _q(dt, x), _q(dt, w), pad=(1, 1))
    np.testing.assert_array_equal(y, x.astype(np.float64))
    np.testing.assert_array_equal(d, np.abs(x).astype(np.float64))


@pytest.mark.parametrize("r,s", [(0, 0), (0, 2), (2, 0), (2, 1), (1, 2)])
def test_single_tap_shifts_the_image_without_flipping_the_filter(oracle, r, s):
    """Tap (r, s) with padding 1 reads x[p + r - 1, q + s - 1]: the top-left tap moves the image down
    and right and leaves a zero first row and column.  A flipped filter (true convolution), swapped
    r/s or a padding of the wrong sign all give a different picture."""
    rng = np.random.default_rng(2)
    N, H, W, C, F = 1, 6, 5, 3, 2
    x = _ints(rng, (N, H, W, C), 1, 3)
    w = np.zeros((F, 3, 3, C), np.float32)
    w[0, r, s, 1] = 2.0
    w[1, r, s, 2] = -1.0
    y, _ = oracle.conv2d(F32, x, w, pad=(1, 1))
    want = np.zeros((N, H, W, F))
    for p in range(H):
        for q in range(W):
            h, ww = p + r - 1, q + s - 1
            if 0 <= h < H and 0 <= ww < W:
                want[0, p, q, 0] = 2.0 * x[0, h, ww, 1]
                want[0, p, q, 1] = -1.0 * x[0, h, ww, 2]
    np.testing.assert_array_equal(y, want)
    if (r, s) == (0, 0):
        assert not y[0, 0, :, :].any() and not y[0, :, 0, :].any() and y[0, 1:, 1:, 0].all()


@pytest.mark.parametrize("dt", DTYPES)
def test_all_ones_counts_the_taps_inside_the_image(oracle, dt):
    N, H, W, C, F = 1, 6, 9, 64, 3
    x = np.ones((N, H, W, C), np.float32)
    w = np.ones((F, 3, 3, C), np.float32)
    y, d = oracle.conv2d(dt, _q(dt, x), _q(dt, w), pad=(1, 1))
    rows = np.array([2] + [3] * (H - 2) + [2])
    cols = np.array([2] + [3] * (W - 2) + [2])
    want = (C * np.outer(rows, cols)).astype(np.float64)
    assert want[0, 0] == 4 * C and want[0, 1] == 6 * C and want[1, 1] == 9 * C
    for f in range(F):
        np.testing.assert_array_equal(y[0, :, :, f], want)
        np.testing.assert_array_equal(d[0, :, :, f], want)


def test_output_size_strides_and_paddings(oracle):
    for H, W, R, S, st, pd in [(56, 56, 3, 3, (1, 1), (1, 1)), (7, 9, 3, 2, (2, 3), (0, 1)), (5, 5, 5, 5, (1, 1), (0, 0)),
                               (8, 8, 1, 1, (2, 2), (0, 0)), (6, 4, 3, 3, (1, 2), (2, 0))]:
        x = np.ones((1, H, W, 1), np.float32)
        w = np.ones((1, R, S, 1), np.float32)
        y, _ = oracle.conv2d(F32, x, w, stride=st, pad=pd)
        want = torch.nn.functional.conv2d(torch.ones(1, 1, H, W, dtype=torch.float64), torch.ones(1, 1, R, S, dtype=torch.float64),
                                          stride=st, padding=pd)
        assert y.shape == (1, want.shape[2], want.shape[3], 1) == (1,) + oracle.conv2d_output_size(H, W, R, S, st, pd) + (1,)
        np.testing.assert_array_equal(y[0, :, :, 0], want[0, 0].numpy())


@pytest.mark.parametrize("dt", DTYPES)
def test_one_by_one_filter_is_a_matrix_product(oracle, dt):
    rng = np.random.default_rng(3)
    N, H, W, C, F = 2, 3, 4, 37, 5
    x, w = _ints(rng, (N, H, W, C)), _ints(rng, (F, 1, 1, C))
    y, d = oracle.conv2d(dt, _q(dt, x), _q(dt, w))
    want = x.reshape(-1, C).astype(np.int64) @ w.reshape(F, C).astype(np.int64).T
    np.testing.assert_array_equal(y.reshape(-1, F), want.astype(np.float64))
    np.testing.assert_array_equal(d.reshape(-1, F), (np.abs(x.reshape(-1, C)).astype(np.int64) @ np.abs(w.reshape(F, C)).astype(np.int64).T).astype(np.float64))


def test_integer_valued_against_scipy_correlate2d(oracle):
    rng = np.random.default_rng(4)
    N, H, W, C, F = 2, 9, 8, 3, 4
    x, w = _ints(rng, (N, H, W, C), -3, 3), _ints(rng, (F, 3, 3, C), -3, 3)
    y, _ = oracle.conv2d(F32, x, w, pad=(1, 1))
    for n in range(N):
        for f in range(F):
            want = sum(scipy.signal.correlate2d(x[n, :, :, c].astype(np.float64), w[f, :, :, c].astype(np.float64),
                                                mode="same", boundary="fill", fillvalue=0) for c in range(C))
            np.testing.assert_array_equal(y[n, :, :, f], want)


@pytest.mark.parametrize("dt", DTYPES)
@pytest.mark.parametrize("geom", [((1, 1), (1, 1), 3, 3), ((2, 2), (1, 1), 3, 3), ((1, 2), (0, 2), 3, 2), ((3, 1), (2, 0), 5, 1), ((2, 3), (0, 0), 2, 4)])
def test_integer_valued_against_torch_fp64_conv2d(oracle, dt, geom):
    st, pd, R, S = geom
    rng = np.random.default_rng(5)
    N, H, W, C, F = 2, 11, 10, 5, 3
    x, w = _ints(rng, (N, H, W, C)), _ints(rng, (F, R, S, C))
    bias = _ints(rng, (F,))
    y, d = oracle.conv2d(dt, _q(dt, x), _q(dt, w), stride=st, pad=pd, bias=bias)
    xt = torch.from_numpy(x.astype(np.float64)).permute(0, 3, 1, 2)
    wt = torch.from_numpy(w.astype(np.float64)).permute(0, 3, 1, 2)
    want = torch.nn.functional.conv2d(xt, wt, bias=torch.from_numpy(bias.astype(np.float64)), stride=st, padding=pd).permute(0, 2, 3, 1).numpy()
    np.testing.assert_array_equal(y, want)
    wantd = torch.nn.functional.conv2d(xt.abs(), wt.abs(), bias=torch.from_numpy(np.abs(bias).astype(np.float64)), stride=st, padding=pd).permute(0, 2, 3, 1).numpy()
    np.testing.assert_array_equal(d, wantd)
    # the point form agrees with the full form
    P, Q = y.shape[1], y.shape[2]
    pn, pp, pq, pf = rng.integers(0, N, 50), rng.integers(0, P, 50), rng.integers(0, Q, 50), rng.integers(0, F, 50)
    yp, dp = oracle.conv2d_points(dt, _q(dt, x), _q(dt, w), pn, pp, pq, pf, stride=st, pad=pd, bias=bias)
    np.testing.assert_array_equal(yp, y[pn, pp, pq, pf])
    np.testing.assert_array_equal(dp, d[pn, pp, pq, pf])


@pytest.mark.parametrize("dt", DTYPES)
def test_exact_rational_brute_force(oracle, dt):
    """Random representable (non-integer) values on a tiny layer against exact fractions."""
    rng = np.random.default_rng(6)
    N, H, W, C, F, R, S, st, pd = 1, 4, 3, 2, 2, 3, 2, (2, 1), (1, 1)
    xs = _q(dt, rng.uniform(-1, 1, (N, H, W, C)).astype(np.float32))
    ws = _q(dt, rng.uniform(-1, 1, (F, R, S, C)).astype(np.float32))
    xv, wv = oracle.decode(dt, xs), oracle.decode(dt, ws)
    y, d = oracle.conv2d(dt, xs, ws, stride=st, pad=pd)
    P, Q = oracle.conv2d_output_size(H, W, R, S, st, pd)
    assert y.shape == (N, P, Q, F)
    for p in range(P):
        for q in range(Q):
            for f in range(F):
                acc, mag = Fraction(0), Fraction(0)
                for r in range(R):
                    for s in range(S):
                        h, ww = p * st[0] - pd[0] + r, q * st[1] - pd[1] + s
                        if 0 <= h < H and 0 <= ww < W:
                            for c in range(C):
                                t = Fraction(float(xv[0, h, ww, c])) * Fraction(float(wv[f, r, s, c]))
                                acc += t
                                mag += abs(t)
                assert abs(Fraction(float(y[0, p, q, f])) - acc) <= Fraction(1, 2 ** 45) * max(mag, Fraction(1, 2 ** 40))
                assert abs(Fraction(float(d[0, p, q, f])) - mag) <= Fraction(1, 2 ** 45) * max(mag, Fraction(1, 2 ** 40))


def test_linearity_and_channel_order(oracle):
    rng = np.random.default_rng(7)
    N, H, W, C, F = 1, 5, 5, 4, 3
    x1, x2, w = _ints(rng, (N, H, W, C)), _ints(rng, (N, H, W, C)), _ints(rng, (F, 3, 3, C))
    y1, _ = oracle.conv2d(F32, x1, w, pad=(1, 1))
    y2, _ = oracle.conv2d(F32, x2, w, pad=(1, 1))
    y12, _ = oracle.conv2d(F32, x1 + 2 * x2, w, pad=(1, 1))
    np.testing.assert_array_equal(y12, y1 + 2 * y2)
    # permuting the channels of x and w alike changes nothing; permuting the filters permutes the outputs
    perm = rng.permutation(C)
    yp, _ = oracle.conv2d(F32, np.ascontiguousarray(x1[..., perm]), np.ascontiguousarray(w[..., perm]), pad=(1, 1))
    np.testing.assert_array_equal(yp, y1)
    fp = rng.permutation(F)
    yf, _ = oracle.conv2d(F32, x1, np.ascontiguousarray(w[fp]), pad=(1, 1))
    np.testing.assert_array_equal(yf, y1[..., fp])
    # images of a batch are independent
    xb = np.concatenate([x1, x2], axis=0)
    yb, _ = oracle.conv2d(F32, xb, w, pad=(1, 1))
    np.testing.assert_array_equal(yb[0], y1[0])
    np.testing.assert_array_equal(yb[1], y2[0])


def test_bad_arguments_are_rejected(oracle):
    x = np.ones((1, 2, 2, 1), np.float32)
    w = np.ones((1, 3, 3, 1), np.float32)
    with pytest.raises(ValueError):
        oracle.conv2d(F32, x, w)                        # filter larger than the unpadded image
    with pytest.raises(ValueError):
        oracle.conv2d(F32, x, np.ones((1, 3, 3, 2), np.float32), pad=(1, 1))
    with pytest.raises(TypeError):
        oracle.conv2d(F16, x, w, pad=(1, 1))
    y, _ = oracle.conv2d(F32, x, w, pad=(1, 1))
    with pytest.raises(ValueError):
        oracle.conv2d_points(F32, x, w, [0], [2], [0], [0], pad=(1, 1))

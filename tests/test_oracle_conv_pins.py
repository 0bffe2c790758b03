"""Pins of the oracle's convolution over level indices (the layer compute of Sec. IV-A for a convolutional layer)
against things it does not share code with: scipy's 2-D cross-correlation channel by channel, an im2col matrix
built with numpy strides and multiplied by numpy, the 1 x 1 case as a plain matrix product, and one-tap kernels,
whose output is the input shifted.  A wrong stride, padding offset, tap order or layout fails one of them."""
import numpy as np
import pytest
from scipy.signal import correlate2d


def _draw(rng, shape, lo=-7, hi=7):
    return rng.integers(lo, hi + 1, size=shape).astype(np.int16)


def _im2col(x, R, S, stride, pad):
    """[B,H,W,C] -> [B*P*Q, R*S*C] with zero padding, by numpy strides (tap order r, s, c)."""
    B, H, W, C = x.shape
    xp = np.zeros((B, H + 2 * pad, W + 2 * pad, C), dtype=np.int64)
    xp[:, pad:pad + H, pad:pad + W, :] = x
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    sb, sh, sw, sc = xp.strides
    win = np.lib.stride_tricks.as_strided(xp, shape=(B, P, Q, R, S, C), strides=(sb, sh * stride, sw * stride, sh, sw, sc))
    return win.reshape(B * P * Q, R * S * C), P, Q


@pytest.mark.parametrize("B,H,W,C,N,R,S,stride,pad", [
    (2, 7, 9, 3, 4, 3, 3, 1, 1), (1, 8, 8, 5, 2, 3, 3, 2, 1), (2, 6, 5, 4, 3, 1, 1, 1, 0), (1, 9, 7, 2, 3, 5, 3, 1, 2),
    (3, 5, 5, 6, 2, 3, 3, 1, 0), (1, 10, 11, 3, 2, 3, 5, 2, 0), (2, 4, 4, 3, 3, 1, 1, 2, 0)])
def test_convolution_equals_numpy_im2col_product(oracle, B, H, W, C, N, R, S, stride, pad):
    rng = np.random.default_rng(B * 100 + H * 10 + W + C)
    x, w = _draw(rng, (B, H, W, C)), _draw(rng, (N, R, S, C))
    acc, y = oracle.qconv_fwd(x, w, stride, pad, 0.25, 0.5)
    cols, P, Q = _im2col(x, R, S, stride, pad)
    want = (cols @ w.reshape(N, -1).astype(np.int64).T).reshape(B, P, Q, N)
    assert acc.shape == (B, P, Q, N)
    assert np.array_equal(acc.astype(np.int64), want)
    assert np.array_equal(y, 0.125 * want)           # 0.25 * 0.5 and the integers are exact in double


def test_convolution_equals_scipy_cross_correlation(oracle):
    rng = np.random.default_rng(11)
    B, H, W, C, N, R, S = 2, 9, 8, 3, 2, 3, 3
    x, w = _draw(rng, (B, H, W, C)), _draw(rng, (N, R, S, C))
    acc, _ = oracle.qconv_fwd(x, w, 1, 1, 1.0, 1.0, want_y=False)
    for b in range(B):
        for n in range(N):
            want = sum(correlate2d(x[b, :, :, c].astype(np.int64), w[n, :, :, c].astype(np.int64), mode="same", boundary="fill")
                       for c in range(C))
            assert np.array_equal(acc[b, :, :, n], want)
    # no padding: the "valid" part
    acc, _ = oracle.qconv_fwd(x, w, 1, 0, 1.0, 1.0, want_y=False)
    want = sum(correlate2d(x[1, :, :, c].astype(np.int64), w[0, :, :, c].astype(np.int64), mode="valid") for c in range(C))
    assert np.array_equal(acc[1, :, :, 0], want)


def test_one_by_one_kernel_is_the_index_product(oracle):
    rng = np.random.default_rng(5)
    x, w = _draw(rng, (2, 5, 6, 8)), _draw(rng, (7, 1, 1, 8))
    acc, y = oracle.qconv_fwd(x, w, 1, 0, 0.3, 0.7)
    acc2, y2 = oracle.qgemm_fwd(x.reshape(-1, 8), w.reshape(7, 8), 0.3, 0.7)
    assert np.array_equal(acc.reshape(-1, 7), acc2)
    assert np.array_equal(y.reshape(-1, 7), y2)


@pytest.mark.parametrize("r,s", [(0, 0), (0, 2), (1, 1), (2, 0), (2, 1)])
def test_one_tap_kernel_shifts_the_image(oracle, r, s):
    rng = np.random.default_rng(r * 3 + s)
    B, H, W, C = 1, 6, 7, 2
    x = _draw(rng, (B, H, W, C))
    w = np.zeros((C, 3, 3, C), dtype=np.int16)
    for c in range(C):
        w[c, r, s, c] = 1                      # output channel c copies input channel c from tap (r, s)
    acc, _ = oracle.qconv_fwd(x, w, 1, 1, 1.0, 1.0, want_y=False)
    want = np.zeros((B, H, W, C), dtype=np.int64)
    for p in range(H):
        for q in range(W):
            h, ww = p + r - 1, q + s - 1
            if 0 <= h < H and 0 <= ww < W:
                want[0, p, q] = x[0, h, ww]
    assert np.array_equal(acc, want)


def test_unsigned_eight_bit_indices_and_the_largest_accumulator(oracle):
    # level indices up to 255 (the unsigned 8-bit alphabet) against 127: 9 * 64 products of 255 * 127 stay inside int32
    x = np.full((1, 3, 3, 64), 255, dtype=np.int16)
    w = np.full((1, 3, 3, 64), 127, dtype=np.int16)
    acc, _ = oracle.qconv_fwd(x, w, 1, 1, 1.0, 1.0, want_y=False)
    assert acc[0, 1, 1, 0] == 9 * 64 * 255 * 127          # the centre sees all nine taps
    assert acc[0, 0, 0, 0] == 4 * 64 * 255 * 127          # a corner sees four


@pytest.mark.parametrize("B,H,W,C,N,R,S,stride,pad", [
    (2, 7, 9, 3, 4, 3, 3, 1, 1), (1, 8, 8, 5, 2, 3, 3, 2, 1), (2, 6, 5, 4, 3, 1, 1, 1, 0), (1, 9, 7, 2, 3, 5, 3, 1, 2),
    (1, 10, 11, 3, 2, 3, 5, 2, 0), (2, 5, 5, 2, 3, 3, 3, 2, 0)])
def test_convolution_backward_equals_the_index_product_backward_on_windows(oracle, B, H, W, C, N, R, S, stride, pad):
    """dL/dQ(w) is the weight gradient of the product on the window matrix; dL/dQ(x) is its activation gradient with
    every window entry added back to the pixel it came from (numpy add.at), padding entries dropped."""
    rng = np.random.default_rng(B * 100 + H * 10 + W + C + stride)
    x, w = _draw(rng, (B, H, W, C)), _draw(rng, (N, R, S, C))
    cols, P, Q = _im2col(x, R, S, stride, pad)
    g = rng.standard_normal((B, P, Q, N)).astype(np.float32)
    dx, dw = oracle.qconv_bwd(g, x, w, stride, pad, 0.25, 0.5)
    da, db = oracle.qgemm_bwd(g.reshape(-1, N), cols, w.reshape(N, -1), 0.25, 0.5)
    assert np.allclose(dw.reshape(N, -1), db, rtol=1e-13, atol=1e-13)
    want = np.zeros((B, H + 2 * pad, W + 2 * pad, C))
    da = da.reshape(B, P, Q, R, S, C)
    for r in range(R):
        for s in range(S):
            bb, pp, qq = np.meshgrid(np.arange(B), np.arange(P), np.arange(Q), indexing="ij")
            np.add.at(want, (bb, pp * stride + r, qq * stride + s), da[:, :, :, r, s, :])
    assert np.allclose(dx, want[:, pad:pad + H, pad:pad + W, :], rtol=1e-13, atol=1e-13)


def test_convolution_backward_is_the_derivative_of_the_forward(oracle):
    """L = sum g * y is bilinear in the two index tensors: moving x by integers u changes L by exactly
    sum d_x_hat * delta_x * u, and likewise for w - with no window matrix anywhere in the check."""
    rng = np.random.default_rng(3)
    B, H, W, C, N, R, S, stride, pad = 2, 7, 6, 3, 4, 3, 3, 2, 1
    x, w = _draw(rng, (B, H, W, C)), _draw(rng, (N, R, S, C))
    dxs, dws = 0.25, 0.5
    _, y = oracle.qconv_fwd(x, w, stride, pad, dxs, dws)
    g = rng.standard_normal(y.shape).astype(np.float32)
    dx, dw = oracle.qconv_bwd(g, x, w, stride, pad, dxs, dws)
    L0 = float((g.astype(np.float64) * y).sum())
    u = _draw(rng, x.shape, -3, 3)
    _, y1 = oracle.qconv_fwd(x + u, w, stride, pad, dxs, dws)
    assert abs(float((g.astype(np.float64) * y1).sum()) - L0 - float((dx * dxs * u).sum())) < 1e-9
    v = _draw(rng, w.shape, -3, 3)
    _, y2 = oracle.qconv_fwd(x, w + v, stride, pad, dxs, dws)
    assert abs(float((g.astype(np.float64) * y2).sum()) - L0 - float((dw * dws * v).sum())) < 1e-9


def test_one_by_one_convolution_backward_is_the_index_product_backward(oracle):
    rng = np.random.default_rng(8)
    x, w = _draw(rng, (2, 5, 6, 8)), _draw(rng, (7, 1, 1, 8))
    g = rng.standard_normal((2, 5, 6, 7)).astype(np.float32)
    dx, dw = oracle.qconv_bwd(g, x, w, 1, 0, 0.3, 0.7)
    da, db = oracle.qgemm_bwd(g.reshape(-1, 7), x.reshape(-1, 8), w.reshape(7, 8), 0.3, 0.7)
    assert np.array_equal(dx.reshape(-1, 8), da) and np.array_equal(dw.reshape(7, 8), db)

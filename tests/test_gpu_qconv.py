"""cdl_qconv_fwd: the forward product of a convolutional layer over level indices without a matrix of input windows.
Every int32 accumulator must equal the oracle's cross-correlation (small cases: everywhere; large cases: on whole
images of the batch) and, bit for bit, what cdl_qgemm_fwd gives on the matrix of windows built on the host; y within
the stated tolerance.  Both kernels are covered: the register-staged one (any C that is a multiple of 16) and the
direct-load one (C a multiple of 128, enough output tiles)."""
import numpy as np
import pytest

import cdl_inputs
import gpu_util as gu

pytestmark = pytest.mark.gpu


def _windows(x, R, S, stride, pad, fill=0):
    """[B,H,W,C] -> [B*P*Q, R*S*C], taps outside the image filled with `fill` (host-side, for the comparison only)."""
    B, H, W, C = x.shape
    xp = np.full((B, H + 2 * pad, W + 2 * pad, C), fill, dtype=x.dtype)
    xp[:, pad:pad + H, pad:pad + W, :] = x
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    sb, sh, sw, sc = xp.strides
    win = np.lib.stride_tricks.as_strided(xp, shape=(B, P, Q, R, S, C), strides=(sb, sh * stride, sw * stride, sh, sw, sc))
    return np.ascontiguousarray(win.reshape(B * P * Q, R * S * C)), P, Q


def _run(cdl, torch, x, w, stride, pad, dx, dw, x_offset=0):
    B, H, W, C = x.shape
    N, R, S, _ = w.shape
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    acc = gu.empty((B, P, Q, N), torch.int32)
    y = gu.empty((B, P, Q, N), torch.float32)
    acc.fill_(-7)
    y.fill_(float("nan"))
    ws = gu.workspace(cdl.qconv_fwd_workspace_bytes(N, x_offset))
    cdl.cdl_qconv_fwd(gu.dev(x), gu.dev(w), B, H, W, C, N, R, S, stride, pad, dx, dw, acc, None, ws, x_offset=x_offset)
    cdl.cdl_qconv_fwd(gu.dev(x), gu.dev(w), B, H, W, C, N, R, S, stride, pad, dx, dw, None, y, ws, x_offset=x_offset)
    torch.cuda.synchronize()
    return acc.cpu().numpy(), y.cpu().numpy()


# (B, H, W, C, N, R, S, stride, pad): the register-staged kernel - ragged tiles in both directions, strides, paddings, kernel
# shapes, one image smaller than the kernel's reach, more than one tile of rows and of columns, contraction not a multiple of 64
SMALL = [(2, 7, 9, 16, 20, 3, 3, 1, 1), (1, 8, 8, 32, 130, 3, 3, 2, 1), (3, 6, 5, 48, 33, 1, 1, 1, 0), (1, 9, 7, 16, 5, 5, 3, 1, 2),
         (5, 12, 12, 16, 16, 3, 3, 1, 1), (1, 10, 11, 64, 40, 3, 5, 2, 0), (2, 4, 4, 80, 3, 1, 1, 2, 0), (1, 3, 3, 16, 8, 3, 3, 1, 1),
         (4, 17, 13, 32, 140, 3, 3, 1, 1), (1, 2, 2, 128, 7, 3, 3, 1, 1), (2, 32, 32, 16, 16, 3, 3, 1, 1)]


@pytest.mark.parametrize("B,H,W,C,N,R,S,stride,pad", SMALL)
def test_convolution_matches_the_oracle_everywhere(oracle, B, H, W, C, N, R, S, stride, pad):
    import paper_2501_09849_amd as cdl
    torch = gu.torch_mod()
    x = cdl_inputs.draw_indices((B, H, W, C), -128, 127, seed=H * W + C)
    w = cdl_inputs.draw_indices((N, R, S, C), -128, 127, seed=N + R)
    x[0, 0, 0, :], w[0, :, :, :] = -128, -128          # the largest products
    dx, dw = float(np.float32(0.15092)), float(np.float32(0.0028209))
    acc, y = _run(cdl, torch, x, w, stride, pad, dx, dw)
    ref_acc, ref_y = oracle.qconv_fwd(x, w, stride, pad, dx, dw)
    assert np.array_equal(acc, ref_acc), "%d accumulators differ" % int((acc != ref_acc).sum())
    gu.assert_close(y, ref_y, "y")
    # and what the index product gives on the matrix of windows, bit for bit
    cols, P, Q = _windows(x, R, S, stride, pad)
    M, K = cols.shape
    acc2, y2 = gu.empty((M, N), torch.int32), gu.empty((M, N), torch.float32)
    ws = gu.workspace(cdl.qgemm_fwd_workspace_bytes(M, N, K))
    cdl.cdl_qgemm_fwd(gu.dev(cols), gu.dev(w.reshape(N, K)), M, N, K, dx, dw, acc2, y2, ws)
    torch.cuda.synchronize()
    assert np.array_equal(acc.reshape(M, N), acc2.cpu().numpy())
    assert np.array_equal(y.reshape(M, N), y2.cpu().numpy())


# the direct-load kernel: C a multiple of 128 and at least 64 tiles of 256 x 256 outputs
LARGE = [(32, 14, 14, 128, 1024, 3, 3, 1, 1), (64, 14, 14, 256, 512, 3, 3, 1, 1), (80, 28, 28, 128, 300, 3, 3, 2, 1),
         (16, 33, 31, 128, 512, 1, 1, 1, 0), (24, 20, 20, 256, 700, 3, 3, 1, 0), (64, 15, 15, 128, 520, 5, 5, 1, 2)]


@pytest.mark.parametrize("B,H,W,C,N,R,S,stride,pad", LARGE)
def test_convolution_with_direct_loads(oracle, B, H, W, C, N, R, S, stride, pad):
    import paper_2501_09849_amd as cdl
    torch = gu.torch_mod()
    x = cdl_inputs.draw_indices((B, H, W, C), -128, 127, seed=B + C)
    w = cdl_inputs.draw_indices((N, R, S, C), -128, 127, seed=N)
    dx, dw = float(np.float32(0.0731)), float(np.float32(0.011))
    acc, y = _run(cdl, torch, x, w, stride, pad, dx, dw)
    # the oracle on the first, a middle and the last image of the batch
    for b in (0, B // 2, B - 1):
        ref_acc, ref_y = oracle.qconv_fwd(x[b:b + 1], w, stride, pad, dx, dw)
        assert np.array_equal(acc[b:b + 1], ref_acc), "image %d: %d accumulators differ" % (b, int((acc[b:b + 1] != ref_acc).sum()))
        gu.assert_close(y[b:b + 1], ref_y, "y of image %d" % b)
    # every accumulator against the index product on the matrix of windows
    cols, P, Q = _windows(x, R, S, stride, pad)
    M, K = cols.shape
    acc2 = gu.empty((M, N), torch.int32)
    ws = gu.workspace(cdl.qgemm_fwd_workspace_bytes(M, N, K))
    cdl.cdl_qgemm_fwd(gu.dev(cols), gu.dev(w.reshape(N, K)), M, N, K, dx, dw, acc2, None, ws)
    torch.cuda.synchronize()
    assert np.array_equal(acc.reshape(M, N), acc2.cpu().numpy())
    assert np.array_equal(y, (np.float32(np.float32(dx) * np.float32(dw)) * acc.astype(np.float32)))


@pytest.mark.parametrize("B,H,W,C,N,R,S,stride,pad", [(2, 7, 9, 16, 20, 3, 3, 1, 1), (3, 9, 9, 32, 130, 3, 3, 2, 1),
                                                        (32, 14, 14, 128, 1024, 3, 3, 1, 1), (1, 5, 5, 64, 9, 5, 5, 1, 2)])
def test_convolution_of_activations_from_the_unsigned_alphabet(oracle, B, H, W, C, N, R, S, stride, pad):
    """Level indices 0..255 stored minus 128: the padding must read as index 0, i.e. as the stored byte -128."""
    import paper_2501_09849_amd as cdl
    torch = gu.torch_mod()
    rng = np.random.default_rng(B * 7 + C)
    x_true = rng.integers(0, 256, size=(B, H, W, C)).astype(np.int16)
    x_true[0, 0, 0, :] = 255
    x_true[-1, -1, -1, :] = 0
    w = cdl_inputs.draw_indices((N, R, S, C), -127, 127, seed=N + 1)
    x_stored = (x_true - 128).astype(np.int8)
    dx, dw = float(np.float32(0.02)), float(np.float32(0.011))
    acc, y = _run(cdl, torch, x_stored, w, stride, pad, dx, dw, x_offset=128)
    images = range(B) if B <= 3 else (0, B - 1)
    for b in images:
        ref_acc, ref_y = oracle.qconv_fwd(x_true[b:b + 1], w, stride, pad, dx, dw)
        assert np.array_equal(acc[b:b + 1], ref_acc), "image %d" % b
        gu.assert_close(y[b:b + 1], ref_y, "y of image %d" % b)


def test_convolution_rejects_what_it_does_not_serve():
    import paper_2501_09849_amd as cdl
    torch = gu.torch_mod()
    t8 = gu.empty((1 << 16,), torch.int8)
    out = gu.empty((1 << 16,), torch.int32)
    # C not a multiple of 16; padding as wide as the kernel; kernel larger than the padded image; contraction too long; bad offset
    for (B, H, W, C, N, R, S, stride, pad, off), status in (((1, 8, 8, 3, 4, 3, 3, 1, 1, 0), -2), ((1, 8, 8, 16, 4, 3, 3, 1, 3, 0), -2),
                                                            ((1, 2, 2, 16, 4, 5, 5, 1, 1, 0), -2), ((1, 8, 8, 4096, 4, 3, 3, 1, 1, 0), -3),
                                                            ((1, 8, 8, 16, 4, 3, 3, 1, 1, 64), -2), ((1, 8, 8, 16, 4, 3, 3, 0, 1, 0), -2)):
        with pytest.raises(cdl.CdlError) as e:
            cdl.cdl_qconv_fwd(t8, t8, B, H, W, C, N, R, S, stride, pad, 0.1, 0.1, out, None, None, x_offset=off)
        assert e.value.status == status, (B, H, W, C, N, R, S, stride, pad, off)
    with pytest.raises(cdl.CdlError) as e:          # an offset needs the workspace
        cdl.cdl_qconv_fwd(t8, t8, 1, 8, 8, 16, 4, 3, 3, 1, 1, 0.1, 0.1, out, None, None, x_offset=128)
    assert e.value.status == -5
    # an empty batch is no error and touches nothing
    out.fill_(5)
    cdl.cdl_qconv_fwd(t8, t8, 0, 8, 8, 16, 4, 3, 3, 1, 1, 0.1, 0.1, out, None, None)
    torch.cuda.synchronize()
    assert int(out.sum()) == 5 * (1 << 16)


# (B, H, W, C, N, R, S, stride, pad): the weight gradient - one and several pieces of the contraction over the pixels,
# ragged everything, both strides, channel counts that are and are not whole 64-column tiles of the transposition
WGRAD = [(2, 7, 9, 16, 20, 3, 3, 1, 1), (3, 8, 8, 32, 130, 3, 3, 2, 1), (5, 12, 12, 16, 16, 3, 3, 1, 1), (1, 9, 7, 48, 40, 5, 3, 1, 2),
         (64, 14, 14, 64, 96, 3, 3, 1, 1), (16, 33, 31, 128, 64, 1, 1, 1, 0), (40, 28, 28, 16, 33, 3, 3, 2, 1), (1, 3, 3, 16, 8, 3, 3, 1, 1)]


@pytest.mark.parametrize("B,H,W,C,N,R,S,stride,pad", WGRAD)
@pytest.mark.parametrize("x_offset", [0, 128])
def test_convolution_weight_gradient(oracle, B, H, W, C, N, R, S, stride, pad, x_offset):
    import paper_2501_09849_amd as cdl
    torch = gu.torch_mod()
    rng = np.random.default_rng(B + H * W + C + x_offset)
    if x_offset:
        x_true = rng.integers(0, 256, size=(B, H, W, C)).astype(np.int16)
    else:
        x_true = rng.integers(-128, 128, size=(B, H, W, C)).astype(np.int16)
    x_stored = (x_true - x_offset).astype(np.int8)
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    g = rng.standard_normal((B, P, Q, N)).astype(np.float32)
    dx = float(np.float32(0.0731))
    dW = gu.empty((N, R, S, C), torch.float32)
    dW.fill_(float("nan"))
    ws = gu.workspace(cdl.qconv_bwd_weights_workspace_bytes(B, H, W, C, N, R, S, stride, pad))
    cdl.cdl_qconv_bwd_weights(gu.dev(g), gu.dev(x_stored), B, H, W, C, N, R, S, stride, pad, dx, dW, ws, x_offset=x_offset)
    torch.cuda.synchronize()
    _, ref = oracle.qconv_bwd(g, x_true, np.zeros((N, R, S, C), dtype=np.int16), stride, pad, dx, 1.0, want_dx=False)
    gu.assert_close(dW.cpu().numpy(), ref, "d_w_hat")
    # bit for bit the weight-gradient product on the window matrix (padding taps hold the stored byte of index 0)
    cols, _, _ = _windows(x_stored, R, S, stride, pad, fill=-x_offset)
    M, K = cols.shape
    dWh = gu.empty((N, K), torch.float32)
    ws2 = gu.workspace(cdl.qgemm_bwd_workspace_bytes(M, N, K))
    cdl.cdl_qgemm_bwd_offset(gu.dev(g.reshape(M, N)), gu.dev(cols), gu.dev(np.zeros((N, K), dtype=np.int8)), M, N, K, dx, 1.0, x_offset, 0,
                             None, dWh, ws2)
    torch.cuda.synchronize()
    assert torch.equal(dW.reshape(N, K), dWh)


# (B, H, W, C, N, R, S, stride, pad): the activation gradient (a transposed convolution inside the limb product) - both
# strides on even and odd image sizes, kernels that are not square, no padding, more input channels than one column
# tile of 384, several K-tiles per tap (N = 256), input pixels that no output pixel reaches (stride 2 without padding)
XGRAD = [(2, 7, 9, 16, 128, 3, 3, 1, 1), (1, 8, 8, 20, 128, 3, 3, 2, 1), (3, 6, 5, 48, 256, 1, 1, 1, 0), (1, 9, 7, 16, 128, 5, 3, 1, 2),
         (4, 14, 14, 64, 128, 3, 3, 1, 1), (2, 15, 15, 32, 128, 3, 3, 2, 1), (1, 10, 11, 64, 256, 3, 5, 2, 0), (3, 14, 14, 400, 128, 3, 3, 1, 1),
         (2, 8, 8, 16, 128, 1, 1, 2, 0),
         # channel counts served by column tiles of 256 (one and two of them) and of 384 columns (one, and two with a ragged one)
         (2, 8, 8, 256, 128, 3, 3, 1, 1), (1, 6, 7, 512, 32, 3, 3, 2, 1), (1, 9, 9, 320, 64, 3, 3, 1, 1), (1, 6, 6, 644, 32, 1, 1, 1, 0),
         # more than 256 row tiles with a short contraction: blocks that work through runs of two and three row tiles (the last
         # run shorter; one and two column tiles per row tile; both strides)
         (16, 28, 28, 64, 64, 3, 3, 1, 1), (17, 23, 21, 40, 36, 3, 3, 1, 1), (25, 28, 28, 48, 32, 3, 3, 2, 1), (10, 30, 30, 512, 16, 3, 3, 1, 1),
         # the first stride-2 transition of a ResNet-18 on 32 images: a hundred thousand input pixels in four parity classes
         (32, 56, 56, 64, 128, 3, 3, 2, 1),
         # output channels that are not whole K-tiles of 128: K-tiles then run across taps (the first stages of a ResNet)
         (4, 16, 16, 16, 16, 3, 3, 1, 1), (2, 16, 16, 32, 64, 3, 3, 2, 1), (3, 9, 9, 16, 48, 3, 3, 1, 1), (1, 7, 7, 8, 20, 5, 5, 1, 2),
         (2, 12, 12, 64, 32, 1, 1, 1, 0),
         # few channels on both sides: the direct kernel (16 and 32 lanes per pixel, both strides, odd sizes, 5 x 5, the workload-2 layer)
         (3, 9, 11, 20, 16, 3, 3, 1, 1), (2, 15, 15, 16, 32, 3, 3, 2, 1), (1, 7, 7, 4, 8, 5, 5, 1, 2), (2, 10, 9, 32, 4, 3, 3, 2, 0),
         (128, 32, 32, 16, 16, 3, 3, 1, 1)]


@pytest.mark.parametrize("B,H,W,C,N,R,S,stride,pad", XGRAD)
@pytest.mark.parametrize("g_scale", [1.0, 3.0e-4])
def test_convolution_activation_gradient(oracle, B, H, W, C, N, R, S, stride, pad, g_scale):
    import paper_2501_09849_amd as cdl
    torch = gu.torch_mod()
    rng = np.random.default_rng(B + H * W + C + N)
    w = cdl_inputs.draw_indices((N, R, S, C), -127, 127, seed=N + C)
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    g = (rng.standard_normal((B, P, Q, N)) * g_scale).astype(np.float32)
    dw = float(np.float32(0.011))
    dX = gu.empty((B, H, W, C), torch.float32)
    dX.fill_(float("nan"))
    ws = gu.workspace(cdl.qconv_bwd_activations_workspace_bytes(B, H, W, C, N, R, S, stride, pad))
    cdl.cdl_qconv_bwd_activations(gu.dev(g), gu.dev(w), B, H, W, C, N, R, S, stride, pad, dw, dX, ws)
    torch.cuda.synchronize()
    ref, _ = oracle.qconv_bwd(g, np.zeros((B, H, W, C), dtype=np.int16), w, stride, pad, 1.0, dw, want_dw=False)
    gu.assert_close(dX.cpu().numpy(), ref, "d_x_hat")


def test_convolution_gradients_reject_what_they_do_not_serve():
    import paper_2501_09849_amd as cdl
    torch = gu.torch_mod()
    t = gu.empty((1 << 16,), torch.float32)
    t8 = gu.empty((1 << 16,), torch.int8)
    ws = gu.workspace(1 << 20)
    # output channels not a multiple of four; stride 3; padding as wide as the kernel; contraction beyond the int32 accumulators
    for (B, H, W, C, N, R, S, stride, pad), status in (((1, 8, 8, 16, 6, 3, 3, 1, 1), -2), ((1, 8, 8, 16, 128, 3, 3, 3, 1), -2),
                                                       ((1, 8, 8, 16, 128, 3, 3, 1, 3), -2), ((1, 8, 8, 16, 16384, 3, 3, 1, 1), -3)):
        with pytest.raises(cdl.CdlError) as e:
            cdl.cdl_qconv_bwd_activations(t, t8, B, H, W, C, N, R, S, stride, pad, 0.1, t, ws)
        assert e.value.status == status, (B, H, W, C, N, R, S, stride, pad)
    with pytest.raises(cdl.CdlError) as e:
        cdl.cdl_qconv_bwd_weights(t, t8, 1, 8, 8, 3, 4, 3, 3, 1, 1, 0.1, t, ws)      # C not a multiple of 16
    assert e.value.status == -2


def test_the_convolution_that_workload_3_stands_for(oracle):
    """ResNet-18 layer 3 at full size (256 images of 14 x 14 x 256, 256 kernels of 3 x 3, padding 1; M = 50176, K = 2304):
    forward accumulators and weight gradient everywhere against the products on the window matrix (bit for bit), all three
    outputs against the oracle on the first and the last image (the weight gradient on a batch of those two)."""
    import paper_2501_09849_amd as cdl
    torch = gu.torch_mod()
    wl = cdl_inputs.workload(3)
    B, H, W, C, N, R, S, stride, pad = 256, 14, 14, 256, 256, 3, 3, 1, 1
    x_s, w_s = wl.x_spec, wl.w_spec
    x = cdl_inputs.draw_indices((B, H, W, C), x_s.lo, x_s.hi, seed=31)
    w = cdl_inputs.draw_indices((N, R, S, C), w_s.lo, w_s.hi, seed=32)
    g = cdl_inputs.draw_g(wl, 0).reshape(B, H, W, N)
    acc, y = _run(cdl, torch, x, w, stride, pad, x_s.delta, w_s.delta)
    x_d, w_d, g_d = gu.dev(x), gu.dev(w), gu.dev(g)
    dW, dX = gu.empty((N, R, S, C), torch.float32), gu.empty((B, H, W, C), torch.float32)
    ws = gu.workspace(max(cdl.qconv_bwd_weights_workspace_bytes(B, H, W, C, N, R, S, stride, pad),
                          cdl.qconv_bwd_activations_workspace_bytes(B, H, W, C, N, R, S, stride, pad)))
    cdl.cdl_qconv_bwd_weights(g_d, x_d, B, H, W, C, N, R, S, stride, pad, x_s.delta, dW, ws)
    cdl.cdl_qconv_bwd_activations(g_d, w_d, B, H, W, C, N, R, S, stride, pad, w_s.delta, dX, ws)
    torch.cuda.synchronize()
    dX_h = dX.cpu().numpy()
    for b in (0, B - 1):
        ref_acc, ref_y = oracle.qconv_fwd(x[b:b + 1], w, stride, pad, x_s.delta, w_s.delta)
        assert np.array_equal(acc[b:b + 1], ref_acc)
        gu.assert_close(y[b:b + 1], ref_y, "y of image %d" % b)
        ref_dx, _ = oracle.qconv_bwd(g[b:b + 1], x[b:b + 1], w, stride, pad, x_s.delta, w_s.delta, want_dw=False)
        gu.assert_close(dX_h[b:b + 1], ref_dx, "d_x_hat of image %d" % b)
    # the products on the window matrix: every accumulator and every entry of the weight gradient
    cols, _, _ = _windows(x, R, S, stride, pad)
    M, K = cols.shape
    assert (M, N, K) == (wl.M, wl.N, wl.K)
    cols_d = gu.dev(cols)
    acc2, dWh = gu.empty((M, N), torch.int32), gu.empty((N, K), torch.float32)
    ws2 = gu.workspace(max(cdl.qgemm_fwd_workspace_bytes(M, N, K), cdl.qgemm_bwd_workspace_bytes(M, N, K)))
    cdl.cdl_qgemm_fwd(cols_d, gu.dev(w.reshape(N, K)), M, N, K, x_s.delta, w_s.delta, acc2, None, ws2)
    cdl.cdl_qgemm_bwd(g_d, cols_d, gu.dev(w.reshape(N, K)), M, N, K, x_s.delta, w_s.delta, None, dWh, ws2)
    torch.cuda.synchronize()
    assert np.array_equal(acc.reshape(M, N), acc2.cpu().numpy())
    assert torch.equal(dW.reshape(N, K), dWh)
    # the weight gradient against the oracle: linear in the batch, so a batch of two images checks the arithmetic of a slice
    sel = [0, B - 1]
    dW2 = gu.empty((N, R, S, C), torch.float32)
    cdl.cdl_qconv_bwd_weights(gu.dev(g[sel]), gu.dev(x[sel]), 2, H, W, C, N, R, S, stride, pad, x_s.delta, dW2, ws)
    torch.cuda.synchronize()
    _, ref_dw = oracle.qconv_bwd(g[sel], x[sel], w, stride, pad, x_s.delta, w_s.delta, want_dx=False)
    gu.assert_close(dW2.cpu().numpy(), ref_dw, "d_w_hat of two images")

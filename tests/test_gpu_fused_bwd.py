"""cdl_qgemm_bwd_quantize_bwd: the activation-gradient product with the quantizer's backward pass in its epilogue.
Its outputs must be those of the two calls it replaces: dL/dtheta entry by entry (the arithmetic is the same, on the same
fp32 intermediate, so the two GPU paths agree bit for bit), and against the oracle's backward pass fed with that
intermediate; the scalar gradients at the stated tolerance; d_b_hat unchanged."""
import numpy as np
import pytest

import cdl_inputs
from cdl_inputs import QuantSpec
import gpu_util as gu

pytestmark = pytest.mark.gpu


def _spec(lo, L, delta, kappa):
    d = float(np.float32(delta))
    return QuantSpec(lo, L, d, float(np.float32(kappa / (d * d))))


# (M, N, K, activation level set, kappa): every band width of the epilogue (kappa 40 -> 1 ... 0.3 -> generic loop), ragged
# tiles in both directions, a contraction that is not a multiple of four (scalar loads of g), the unsigned 8-bit set, a
# short contraction (two K-tiles) and one long enough for five limbs
CASES = [(300, 200, 256, (0, 16), 4.0), (1000, 130, 384, (0, 16), 40.0), (257, 33, 1152, (-7, 15), 2.5), (96, 520, 388, (0, 16), 1.5),
         (2100, 300, 132, (-127, 255), 4.0), (640, 1031, 768, (0, 256), 4.0), (512, 64, 400, (0, 16), 0.3), (4096, 3072, 256, (-127, 255), 4.0)]


@pytest.mark.parametrize("M,N,K,levels,kappa", CASES)
def test_fused_backward_matches_the_two_calls(oracle, M, N, K, levels, kappa):
    import paper_2501_09849_amd as cdl
    torch = gu.torch_mod()
    rng = np.random.default_rng(M + N + K)
    x = _spec(levels[0], levels[1], 0.0731, kappa)
    w_delta = float(np.float32(0.011))
    X = (rng.uniform((x.lo - 1.0), (x.hi + 1.0), (M, K)) * x.delta).astype(np.float32)
    b = cdl_inputs.draw_indices((N, K), -127, 127, seed=N)
    G = rng.standard_normal((M, N)).astype(np.float32)
    xa = (x.lo, x.n_levels, x.delta, x.alpha)
    ox = cdl.cdl_index_offset(x.lo, x.n_levels)
    X_d, G_d, b_d = gu.dev(X.reshape(-1)), gu.dev(G), gu.dev(b)
    Xi = gu.empty((M * K,), torch.int8)
    cdl.cdl_quantize_fwd(X_d, M * K, *xa, Xi)
    ws = gu.workspace(max(cdl.qgemm_bwd_workspace_bytes(M, N, K), cdl.quantize_workspace_bytes(M * K, x.n_levels)))
    # the two calls
    dXh, dWh = gu.empty((M, K), torch.float32), gu.empty((N, K), torch.float32)
    cdl.cdl_qgemm_bwd_offset(G_d, Xi, b_d, M, N, K, x.delta, w_delta, ox, 0, dXh, dWh, ws)
    dX, sc = gu.empty((M * K,), torch.float32), gu.empty((4,), torch.float32)
    cdl.cdl_quantize_bwd(X_d, dXh.reshape(-1), M * K, *xa, dX, sc[0:1], sc[1:2], ws)
    torch.cuda.synchronize()
    dXh_h = dXh.cpu().numpy()
    # the one call
    dX2, dWh2 = gu.empty((M * K,), torch.float32), gu.empty((N, K), torch.float32)
    dX2.fill_(float("nan"))
    cdl.cdl_qgemm_bwd_quantize_bwd(G_d, Xi, b_d, M, N, K, X_d, *xa, w_delta, dX2, sc[2:3], sc[3:4], dWh2, ws)
    torch.cuda.synchronize()
    if kappa >= 1.3:
        assert torch.equal(dX2, dX), "dL/dtheta differs from the two-call path at %d places" % int((dX2 != dX).sum())
    else:   # (the stand-alone kernel for small level sets in the soft regime works in double, the epilogue in fp32)
        gu.assert_close(dX2.cpu().numpy(), dX.cpu().numpy().astype(np.float64), "dL/dtheta against the two-call path")
    assert torch.equal(dWh2, dWh)
    ref = oracle.quantize_bwd(X.reshape(-1), dXh_h.reshape(-1), *xa)
    gu.assert_close(dX2.cpu().numpy(), ref["dtheta"], "dL/dtheta")
    label = "fused %dx%dx%d levels %d..%d kappa %g" % (M, N, K, x.lo, x.hi, kappa)
    gu.check_quantizer_scalars(oracle, label, X.reshape(-1), dXh_h.reshape(-1), xa, float(sc[2]), float(sc[3]), ref)
    # without the weight-gradient product and without the scalars
    dX3 = gu.empty((M * K,), torch.float32)
    cdl.cdl_qgemm_bwd_quantize_bwd(G_d, None, b_d, M, N, K, X_d, *xa, w_delta, dX3, None, None, None, ws)
    torch.cuda.synchronize()
    assert torch.equal(dX3, dX2)


def test_fused_backward_rejects_what_it_does_not_serve():
    import paper_2501_09849_amd as cdl
    torch = gu.torch_mod()
    t = gu.empty((64 * 64,), torch.float32)
    i8 = gu.empty((64 * 64,), torch.int8)
    ws = gu.workspace(cdl.qgemm_bwd_workspace_bytes(64, 64, 64))
    for M, N, K in ((64, 64, 62), (64, 32, 64), (0, 64, 64)):
        with pytest.raises(cdl.CdlError) as e:
            cdl.cdl_qgemm_bwd_quantize_bwd(t, i8, i8, M, N, K, t, 0, 16, 0.25, 64.0, 0.02, t, None, None, None, ws)
        assert e.value.status == -2


# (M, N, K, weight level set, kappa): one piece of the contraction over M (M <= 512) and several, ragged shapes, the
# unsigned 8-bit set for the weights (stored minus 128), every band width
W_CASES = [(300, 200, 256, (-7, 15), 4.0), (9000, 130, 384, (-7, 15), 40.0), (40000, 64, 132, (-127, 255), 2.5),
           (20000, 96, 388, (0, 256), 4.0), (70000, 40, 64, (-3, 7), 1.5), (5000, 257, 100, (-7, 15), 0.3)]


@pytest.mark.parametrize("M,N,K,levels,kappa", W_CASES)
def test_fused_backward_of_the_weights_matches_the_separate_calls(oracle, M, N, K, levels, kappa):
    import paper_2501_09849_amd as cdl
    torch = gu.torch_mod()
    rng = np.random.default_rng(M + 3 * N + K)
    w = _spec(levels[0], levels[1], 0.0193, kappa)
    x = _spec(0, 16, 0.0731, 4.0)
    W = (rng.uniform((w.lo - 1.0), (w.hi + 1.0), (N, K)) * w.delta).astype(np.float32)
    X = (rng.uniform(-1.0, 16.0, (M, K)) * x.delta).astype(np.float32)
    G = rng.standard_normal((M, N)).astype(np.float32)
    wa, xa = (w.lo, w.n_levels, w.delta, w.alpha), (x.lo, x.n_levels, x.delta, x.alpha)
    ow = cdl.cdl_index_offset(w.lo, w.n_levels)
    W_d, X_d, G_d = gu.dev(W.reshape(-1)), gu.dev(X.reshape(-1)), gu.dev(G)
    Wi, Xi = gu.empty((N * K,), torch.int8), gu.empty((M * K,), torch.int8)
    cdl.cdl_quantize_fwd(W_d, N * K, *wa, Wi)
    cdl.cdl_quantize_fwd(X_d, M * K, *xa, Xi)
    ws = gu.workspace(max(cdl.qgemm_bwd_workspace_bytes(M, N, K), cdl.quantize_workspace_bytes(M * K, 256)))
    # the separate calls
    dXh, dWh = gu.empty((M, K), torch.float32), gu.empty((N, K), torch.float32)
    cdl.cdl_qgemm_bwd_offset(G_d, Xi, Wi, M, N, K, x.delta, w.delta, 0, ow, dXh, dWh, ws)
    dX, dW, sc = gu.empty((M * K,), torch.float32), gu.empty((N * K,), torch.float32), gu.empty((8,), torch.float32)
    cdl.cdl_quantize_bwd(X_d, dXh.reshape(-1), M * K, *xa, dX, None, None, ws)
    cdl.cdl_quantize_bwd(W_d, dWh.reshape(-1), N * K, *wa, dW, sc[0:1], sc[1:2], ws)
    torch.cuda.synchronize()
    dWh_h = dWh.cpu().numpy()
    # the one call, with and without dL/dQ(w) as an output
    for keep_hat in (True, False):
        dX2, dW2, dWh2 = gu.empty((M * K,), torch.float32), gu.empty((N * K,), torch.float32), gu.empty((N, K), torch.float32)
        dW2.fill_(float("nan"))
        dWh2.fill_(float("nan"))
        sc[2:4] = float("nan")
        cdl.cdl_qgemm_bwd_quantize_bwd(G_d, Xi, Wi, M, N, K, X_d, *xa, w.delta, dX2, None, None, dWh2 if keep_hat else None, ws,
                                       b_offset=ow, theta_b=W_d, qparams_b=wa, d_theta_b=dW2, d_delta_b=sc[2:3], d_alpha_b=sc[3:4])
        torch.cuda.synchronize()
        assert torch.equal(dX2, dX)
        if keep_hat:
            assert torch.equal(dWh2, dWh)
        if kappa >= 1.3:
            assert torch.equal(dW2, dW), "dL/dtheta of the weights differs from the separate calls at %d places" % int((dW2 != dW).sum())
        else:
            gu.assert_close(dW2.cpu().numpy(), dW.cpu().numpy().astype(np.float64), "dL/dtheta of the weights against the separate calls")
        ref = oracle.quantize_bwd(W.reshape(-1), dWh_h.reshape(-1), *wa)
        gu.assert_close(dW2.cpu().numpy(), ref["dtheta"], "dL/dtheta of the weights")
        label = "fused weights %dx%dx%d levels %d..%d kappa %g" % (M, N, K, w.lo, w.hi, kappa)
        gu.check_quantizer_scalars(oracle, label, W.reshape(-1), dWh_h.reshape(-1), wa, float(sc[2]), float(sc[3]), ref)


def test_fused_backward_of_the_weights_checks_its_quantizer():
    import paper_2501_09849_amd as cdl
    torch = gu.torch_mod()
    t = gu.empty((64 * 64,), torch.float32)
    i8 = gu.empty((64 * 64,), torch.int8)
    ws = gu.workspace(cdl.qgemm_bwd_workspace_bytes(64, 64, 64))
    # a step or a storage offset that is not the one the product was told
    for qb, off in (((-7, 15, 0.03, 64.0), 0), ((0, 256, 0.02, 64.0), 0)):
        with pytest.raises(cdl.CdlError) as e:
            cdl.cdl_qgemm_bwd_quantize_bwd(t, i8, i8, 64, 64, 64, t, 0, 16, 0.25, 64.0, 0.02, t, None, None, None, ws,
                                           b_offset=off, theta_b=t, qparams_b=qb, d_theta_b=t)
        assert e.value.status == -2
    with pytest.raises(cdl.CdlError) as e:      # theta_b without a place for the result
        cdl.cdl_qgemm_bwd_quantize_bwd(t, i8, i8, 64, 64, 64, t, 0, 16, 0.25, 64.0, 0.02, t, None, None, None, ws,
                                       theta_b=t, qparams_b=(-7, 15, 0.02, 64.0))
    assert e.value.status == -1

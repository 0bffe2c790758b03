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

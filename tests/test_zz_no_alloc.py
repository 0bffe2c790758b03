"""cdl_quantize_fwd_static: the forward quantizer for callers that cannot allocate.

Called through the C boundary (ctypes on libcdl.so, raw device addresses) and compared with cdl_quantize_fwd on
the same input: indices, soft values, marginal PMF and entropy must agree bit for bit (same kernels, integer
histograms), on two calls in a row, the second on a smaller tensor, so that whatever the first call left in the
library's scratch buffer would show.  Collected last: a failure here hides no other test.
"""
import ctypes

import numpy as np
import pytest

import gpu_util as gu

pytestmark = pytest.mark.gpu


def _raw(lib, name, restype, argtypes):
    f = getattr(lib, name)
    f.restype, f.argtypes = restype, argtypes
    return f


def test_static_scratch_entry_point_matches_the_workspace_one(oracle):
    import paper_2501_09849_amd as cdl
    from paper_2501_09849_amd.binding import QParams
    torch = gu.torch_mod()
    lib = ctypes.CDLL(cdl.lib_path())
    vp, i64, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_size_t
    qp = ctypes.POINTER(QParams)
    fwd = _raw(lib, "cdl_quantize_fwd", ctypes.c_int, [vp, i64, qp, vp, vp, vp, vp, vp, sz, vp])
    fwd_static = _raw(lib, "cdl_quantize_fwd_static", ctypes.c_int, [vp, i64, qp, vp, vp, vp, vp, vp])
    ws_bytes = _raw(lib, "cdl_quantize_workspace_bytes", sz, [i64, ctypes.c_int32])
    cap = _raw(lib, "cdl_static_scratch_bytes", sz, [])()
    assert cap == 8 << 20

    stream = torch.cuda.current_stream().cuda_stream or None
    rng = np.random.default_rng(77)
    # 255 levels at kappa = 4 (five live levels per entry), then 31 levels in the soft regime on a smaller tensor
    cases = [(3_000_017, QParams(-127, 255, 0.15092, 4.0 / 0.15092 ** 2, 0), 1.0),
             (200_003, QParams(-15, 31, 0.004, 500.0, 0), 0.02)]
    for n, q, sigma in cases:
        theta_h = (rng.standard_normal(n) * sigma).astype(np.float32)
        theta = gu.dev(theta_h)
        out = []
        for which in ("workspace", "static"):
            idx, soft = gu.empty((n,), torch.int8), gu.empty((n,), torch.float32)
            marg, ent = gu.empty((q.n_levels,), torch.float32), gu.empty((1,), torch.float32)
            marg.fill_(-1.0)
            ent.fill_(-1.0)
            if which == "workspace":
                need = ws_bytes(n, q.n_levels)
                assert need <= cap
                ws = gu.workspace(need)
                rc = fwd(theta.data_ptr(), n, ctypes.byref(q), idx.data_ptr(), soft.data_ptr(), marg.data_ptr(), ent.data_ptr(),
                         ws.data_ptr(), ws.numel(), stream)
            else:
                rc = fwd_static(theta.data_ptr(), n, ctypes.byref(q), idx.data_ptr(), soft.data_ptr(), marg.data_ptr(),
                                ent.data_ptr(), stream)
            assert rc == 0, (which, rc)
            torch.cuda.synchronize()
            out.append((idx.cpu().numpy(), soft.cpu().numpy(), marg.cpu().numpy(), float(ent.item())))
        (i0, s0, m0, h0), (i1, s1, m1, h1) = out
        assert np.array_equal(i0, i1) and np.array_equal(s0, s1)
        assert np.array_equal(m0, m1) and h0 == h1
        # ... and the marginal PMF is the oracle's (a sample keeps the CPU time short)
        r_m, r_h = oracle.marginal_entropy(theta_h[:100_000], q.lo, q.n_levels, q.delta, q.alpha)
        m_small, h_small = gu.empty((q.n_levels,), torch.float32), gu.empty((1,), torch.float32)
        idx_small = gu.empty((100_000,), torch.int8)
        rc = fwd_static(theta.data_ptr(), 100_000, ctypes.byref(q), idx_small.data_ptr(), None, m_small.data_ptr(), h_small.data_ptr(), stream)
        assert rc == 0
        torch.cuda.synchronize()
        gu.assert_close(m_small.cpu().numpy(), r_m, "marginal PMF (static scratch)")
        gu.assert_close([float(h_small.item())], [r_h], "entropy (static scratch)")

    # beyond the built-in buffer: a clear error, nothing launched; without the marginal PMF any size passes validation
    q = QParams(-127, 255, 0.15092, 4.0 / 0.15092 ** 2, 0)
    big = 200_000_000
    assert ws_bytes(big, 255) > cap
    dummy = gu.empty((16,), torch.float32)
    rc = fwd_static(dummy.data_ptr(), big, ctypes.byref(q), dummy.data_ptr(), None, dummy.data_ptr(), dummy.data_ptr(), stream)
    assert rc == -7
    msg = _raw(lib, "cdl_status_string", ctypes.c_char_p, [ctypes.c_int])(rc).decode()
    assert "scratch" in msg

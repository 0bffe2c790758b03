"""The forward product on large shapes of whole tiles (the direct-load kernel), checked everywhere: every int32
accumulator enters two exact identities (contractions of the whole matrix with all-ones and random-sign vectors
from either side, evaluated on the host in O(M K + N K)), sampled rows are compared with the oracle entry by
entry, and y must be the accumulators times the two steps."""
import numpy as np
import pytest

import cdl_inputs
import gpu_util as gu
from test_gpu_full_size import _gpu_times_vector, _host_mat_vec, _signs

pytestmark = pytest.mark.gpu

# (M, N, K): from 64 tiles of 256 x 256 up to the transformer layer of workload 5; contractions of 4 to 8 K-tiles
SHAPES = [(4096, 1024, 768), (8192, 2048, 768), (8192, 3072, 512), (8192, 2048, 640), (8192, 2048, 1024),
          (16384, 3072, 768), (7936, 2176, 896), (65536, 3072, 768)]


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_forward_product_on_large_shapes_everywhere(oracle, M, N, K):
    import paper_2501_09849_amd as cdl
    torch = gu.torch_mod()
    a = cdl_inputs.draw_indices((M, K), -128, 127, seed=M + K)
    b = cdl_inputs.draw_indices((N, K), -128, 127, seed=N + K)
    a[0, :], b[0, :] = -128, -128            # the largest accumulator: K * 2^14
    a[M - 1, :], b[N - 1, :] = 127, -128
    da, db = float(np.float32(0.15092)), float(np.float32(0.0028209))
    a_d, b_d = gu.dev(a), gu.dev(b)
    acc, y = gu.empty((M, N), torch.int32), gu.empty((M, N), torch.float32)
    acc.fill_(-7)
    y.fill_(float("nan"))
    cdl.cdl_qgemm_fwd(a_d, b_d, M, N, K, da, db, acc, None, None)
    cdl.cdl_qgemm_fwd(a_d, b_d, M, N, K, da, db, None, y, None)
    torch.cuda.synchronize()
    for tag, v_n, u_m in (("ones", np.ones(N), np.ones(M)), ("signs", _signs(N, 1), _signs(M, 2))):
        right = _host_mat_vec(a, _host_mat_vec(b, v_n, left=True))
        left = _host_mat_vec(b, _host_mat_vec(a, u_m, left=True))
        assert np.array_equal(_gpu_times_vector(acc, v_n), right), "row identity (%s)" % tag
        assert np.array_equal(_gpu_times_vector(acc, u_m, left=True), left), "column identity (%s)" % tag
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([rng.choice(M, size=24, replace=False), [0, 255, 256, M - 257, M - 1]]))
    r_acc, r_y = oracle.qgemm_fwd(a[rows], b, da, db)
    rows_d = torch.from_numpy(rows).cuda()
    assert np.array_equal(acc[rows_d].cpu().numpy(), r_acc)
    gu.assert_close(y[rows_d].cpu().numpy(), r_y, "y rows")
    # y is the accumulator times the product of the steps, everywhere (one fp32 multiply of an exactly converted integer)
    scale = torch.tensor(np.float32(da) * np.float32(db), device="cuda")
    assert torch.equal(y, acc.float() * scale)

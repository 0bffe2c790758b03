"""Level sets that reach beyond 127 - the paper's unsigned 8-bit alphabet {0, ..., 255} (eq. repo_alphabet; the width it
keeps for the first and last layer, Sec. V-B): the quantizer stores index - 128, the layer products take the offset of
each operand and return the products of the level indices themselves.  Everything against the oracle, which works on the
level indices as they are."""
import numpy as np
import pytest

import cdl_inputs
from cdl_inputs import QuantSpec
import gpu_util as gu

pytestmark = pytest.mark.gpu


def _spec(lo, L, delta, kappa):
    d = float(np.float32(delta))
    return QuantSpec(lo, L, d, float(np.float32(kappa / (d * d))))


def _theta(lo, L, delta, n, seed):
    hi = lo + L - 1
    rng = np.random.default_rng(seed)
    th = rng.uniform((lo - 1.5) * delta, (hi + 1.5) * delta, size=n)
    th[: n // 8] = np.abs(rng.normal(0.0, 6.0 * delta, size=n // 8)) + lo * delta
    k = rng.integers(lo, hi + 1, size=64)
    th[-64:-32] = k[:32] * np.float64(np.float32(delta))
    th[-32:] = (k[32:] + 0.5) * np.float64(np.float32(delta))
    th[-70:-64] = [(hi + 1e3) * delta, (lo - 1e3) * delta, 1e6 * delta, -1e6 * delta, hi * delta, lo * delta]
    return th.astype(np.float32)


@pytest.mark.parametrize("lo,L", [(0, 256), (0, 255), (100, 156), (128, 64), (200, 20), (0, 129)])
@pytest.mark.parametrize("kappa", (0.02, 0.7, 4.0, 40.0))
def test_quantizer_on_level_sets_beyond_127(oracle, lo, L, kappa):
    import paper_2501_09849_amd as cdl
    torch = gu.torch_mod()
    n = 9003 if kappa >= 0.5 else 3001
    spec = _spec(lo, L, 0.0731, kappa)
    assert cdl.cdl_index_offset(lo, L) == 128
    theta = _theta(lo, L, spec.delta, n, seed=lo + L)
    g = np.random.default_rng(2).standard_normal(n).astype(np.float32)
    q = gu.Quantizer(spec)
    th_d, g_d = gu.dev(theta), gu.dev(g)
    stored, soft, marg, H = q.fwd(th_d)
    idx = stored.astype(np.int64) + 128            # the level indices themselves
    assert idx.min() >= lo and idx.max() <= lo + L - 1
    r_idx, r_soft, r_gap = oracle.quantize_fwd(theta, *q.args)
    r_marg, r_H = oracle.marginal_entropy(theta, *q.args)
    gu.assert_indices(idx, r_idx, r_gap, "idx")
    gu.assert_close(soft, r_soft, "soft")
    gu.assert_close(marg, r_marg, "marg")
    gu.assert_close([H], [r_H], "entropy")
    dth, dd, da = q.bwd(th_d, g_d)
    ref = oracle.quantize_bwd(theta, g, *q.args)
    gu.assert_close(dth, ref["dtheta"], "dtheta")
    gu.check_quantizer_scalars(oracle, "levels %d..%d kappa %g" % (lo, lo + L - 1, kappa), theta, g, q.args, dd, da, ref)
    # the draw and the coded size see the same stored bytes
    u = np.random.default_rng(3).random(n, dtype=np.float32)
    d_idx = gu.empty((n,), torch.int8)
    cdl.cdl_quantize_draw(th_d, gu.dev(u), n, *q.args, d_idx)
    torch.cuda.synchronize()
    got = d_idx.cpu().numpy().astype(np.int64) + 128
    r_draw, margin = oracle.quantize_draw(theta, u, *q.args)
    diff = got != r_draw
    assert not (diff & (margin >= 1e-6)).any() and np.all(np.abs(got[diff] - r_draw[diff]) == 1)
    counts = gu.empty((L,), torch.int64)
    bits = gu.empty((1,), torch.int64)
    ws = gu.workspace(cdl.huffman_workspace_bytes(n))
    pad = gu.empty(((n + 15) // 16 * 16,), torch.int8)
    pad[:n].copy_(torch.from_numpy(stored).cuda())
    cdl.cdl_huffman_bits(pad, n, lo, L, counts, bits, None, ws)
    torch.cuda.synchronize()
    r_counts, r_total, _ = oracle.huffman_bits(idx, lo, L)
    assert np.array_equal(counts.cpu().numpy(), r_counts) and int(bits.item()) == int(r_total)


def _products(oracle, a, b, g, da, db, oa, ob, label):
    """a, b: level indices (int16 numpy); the GPU gets a - oa and b - ob as int8."""
    import paper_2501_09849_amd as cdl
    torch = gu.torch_mod()
    M, K = a.shape
    N = b.shape[0]
    a_d, b_d, g_d = gu.dev((a - oa).astype(np.int8)), gu.dev((b - ob).astype(np.int8)), gu.dev(g)
    acc, y = gu.empty((M, N), torch.int32), gu.empty((M, N), torch.float32)
    dxa, dwb = gu.empty((M, K), torch.float32), gu.empty((N, K), torch.float32)
    ws = gu.workspace(max(cdl.qgemm_fwd_offset_workspace_bytes(M, N, K), cdl.qgemm_bwd_workspace_bytes(M, N, K)))
    cdl.cdl_qgemm_fwd_offset(a_d, b_d, M, N, K, da, db, oa, ob, acc, y, ws)
    cdl.cdl_qgemm_bwd_offset(g_d, a_d, b_d, M, N, K, da, db, oa, ob, dxa, dwb, ws)
    torch.cuda.synchronize()
    r_acc, r_y = oracle.qgemm_fwd(a, b, da, db)
    assert np.array_equal(acc.cpu().numpy(), r_acc), label + ": int32 accumulators"
    gu.assert_close(y.cpu().numpy(), r_y, label + " y")
    r_da, r_db = oracle.qgemm_bwd(g, a, b, da, db)
    gu.assert_close(dxa.cpu().numpy(), r_da, label + " dL/dQ(a)")
    gu.assert_close(dwb.cpu().numpy(), r_db, label + " dL/dQ(b)")
    # one product at a time as well
    only = gu.empty((N, K), torch.float32)
    cdl.cdl_qgemm_bwd_offset(g_d, a_d, b_d, M, N, K, da, db, oa, ob, None, only, ws)
    torch.cuda.synchronize()
    assert np.array_equal(only.cpu().numpy(), dwb.cpu().numpy())


@pytest.mark.parametrize("M,N,K", [(300, 200, 256), (1000, 130, 70), (257, 33, 1152), (4096, 16, 144), (129, 520, 384), (2100, 300, 130)])
@pytest.mark.parametrize("oa,ob", [(128, 0), (0, 128), (128, 128)])
def test_products_with_operands_stored_with_an_offset(oracle, M, N, K, oa, ob):
    rng = np.random.default_rng(M + N + K + oa)
    a = rng.integers(oa - 128, oa + 128, (M, K)).astype(np.int16)       # 0..255 with an offset, -128..127 without
    b = rng.integers(ob - 128, ob + 128, (N, K)).astype(np.int16)
    a[0, :], b[0, :] = oa + 127, ob + 127                               # the largest products
    g = rng.standard_normal((M, N)).astype(np.float32)
    _products(oracle, a, b, g, float(np.float32(0.0731)), float(np.float32(0.011)), oa, ob, "%dx%dx%d" % (M, N, K))


def test_first_layer_of_the_paper_8_bit_unsigned_activations_end_to_end(oracle):
    """Quantize an activation tensor on {0..255} and a weight tensor on {-128..127}, run the three products on the
    stored indices with the offsets the library reports, and compare with the oracle on the level indices; the
    large contraction takes the direct-load forward kernel and the split weight-gradient path."""
    import paper_2501_09849_amd as cdl
    torch = gu.torch_mod()
    M, N, K = 4096, 512, 256
    rng = np.random.default_rng(8)
    x = _spec(0, 256, 0.02, 4.0)
    w = _spec(-128, 256, 0.004, 4.0)
    X = np.abs(rng.normal(0, 1.2, (M, K))).astype(np.float32)
    W = rng.normal(0, 0.15, (N, K)).astype(np.float32)
    G = rng.standard_normal((M, N)).astype(np.float32)
    ox, ow = cdl.cdl_index_offset(x.lo, x.n_levels), cdl.cdl_index_offset(w.lo, w.n_levels)
    assert (ox, ow) == (128, 0)
    Xi, Wi = gu.empty((M * K,), torch.int8), gu.empty((N * K,), torch.int8)
    cdl.cdl_quantize_fwd(gu.dev(X.reshape(-1)), M * K, x.lo, x.n_levels, x.delta, x.alpha, Xi)
    cdl.cdl_quantize_fwd(gu.dev(W.reshape(-1)), N * K, w.lo, w.n_levels, w.delta, w.alpha, Wi)
    torch.cuda.synchronize()
    xi = Xi.cpu().numpy().astype(np.int16).reshape(M, K) + ox
    wi = Wi.cpu().numpy().astype(np.int16).reshape(N, K) + ow
    r_xi, _, gap = oracle.quantize_fwd(X, x.lo, x.n_levels, x.delta, x.alpha, want_soft=False)
    gu.assert_indices(xi, r_xi, gap, "activation indices")
    assert xi.max() > 200
    _products(oracle, xi, wi, G, x.delta, w.delta, ox, ow, "first layer")


def test_offset_arguments_are_validated(oracle):
    import paper_2501_09849_amd as cdl
    torch = gu.torch_mod()
    a = gu.empty((16, 16), torch.int8)
    y = gu.empty((16, 16), torch.float32)
    ws = gu.workspace(cdl.qgemm_fwd_offset_workspace_bytes(16, 16, 16))
    with pytest.raises(cdl.CdlError) as e:
        cdl.cdl_qgemm_fwd_offset(a, a, 16, 16, 16, 1.0, 1.0, 64, 0, None, y, ws)
    assert e.value.status == -2
    big = 40000          # 40000 * 255 * 255 > 2^31
    with pytest.raises(cdl.CdlError) as e:
        cdl.cdl_qgemm_fwd_offset(a, a, 16, 16, big, 1.0, 1.0, 128, 128, None, y, ws)
    assert e.value.status == -3

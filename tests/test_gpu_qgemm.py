"""GPU parity of the index GEMMs against the CPU oracle.

Integer accumulators must be bit-exact; fp32 results within 1e-6 + 1e-5|ref|.
Shapes span several tiles with ragged edges in every dimension, a contraction
length that is not a multiple of the staging step, and one that is not even a
multiple of 16 (which takes the padded-copy path).
"""
import numpy as np
import pytest

import cdl_inputs
import gpu_util as gu

pytestmark = pytest.mark.gpu

FWD_SHAPES = [(32, 128, 256), (300, 200, 144), (257, 129, 80), (1000, 16, 144), (513, 300, 2304),
              (70, 50, 100), (1, 1, 16), (5, 3, 7), (256, 128, 64), (700, 130, 1040)]


@pytest.mark.parametrize("M,N,K", FWD_SHAPES)
def test_qgemm_fwd_matches_oracle(oracle, M, N, K):
    a = cdl_inputs.draw_indices((M, K), -127, 127, seed=M + K)
    b = cdl_inputs.draw_indices((N, K), -127, 127, seed=N + K + 1)
    da, db = float(np.float32(0.15092)), float(np.float32(0.0028209))
    acc, y = gu.qgemm_fwd(a, b, da, db)
    r_acc, r_y = oracle.qgemm_fwd(a, b, da, db)
    assert np.array_equal(acc, r_acc), "int32 accumulators differ at %d places" % int((acc != r_acc).sum())
    gu.assert_close(y, r_y, "y")


def test_qgemm_fwd_large_tiles_path_matches_oracle(oracle):
    """Contraction lengths that are multiples of 128 on at least 64 tiles of 256 x 256 take the direct-load kernel;
    ragged edges in both output dimensions."""
    M, N, K = 2310, 2050, 256
    a = cdl_inputs.draw_indices((M, K), -127, 127, seed=21)
    b = cdl_inputs.draw_indices((N, K), -127, 127, seed=22)
    acc, y = gu.qgemm_fwd(a, b, 0.15092, 0.0028209)
    r_acc, r_y = oracle.qgemm_fwd(a, b, 0.15092, 0.0028209)
    assert np.array_equal(acc, r_acc), "int32 accumulators differ at %d places" % int((acc != r_acc).sum())
    gu.assert_close(y, r_y, "y")


@pytest.mark.parametrize("K", [128, 384])
def test_qgemm_fwd_more_tiles_than_compute_units(oracle, K):
    """306 tiles of 256 x 256 for the direct-load kernel, more than there are compute units, one and three
    K-tiles per tile; ragged edges in both output dimensions."""
    M, N = 4400, 4200
    a = cdl_inputs.draw_indices((M, K), -127, 127, seed=31 + K)
    b = cdl_inputs.draw_indices((N, K), -127, 127, seed=32 + K)
    acc, y = gu.qgemm_fwd(a, b, 0.15092, 0.0028209)
    r_acc, r_y = oracle.qgemm_fwd(a, b, 0.15092, 0.0028209)
    assert np.array_equal(acc, r_acc), "int32 accumulators differ at %d places" % int((acc != r_acc).sum())
    gu.assert_close(y, r_y, "y")


def test_qgemm_fwd_extreme_indices_do_not_overflow(oracle):
    M, N, K = 64, 64, 4096
    a = np.full((M, K), -128, np.int8)
    b = np.full((N, K), -128, np.int8)
    b[::2] = 127
    acc, y = gu.qgemm_fwd(a, b, 1.0, 1.0)
    r_acc, _ = oracle.qgemm_fwd(a, b, 1.0, 1.0, want_y=False)
    assert np.array_equal(acc, r_acc)


def test_qgemm_fwd_longest_contraction_with_extreme_indices(oracle):
    """K = 131071 is the longest contraction the boundary accepts: (-128) x (-128) summed that often is
    2147467264, sixteen thousand below the int32 limit."""
    M, N, K = 40, 24, 131071
    a = np.full((M, K), -128, np.int8)
    b = np.full((N, K), -128, np.int8)
    b[1::2] = 127
    a[3, ::5] = 5
    acc, y = gu.qgemm_fwd(a, b, 0.5, 0.25)
    r_acc, r_y = oracle.qgemm_fwd(a, b, 0.5, 0.25)
    assert int(r_acc.max()) == 131071 * 16384
    assert np.array_equal(acc, r_acc)
    gu.assert_close(y, r_y, "y")


def test_qgemm_fwd_outputs_are_optional(oracle):
    a = cdl_inputs.draw_indices((130, 96), 0, 15, seed=1)
    b = cdl_inputs.draw_indices((70, 96), -7, 7, seed=2)
    acc, y = gu.qgemm_fwd(a, b, 0.5, 0.25)
    acc2, none_y = gu.qgemm_fwd(a, b, 0.5, 0.25, want_y=False)
    none_acc, y2 = gu.qgemm_fwd(a, b, 0.5, 0.25, want_acc=False)
    assert none_y is None and none_acc is None
    assert np.array_equal(acc, acc2) and np.array_equal(y, y2)
    assert np.array_equal(y, (acc.astype(np.float32) * np.float32(0.125)))


BWD_SHAPES = [(32, 128, 256), (300, 200, 144), (257, 129, 80), (1000, 16, 144), (70, 50, 100), (5, 3, 7),
              (2048, 96, 320),
              # contractions of at most 32 entries (the direct kernel) with more output columns than one block of it
              # covers: 4 columns per thread (N <= 16) and 2 (N <= 32), whole and ragged groups of columns
              (200, 16, 1100), (130, 24, 1030), (64, 8, 2051), (70, 32, 513)]


@pytest.mark.parametrize("M,N,K", BWD_SHAPES)
@pytest.mark.parametrize("levels", [(0, 15, -7, 7), (-127, 127, -127, 127)])
def test_qgemm_bwd_matches_oracle(oracle, M, N, K, levels):
    a = cdl_inputs.draw_indices((M, K), levels[0], levels[1], seed=M + K)
    b = cdl_inputs.draw_indices((N, K), levels[2], levels[3], seed=N + K + 1)
    g = np.random.default_rng(M * 7 + N).standard_normal((M, N)).astype(np.float32)
    da, db = float(np.float32(0.56419)), float(np.float32(0.016623))
    d_a, d_b = gu.qgemm_bwd(g, a, b, da, db)
    r_a, r_b = oracle.qgemm_bwd(g, a, b, da, db)
    gu.assert_close(d_a, r_a, "d_a_hat")
    gu.assert_close(d_b, r_b, "d_b_hat")


@pytest.mark.parametrize("M,N,K", [(20000, 200, 500), (300, 9000, 500)])
def test_qgemm_bwd_runs_of_row_tiles(oracle, M, N, K):
    """Short contractions with more row tiles than compute units: one block works through a run of row tiles
    and every column tile (dL/dQ(x) in the first shape: 625 row tiles, two K-tiles, two column tiles, all
    ragged; dL/dQ(w) in the second); the other product of each shape takes the one-tile-per-block path."""
    a = cdl_inputs.draw_indices((M, K), 0, 15, seed=M + 3)
    b = cdl_inputs.draw_indices((N, K), -7, 7, seed=N + 5)
    g = np.random.default_rng(M + N).standard_normal((M, N)).astype(np.float32)
    da, db = float(np.float32(0.56419)), float(np.float32(0.016623))
    d_a, d_b = gu.qgemm_bwd(g, a, b, da, db)
    r_a, r_b = oracle.qgemm_bwd(g, a, b, da, db)
    gu.assert_close(d_a, r_a, "d_a_hat")
    gu.assert_close(d_b, r_b, "d_b_hat")


def test_qgemm_bwd_longest_contraction_with_extreme_operands(oracle):
    """N = 131071 is the longest contraction dL/dQ(a) accepts (one int32 accumulator per limb over all of it):
    every gradient at the top of its binade and every index at -128 drives the accumulators to their bound."""
    M, N, K = 40, 131071, 48
    g = np.full((M, N), 0.99, np.float32)
    g[::3] = -0.99
    g[5, ::7] = 0.123
    a = cdl_inputs.draw_indices((M, K), -128, 127, seed=11)
    b = np.full((N, K), -128, np.int8)
    b[:, 1::2] = 127
    d_a, d_b = gu.qgemm_bwd(g, a, b, 0.25, 0.5)
    r_a, r_b = oracle.qgemm_bwd(g, a, b, 0.25, 0.5)
    gu.assert_close(d_a, r_a, "d_a_hat")
    gu.assert_close(d_b, r_b, "d_b_hat")


def test_qgemm_bwd_wide_dynamic_range_gradient(oracle):
    # gradients spanning many binades, a few exact zeros, one large outlier
    M, N, K = 384, 160, 192
    rng = np.random.default_rng(4)
    g = (rng.standard_normal((M, N)) * np.exp(rng.uniform(-12, 2, (M, N)))).astype(np.float32)
    g[0, :7] = 0.0
    g[5, 5] = 300.0
    a = cdl_inputs.draw_indices((M, K), 0, 15, seed=8)
    b = cdl_inputs.draw_indices((N, K), -7, 7, seed=9)
    d_a, d_b = gu.qgemm_bwd(g, a, b, 0.25, 0.02)
    r_a, r_b = oracle.qgemm_bwd(g, a, b, 0.25, 0.02)
    gu.assert_close(d_a, r_a, "d_a_hat")
    gu.assert_close(d_b, r_b, "d_b_hat")


def test_qgemm_bwd_single_output_and_zero_gradient(oracle):
    M, N, K = 200, 72, 112
    a = cdl_inputs.draw_indices((M, K), 0, 15, seed=3)
    b = cdl_inputs.draw_indices((N, K), -7, 7, seed=4)
    g = np.random.default_rng(1).standard_normal((M, N)).astype(np.float32)
    both = gu.qgemm_bwd(g, a, b, 0.5, 0.125)
    only_a = gu.qgemm_bwd(g, a, b, 0.5, 0.125, want_db=False)
    only_b = gu.qgemm_bwd(g, a, b, 0.5, 0.125, want_da=False)
    assert only_a[1] is None and only_b[0] is None
    assert np.array_equal(both[0], only_a[0]) and np.array_equal(both[1], only_b[1])
    z = gu.qgemm_bwd(np.zeros((M, N), np.float32), a, b, 0.5, 0.125)
    assert not z[0].any() and not z[1].any()


def test_workload_1_layer_step_end_to_end(oracle):
    """Quantize W and X, forward product, backward products, quantizer backward: the whole chain on workload 1."""
    wl = cdl_inputs.workload(1)
    W, X, G = cdl_inputs.draw_w(wl), cdl_inputs.draw_x(wl), cdl_inputs.draw_g(wl)
    qw, qx = gu.Quantizer(wl.w_spec), gu.Quantizer(wl.x_spec)
    wi, _, _, _ = qw.fwd(gu.dev(W.reshape(-1)))
    xi, _, _, _ = qx.fwd(gu.dev(X.reshape(-1)))
    wi, xi = wi.reshape(W.shape), xi.reshape(X.shape)
    r_wi, _, gap_w = oracle.quantize_fwd(W, *qw.args)
    r_xi, _, gap_x = oracle.quantize_fwd(X, *qx.args)
    gu.assert_indices(wi, r_wi, gap_w, "w idx")
    gu.assert_indices(xi, r_xi, gap_x, "x idx")
    acc, y = gu.qgemm_fwd(xi, wi, wl.x_spec.delta, wl.w_spec.delta)
    r_acc, r_y = oracle.qgemm_fwd(xi, wi, wl.x_spec.delta, wl.w_spec.delta)
    assert np.array_equal(acc, r_acc)
    gu.assert_close(y, r_y, "y")
    dxh, dwh = gu.qgemm_bwd(G, xi, wi, wl.x_spec.delta, wl.w_spec.delta)
    r_dxh, r_dwh = oracle.qgemm_bwd(G, xi, wi, wl.x_spec.delta, wl.w_spec.delta)
    gu.assert_close(dxh, r_dxh, "dL/dQ(x)")
    gu.assert_close(dwh, r_dwh, "dL/dQ(w)")
    # quantizer backward fed with the GPU's own fp32 GEMM gradients, oracle fed the same fp32 values
    dx, ddx, dax = qx.bwd(gu.dev(X.reshape(-1)), gu.dev(dxh.reshape(-1)))
    dw, ddw, daw = qw.bwd(gu.dev(W.reshape(-1)), gu.dev(dwh.reshape(-1)))
    rx = oracle.quantize_bwd(X, dxh, *qx.args)
    rw = oracle.quantize_bwd(W, dwh, *qw.args)
    gu.assert_close(dx, rx["dtheta"], "dX")
    gu.assert_close(dw, rw["dtheta"], "dW")
    gu.assert_close([ddx, ddw], [rx["d_delta"], rw["d_delta"]], "d_delta")
    gu.assert_close([dax, daw], [rx["d_alpha"], rw["d_alpha"]], "d_alpha")


def _sweep_shapes():
    """Forty seeded shapes: sizes either side of what switches a code path (contractions of 32 / 33 for the
    direct kernel, multiples of 4, 16, 64 and 128 plus one, 32-row and 384-column tile edges, one to five
    K-tiles), mixed with sizes drawn at random."""
    rng = np.random.default_rng(20250109)
    pool_m = [1, 31, 32, 33, 63, 65, 127, 129, 255, 257, 383, 385, 700]
    pool_n = [1, 15, 16, 17, 31, 32, 33, 64, 127, 128, 129, 255, 257, 385, 513]
    pool_k = [1, 3, 4, 15, 16, 17, 63, 64, 65, 127, 128, 129, 383, 384, 385, 640]
    shapes = []
    for i in range(40):
        if i % 2 == 0:
            shapes.append((int(rng.choice(pool_m)), int(rng.choice(pool_n)), int(rng.choice(pool_k))))
        else:
            shapes.append((int(rng.integers(1, 600)), int(rng.integers(1, 600)), int(rng.integers(1, 600))))
    return shapes


@pytest.mark.parametrize("M,N,K", _sweep_shapes())
def test_qgemm_all_three_products_on_seeded_random_shapes(oracle, M, N, K):
    """Every product of one layer on the same operands; the scale of the gradient varies over twelve orders of
    magnitude from case to case (the limb count and the scale are chosen on the device from max|g|)."""
    rng = np.random.default_rng(M * 1000003 + N * 1009 + K)
    lo_a, hi_a = (0, 15) if (M + K) % 3 else (-128, 127)
    lo_b, hi_b = (-7, 7) if (N + K) % 2 else (-128, 127)
    a = cdl_inputs.draw_indices((M, K), lo_a, hi_a, seed=M + 11 * K)
    b = cdl_inputs.draw_indices((N, K), lo_b, hi_b, seed=N + 13 * K)
    g = (rng.standard_normal((M, N)) * 10.0 ** int(rng.integers(-6, 7))).astype(np.float32)
    da, db = float(np.float32(0.56419)), float(np.float32(0.016623))
    acc, y = gu.qgemm_fwd(a, b, da, db)
    r_acc, r_y = oracle.qgemm_fwd(a, b, da, db)
    assert np.array_equal(acc, r_acc), "int32 accumulators differ at %d places" % int((acc != r_acc).sum())
    gu.assert_close(y, r_y, "y")
    d_a, d_b = gu.qgemm_bwd(g, a, b, da, db)
    r_a, r_b = oracle.qgemm_bwd(g, a, b, da, db)
    gu.assert_close(d_a, r_a, "d_a_hat")
    gu.assert_close(d_b, r_b, "d_b_hat")


def test_qgemm_bwd_leaves_the_limb_counts_in_the_workspace():
    """The header documents two diagnostic words at the start of the workspace: the limb counts (3..6) the device
    chose; a gradient a million times larger cannot need fewer, coarser indices cannot need more."""
    import paper_2501_09849_amd as cdl
    torch = gu.torch_mod()
    M, N, K = 640, 256, 384
    rng = np.random.default_rng(3)
    g = rng.standard_normal((M, N)).astype(np.float32)
    a_d = gu.dev(cdl_inputs.draw_indices((M, K), -127, 127, seed=1))
    b_d = gu.dev(cdl_inputs.draw_indices((N, K), -127, 127, seed=2))
    da, db = gu.empty((M, K), torch.float32), gu.empty((N, K), torch.float32)
    ws = gu.workspace(cdl.qgemm_bwd_workspace_bytes(M, N, K))

    def limbs(gh, ad, bd):
        cdl.cdl_qgemm_bwd(gu.dev(gh), ad, bd, M, N, K, 0.15, 0.15, da, db, ws)
        torch.cuda.synchronize()
        return ws[:8].view(torch.int32).cpu().tolist()

    base = limbs(g, a_d, b_d)
    assert all(3 <= v <= 6 for v in base), base
    big = limbs(g * np.float32(2.0 ** 20), a_d, b_d)          # the absolute error bound is fixed: a larger g needs more digits
    assert all(3 <= v <= 6 for v in big) and all(v >= w for v, w in zip(big, base)), (big, base)
    small = limbs(g, gu.dev(cdl_inputs.draw_indices((M, K), 0, 3, seed=1)), gu.dev(cdl_inputs.draw_indices((N, K), -1, 1, seed=2)))
    assert all(s <= v for s, v in zip(small, base)), (small, base)


def _limb_diagnostics(ws):
    torch = gu.torch_mod()
    head = ws[:48].cpu().numpy().tobytes()
    limbs = np.frombuffer(head[:8], dtype=np.int32).tolist()
    bounds = np.frombuffer(head[32:48], dtype=np.float64).tolist()
    return limbs, bounds


@pytest.mark.parametrize("M,N,K,lo_a,hi_a,lo_b,hi_b,scale", [
    (640, 256, 384, -127, 127, -127, 127, 1.0), (3000, 96, 200, 0, 15, -7, 7, 1.0), (20000, 48, 130, 0, 15, -7, 7, 37.0),
    (512, 2048, 256, -128, 127, -128, 127, 1e-3)])
def test_limb_count_meets_the_worst_case_bound(oracle, M, N, K, lo_a, hi_a, lo_b, hi_b, scale):
    """The bound the library reports for the rounding of g - step * sigma * 2^-8L * max over output columns of the sum
    of |index| over the contraction - recomputed on the host from the operands and the limb counts, and at most
    9e-7 (so that, whatever g looks like, the limbs cost less than the absolute tolerance)."""
    import paper_2501_09849_amd as cdl
    torch = gu.torch_mod()
    rng = np.random.default_rng(M + N)
    a = cdl_inputs.draw_indices((M, K), lo_a, hi_a, seed=M)
    b = cdl_inputs.draw_indices((N, K), lo_b, hi_b, seed=N)
    g = (rng.standard_normal((M, N)) * scale).astype(np.float32)
    da, db = float(np.float32(0.56419)), float(np.float32(0.016623))
    d_a, d_b = gu.empty((M, K), torch.float32), gu.empty((N, K), torch.float32)
    ws = gu.workspace(cdl.qgemm_bwd_workspace_bytes(M, N, K))
    cdl.cdl_qgemm_bwd(gu.dev(g), gu.dev(a), gu.dev(b), M, N, K, da, db, d_a, d_b, ws)
    torch.cuda.synchronize()
    (la, lb), (bound_a, bound_b) = _limb_diagnostics(ws)
    sigma = 2.0 ** np.frexp(np.float32(np.abs(g).max()) * np.float32(1.01))[1]
    want_a = db * sigma * 2.0 ** (-8 * la) * np.abs(b.astype(np.int64)).sum(axis=0).max()     # d_a_hat contracts over n with b_idx
    want_b = da * sigma * 2.0 ** (-8 * lb) * np.abs(a.astype(np.int64)).sum(axis=0).max()
    if N > 32:      # (shorter contractions form d_a_hat directly in double)
        assert bound_a == pytest.approx(want_a, rel=1e-12) and bound_a <= 9e-7
        assert la == 3 or db * sigma * 2.0 ** (-8 * (la - 1)) * np.abs(b.astype(np.int64)).sum(axis=0).max() > 9e-7   # and no limb too many
    assert bound_b == pytest.approx(want_b, rel=1e-12) and bound_b <= 9e-7
    assert lb == 3 or da * sigma * 2.0 ** (-8 * (lb - 1)) * np.abs(a.astype(np.int64)).sum(axis=0).max() > 9e-7
    r_a, r_b = oracle.qgemm_bwd(g, a, b, da, db)
    gu.assert_close(d_a.cpu().numpy(), r_a, "d_a_hat")
    gu.assert_close(d_b.cpu().numpy(), r_b, "d_b_hat")
    # the error actually made stays under the bound (plus the fp32 rounding of the result)
    assert np.max(np.abs(d_b.cpu().numpy() - r_b) - 6e-8 * np.abs(r_b)) <= bound_b
    if N > 32:
        assert np.max(np.abs(d_a.cpu().numpy() - r_a) - 6e-8 * np.abs(r_a)) <= bound_a


@pytest.mark.parametrize("limbs_if_statistical", [3])
def test_coherent_rounding_of_a_two_valued_gradient(oracle, limbs_if_statistical):
    """The case a statistical choice of the limb count gets wrong: indices of one sign, a gradient of two values whose
    roundings to three limbs err in the same direction, and outputs that nearly cancel - every entry's rounding
    error then adds up instead of averaging out, and only the relative part of the tolerance could hide it, which a
    result near zero does not have.  Three limbs would leave an error of about half a unit per entry times the sum of
    the indices; the library's bound makes it choose more, and the result meets the stated tolerance."""
    import paper_2501_09849_amd as cdl
    torch = gu.torch_mod()
    M, N, K = 4096, 64, 256
    rng = np.random.default_rng(0)
    a = rng.integers(8, 16, (M, K)).astype(np.int8)            # all positive
    b = rng.integers(1, 8, (N, K)).astype(np.int8)
    unit = 2.0 ** -23                                           # three limbs on sigma = 1 resolve 2^-23
    v_plus = np.float32((3_000_000 + 0.49) * unit)              # rounds down by 0.49 units
    v_minus = np.float32(-(3_000_000 + 0.51) * unit)            # rounds down (away from zero) by 0.49 units
    assert abs(float(v_plus)) < 0.5 and abs(float(v_minus)) < 0.5
    g = np.where(rng.random((M, N)) < 0.5, v_plus, v_minus).astype(np.float32)
    g[0, 0] = np.float32(0.99)                                  # fixes sigma = 1
    da, db = float(np.float32(0.25)), float(np.float32(0.02))
    d_a, d_b = gu.empty((M, K), torch.float32), gu.empty((N, K), torch.float32)
    ws = gu.workspace(cdl.qgemm_bwd_workspace_bytes(M, N, K))
    cdl.cdl_qgemm_bwd(gu.dev(g), gu.dev(a), gu.dev(b), M, N, K, da, db, d_a, d_b, ws)
    torch.cuda.synchronize()
    (la, lb), (bound_a, bound_b) = _limb_diagnostics(ws)
    # what three limbs would have cost on d_b_hat: 0.49 units per entry, all in one direction
    coherent = da * 0.49 * unit * a.astype(np.int64).sum(axis=0).min()
    assert coherent > 3e-6 and lb > limbs_if_statistical and bound_b <= 9e-7
    r_a, r_b = oracle.qgemm_bwd(g, a, b, da, db)
    assert np.median(np.abs(r_b)) < 0.2 * da * float(v_plus) * a.astype(np.int64).sum(axis=0).mean()   # the outputs do cancel
    gu.assert_close(d_a.cpu().numpy(), r_a, "d_a_hat")
    gu.assert_close(d_b.cpu().numpy(), r_b, "d_b_hat")

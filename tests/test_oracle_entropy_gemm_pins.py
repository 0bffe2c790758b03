"""Pins of the CPU oracle's marginal PMF / entropy and of its index GEMMs."""
import math

import numpy as np
import pytest

import cdl_inputs


# ---------------------------------------------------------------- marginal PMF and entropy (Sec. IV-C)

@pytest.mark.parametrize("lo,L", [(-7, 15), (0, 16), (-15, 31), (-127, 255)])
def test_marginal_is_a_distribution_and_entropy_is_bounded(oracle, lo, L):
    rng = np.random.default_rng(10)
    delta = 0.05
    theta = rng.normal(0, 3 * delta, 5000).astype(np.float32)
    for kappa in (0.01, 1.0, 4.0, 30.0):
        marg, H = oracle.marginal_entropy(theta, lo, L, delta, kappa / delta ** 2)
        assert marg.sum() == pytest.approx(1.0, abs=1e-12)
        assert np.all(marg >= 0)
        assert 0.0 <= H <= math.log2(L) + 1e-12
        # entropy of the returned vector with numpy's log2 (library routine for the definition in Sec. II-A)
        nz = marg[marg > 0]
        assert H == pytest.approx(float(-(nz * np.log2(nz)).sum()), rel=1e-12)


def test_marginal_is_the_mean_of_the_elementwise_cpmfs(oracle):
    lo, L, delta, alpha = -4, 8, 0.1, 300.0
    theta = np.array([-0.31, -0.1, 0.0, 0.04, 0.26, 0.9], np.float32)
    want = np.mean([oracle.cpmf(float(t), lo, L, float(np.float32(delta)), alpha)[0] for t in theta], axis=0)
    marg, _ = oracle.marginal_entropy(theta, lo, L, delta, alpha)
    np.testing.assert_allclose(marg, want, rtol=1e-13, atol=1e-300)


def test_entropy_limits_in_the_sharpness(oracle):
    rng = np.random.default_rng(11)
    lo, L, delta = -7, 15, 0.02
    theta = rng.normal(0, 0.05, 20000).astype(np.float32)
    # alpha -> 0: every CPMF is uniform, so is the marginal, H = log2 L exactly
    marg, H = oracle.marginal_entropy(theta, lo, L, delta, 1e-9)
    np.testing.assert_allclose(marg, 1.0 / L, rtol=1e-6)
    assert H == pytest.approx(math.log2(L), abs=1e-9)
    # alpha -> infinity: one-hot CPMFs, marginal = normalised histogram of the hard indices
    alpha = 1e8 / delta ** 2
    idx, _, gap = oracle.quantize_fwd(theta, lo, L, delta, alpha)
    assert gap.min() > 40.0
    hist = np.bincount(idx - lo, minlength=L) / theta.size
    marg, H = oracle.marginal_entropy(theta, lo, L, delta, alpha)
    np.testing.assert_allclose(marg, hist, atol=1e-12)
    nz = hist[hist > 0]
    assert H == pytest.approx(float(-(nz * np.log2(nz)).sum()), abs=1e-9)
    # a constant tensor sitting on a level: nothing to code
    marg, H = oracle.marginal_entropy(np.full(100, 3 * np.float32(delta), np.float32), lo, L, delta, alpha)
    assert H == pytest.approx(0.0, abs=1e-12) and marg[3 - lo] == pytest.approx(1.0)


def test_entropy_of_two_equal_masses_is_one_bit(oracle):
    # half the tensor on level 1, half on level 5, very sharp quantizer
    theta = np.array([0.25] * 8 + [1.25] * 8, np.float32)
    marg, H = oracle.marginal_entropy(theta, 0, 16, 0.25, 1e6)
    assert H == pytest.approx(1.0, abs=1e-12)
    assert marg[1] == pytest.approx(0.5) and marg[5] == pytest.approx(0.5)


# ---------------------------------------------------------------- index GEMM forward

def test_qgemm_fwd_matches_brute_force_integers(oracle):
    a = cdl_inputs.draw_indices((5, 7), -7, 7, seed=1)
    b = cdl_inputs.draw_indices((3, 7), 0, 15, seed=2)
    acc, y = oracle.qgemm_fwd(a, b, 0.25, 0.02)
    for m in range(5):
        for n in range(3):
            s = sum(int(a[m, k]) * int(b[n, k]) for k in range(7))
            assert acc[m, n] == s
            assert y[m, n] == pytest.approx(float(np.float32(0.25)) * float(np.float32(0.02)) * s, rel=1e-15)


def test_qgemm_fwd_matches_numpy_and_dequantised_product(oracle):
    a = cdl_inputs.draw_indices((37, 129), -127, 127, seed=3)
    b = cdl_inputs.draw_indices((11, 129), -127, 127, seed=4)
    da, db = float(np.float32(0.15)), float(np.float32(0.0028))
    acc, y = oracle.qgemm_fwd(a, b, da, db)
    ref = a.astype(np.int64) @ b.astype(np.int64).T
    assert np.array_equal(acc.astype(np.int64), ref)
    deq = (a.astype(np.float64) * da) @ (b.astype(np.float64) * db).T
    np.testing.assert_allclose(y, deq, rtol=1e-12, atol=1e-15)


def test_qgemm_on_the_unsigned_8_bit_alphabet(oracle):
    """The paper's unsigned b-bit activation alphabet {0, ..., 2^b - 1} (eq. repo_alphabet) with b = 8, the width it
    keeps for the first and last layers (Sec. V-B): indices up to 255 on either operand.  Brute force with Python
    integers on a tiny case, numpy int64 / float64 on a larger one, for the forward product and both gradients."""
    rng = np.random.default_rng(77)
    a = rng.integers(0, 256, (4, 9)).astype(np.int16)
    b = rng.integers(0, 256, (3, 9)).astype(np.int16)
    a[0, :] = 255
    b[0, :] = 255
    acc, y = oracle.qgemm_fwd(a, b, 0.5, 0.25)
    for m in range(4):
        for n in range(3):
            s = sum(int(a[m, k]) * int(b[n, k]) for k in range(9))
            assert acc[m, n] == s and y[m, n] == pytest.approx(0.125 * s, rel=1e-15)
    assert acc[0, 0] == 9 * 255 * 255
    M, N, K = 33, 12, 257
    a = rng.integers(0, 256, (M, K)).astype(np.int16)
    b = rng.integers(-128, 128, (N, K)).astype(np.int16)
    g = rng.normal(0, 1, (M, N)).astype(np.float32)
    da, db = float(np.float32(0.0731)), float(np.float32(0.011))
    acc, y = oracle.qgemm_fwd(a, b, da, db)
    assert np.array_equal(acc.astype(np.int64), a.astype(np.int64) @ b.astype(np.int64).T)
    d_a, d_b = oracle.qgemm_bwd(g, a, b, da, db)
    g64 = g.astype(np.float64)
    # (sums of a few hundred terms of size 10 in two different orders: 1e-12 absolute)
    np.testing.assert_allclose(d_a, g64 @ (b.astype(np.float64) * db), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(d_b, g64.T @ (a.astype(np.float64) * da), rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- index GEMM backward

def test_qgemm_bwd_matches_numpy_and_directional_derivative(oracle):
    rng = np.random.default_rng(12)
    M, N, K = 19, 6, 23
    a = cdl_inputs.draw_indices((M, K), 0, 15, seed=5)
    b = cdl_inputs.draw_indices((N, K), -7, 7, seed=6)
    g = rng.normal(0, 1, (M, N)).astype(np.float32)
    da, db = float(np.float32(0.56)), float(np.float32(0.0166))
    d_a, d_b = oracle.qgemm_bwd(g, a, b, da, db)
    g64 = g.astype(np.float64)
    np.testing.assert_allclose(d_a, g64 @ (b.astype(np.float64) * db), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(d_b, g64.T @ (a.astype(np.float64) * da), rtol=1e-13, atol=1e-15)
    # the loss <g, Ahat Bhat^T> is bilinear, so a one-sided difference in a direction is exact up to rounding
    Ah, Bh = a.astype(np.float64) * da, b.astype(np.float64) * db
    loss = lambda A_, B_: float(np.sum(g64 * (A_ @ B_.T)))
    dA_dir, dB_dir = rng.normal(size=Ah.shape), rng.normal(size=Bh.shape)
    assert loss(Ah + dA_dir, Bh) - loss(Ah, Bh) == pytest.approx(float(np.sum(d_a * dA_dir)), rel=1e-10)
    assert loss(Ah, Bh + dB_dir) - loss(Ah, Bh) == pytest.approx(float(np.sum(d_b * dB_dir)), rel=1e-10)


# ---------------------------------------------------------------- the whole tiny layer, end to end

def test_layer_chain_matches_finite_differences_when_the_layer_runs_on_soft_values(oracle):
    """R-CDL (Sec. IV-F) is differentiable end to end: L = <G, Q_d(X) Q_d(W)^T>.

    Its exact gradient is quantize_bwd applied to the GEMM backward of the soft
    operands; this pins the composition order of the two backward steps
    (which operand each GEMM gradient belongs to, which step size scales it).
    """
    wl = cdl_inputs.workload(1)
    M, N, K = 6, 5, 16
    W = cdl_inputs.draw_w(wl)[:N, :K].copy()
    X = cdl_inputs.draw_x(wl)[:M, :K].copy()
    G = cdl_inputs.draw_g(wl)[:M, :N].astype(np.float64)
    ws, xs = wl.w_spec, wl.x_spec
    # soften both quantizers so that every entry has a visible gradient
    ws, xs = ws.with_kappa(1.5), xs.with_kappa(1.5)

    def soft_mat(T, spec, delta=None, alpha=None):
        d = spec.delta if delta is None else delta
        a = spec.alpha if alpha is None else alpha
        return np.array([[oracle.element(float(t), spec.lo, spec.n_levels, d, a)["soft"] for t in row] for row in T])

    def loss(Wm=W, Xm=X, dw=None, dx=None):
        return float(np.sum(G * (soft_mat(Xm, xs, dx) @ soft_mat(Wm, ws, dw).T)))

    Xs, Ws = soft_mat(X, xs), soft_mat(W, ws)
    dXhat, dWhat = G @ Ws, G.T @ Xs                    # gradients wrt the (soft-)quantized operands
    bx = oracle.quantize_bwd(X, dXhat.astype(np.float32), xs.lo, xs.n_levels, xs.delta, xs.alpha)
    bw = oracle.quantize_bwd(W, dWhat.astype(np.float32), ws.lo, ws.n_levels, ws.delta, ws.alpha)
    # the fp32 rounding of dXhat/dWhat on the way into quantize_bwd limits agreement to ~1e-7
    for (m, k) in [(0, 0), (3, 7), (5, 15)]:
        Xp, Xm_ = X.astype(np.float64).copy(), X.astype(np.float64).copy()
        h = 1e-6 * xs.delta
        Xp[m, k] += h; Xm_[m, k] -= h
        assert bx["dtheta"].reshape(M, K)[m, k] == pytest.approx((loss(Xm=Xp) - loss(Xm=Xm_)) / (2 * h), rel=1e-5, abs=1e-7)
    for (n, k) in [(0, 1), (4, 9)]:
        Wp, Wm_ = W.astype(np.float64).copy(), W.astype(np.float64).copy()
        h = 1e-6 * ws.delta
        Wp[n, k] += h; Wm_[n, k] -= h
        assert bw["dtheta"].reshape(N, K)[n, k] == pytest.approx((loss(Wm=Wp) - loss(Wm=Wm_)) / (2 * h), rel=1e-5, abs=1e-7)
    hx, hw = 1e-6 * xs.delta, 1e-6 * ws.delta
    assert bx["d_delta"] == pytest.approx((loss(dx=xs.delta + hx) - loss(dx=xs.delta - hx)) / (2 * hx), rel=1e-5)
    assert bw["d_delta"] == pytest.approx((loss(dw=ws.delta + hw) - loss(dw=ws.delta - hw)) / (2 * hw), rel=1e-5)

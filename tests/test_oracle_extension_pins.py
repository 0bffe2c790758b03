"""Pins for the oracle's extensions of the path: the truncated (top-k) CPMF, the probabilistic draw Q_p,
and the gradient of the entropy term.  Each is checked against something other than the oracle's own
formula: brute force / a library routine, finite differences of a quantity built from the plain CPMF,
invariants and limits.
"""
import math

import numpy as np
import pytest


def _cpmf_np(theta, lo, n_levels, delta, alpha):
    """Plain numpy softmax of -alpha (theta - i delta)^2 (eq. CPMF): an independent restatement for the pins."""
    i = np.arange(lo, lo + n_levels, dtype=np.float64)
    s = -alpha * (theta - i * delta) ** 2
    w = np.exp(s - s.max())
    return w / w.sum()


# ------------------------------------------------------------------ truncated CPMF (Sec. V-B, top five values)

@pytest.mark.parametrize("lo,n_levels", [(0, 16), (-7, 15), (-127, 255), (-4, 8)])
@pytest.mark.parametrize("top_k", [1, 3, 5])
def test_top_k_keeps_the_k_most_probable_levels_renormalised(oracle, lo, n_levels, top_k):
    rng = np.random.default_rng(abs(lo) * 31 + n_levels + top_k)
    delta = 0.1
    for alpha in (0.5, 30.0, 400.0):
        for theta in np.concatenate([rng.uniform((lo - 2) * delta, (lo + n_levels + 1) * delta, 40), [0.0, 0.05, -0.05]]):
            full = _cpmf_np(theta, lo, n_levels, delta, alpha)
            P, mode, _ = oracle.cpmf(theta, lo, n_levels, delta, alpha, top_k=top_k)
            # brute force: sort by score (descending; the exponential would merge scores one rounding apart),
            # equal scores by lower index
            score = -alpha * (theta - np.arange(lo, lo + n_levels, dtype=np.float64) * delta) ** 2
            order = sorted(range(n_levels), key=lambda k: (-score[k], k))[:top_k]
            ref = np.zeros(n_levels)
            ref[order] = full[order] / full[order].sum()
            assert np.count_nonzero(P) <= top_k
            np.testing.assert_allclose(P, ref, rtol=1e-12, atol=1e-300)
            assert abs(P.sum() - 1.0) < 1e-14
            assert mode == lo + int(np.argmax(full))     # the mode is always kept


def test_top_k_is_the_k_nearest_levels_and_slides_at_the_ends(oracle):
    lo, n, d = 0, 16, 0.25
    P, _, _ = oracle.cpmf(1.30, lo, n, d, 2.0, top_k=5)          # nearest level 5 (1.25): keeps 3..7
    assert list(np.nonzero(P)[0]) == [3, 4, 5, 6, 7]
    P, _, _ = oracle.cpmf(0.05, lo, n, d, 2.0, top_k=5)          # at the lower end the window is 0..4
    assert list(np.nonzero(P)[0]) == [0, 1, 2, 3, 4]
    P, _, _ = oracle.cpmf(9.0, lo, n, d, 2.0, top_k=5)           # far above the range: 11..15
    assert list(np.nonzero(P)[0]) == [11, 12, 13, 14, 15]
    P, _, _ = oracle.cpmf(1.375, lo, n, d, 2.0, top_k=2)         # exact midpoint of 5 and 6: both, then 4 before 7
    assert list(np.nonzero(P)[0]) == [5, 6]
    P, _, _ = oracle.cpmf(1.375, lo, n, d, 2.0, top_k=3)
    assert list(np.nonzero(P)[0]) == [4, 5, 6]


def test_top_k_equals_the_full_cpmf_when_it_covers_the_set_or_the_tails_are_negligible(oracle):
    P5, _, _ = oracle.cpmf(0.11, -2, 5, 0.1, 3.0, top_k=5)
    P0, _, _ = oracle.cpmf(0.11, -2, 5, 0.1, 3.0)
    np.testing.assert_array_equal(P5, P0)
    # kappa = 4: levels three or more steps away carry < exp(-4*6) of the mass
    P5, _, _ = oracle.cpmf(0.537, -127, 255, 0.1, 400.0, top_k=5)
    P0, _, _ = oracle.cpmf(0.537, -127, 255, 0.1, 400.0)
    assert np.abs(P5 - P0).max() < 1e-9


def test_top_k_lemma_1_matches_finite_differences_of_the_truncated_soft_value(oracle):
    """The analytic derivatives hold for the truncated CPMF wherever the kept set is locally constant."""
    lo, n, d, a, k = 0, 16, 0.25, 3.0, 5          # kappa = 0.19: the truncation changes the values a lot
    for theta in (0.31, 1.07, 2.2, 3.6, 0.02, 3.9):
        def soft(th, dd, aa):
            P, _, _ = oracle.cpmf(th, lo, n, dd, aa, top_k=k)
            return float(np.sum(P * np.arange(lo, lo + n) * dd))
        el = oracle.element(theta, lo, n, d, a, top_k=k)
        full = oracle.element(theta, lo, n, d, a)
        assert abs(el["soft"] - full["soft"]) > 1e-3            # the case really differs from the full CPMF
        h = 1e-6
        assert el["dtheta"] == pytest.approx((soft(theta + h, d, a) - soft(theta - h, d, a)) / (2 * h), rel=1e-6, abs=1e-9)
        assert el["ddelta"] == pytest.approx((soft(theta, d + h, a) - soft(theta, d - h, a)) / (2 * h), rel=1e-6, abs=1e-9)
        assert el["dalpha"] == pytest.approx((soft(theta, d, a + h) - soft(theta, d, a - h)) / (2 * h), rel=1e-6, abs=1e-9)


def test_top_k_tensor_routines_agree_with_the_single_element_routine(oracle):
    rng = np.random.default_rng(5)
    th = np.abs(rng.normal(0, 1, 300)).astype(np.float32)
    g = rng.normal(0, 1, 300).astype(np.float32)
    a = (0, 16, 0.25, 1.5)
    idx, soft, _ = oracle.quantize_fwd(th, *a, top_k=5)
    marg, H = oracle.marginal_entropy(th, *a, top_k=5)
    bw = oracle.quantize_bwd(th, g, *a, top_k=5)
    els = [oracle.element(float(t), *[float(np.float32(x)) if i >= 2 else x for i, x in enumerate(a)], top_k=5) for t in th]
    np.testing.assert_array_equal(idx, [e["idx"] for e in els])
    np.testing.assert_allclose(soft, [e["soft"] for e in els], rtol=1e-13)
    np.testing.assert_allclose(bw["dtheta"], [gg * e["dtheta"] for gg, e in zip(g.astype(np.float64), els)], rtol=1e-12, atol=1e-300)
    Ps = np.array([oracle.cpmf(float(t), 0, 16, 0.25, 1.5, top_k=5)[0] for t in th])
    np.testing.assert_allclose(marg, Ps.mean(axis=0), rtol=1e-12, atol=1e-18)
    assert H == pytest.approx(-np.sum(np.where(marg > 0, marg * np.log2(np.maximum(marg, 1e-300)), 0)), rel=1e-12)


# ------------------------------------------------------------------ the probabilistic quantizer Q_p (eq. Qprob)

@pytest.mark.parametrize("lo,n_levels,delta,alpha", [(0, 16, 0.25, 8.0), (-7, 15, 0.02, 2500.0), (-127, 255, 0.15, 3.0), (-4, 8, 0.1, 100.0)])
def test_draw_is_numpys_inverse_cdf(oracle, lo, n_levels, delta, alpha):
    """Library cross-check: searchsorted on the cumulative sums of the (independently restated) CPMF."""
    rng = np.random.default_rng(n_levels)
    d32, a32 = float(np.float32(delta)), float(np.float32(alpha))
    th = rng.uniform((lo - 1) * delta, (lo + n_levels) * delta, 4000).astype(np.float32)
    u = rng.random(4000, dtype=np.float32)
    idx, margin = oracle.quantize_draw(th, u, lo, n_levels, delta, alpha)
    for e in range(0, 4000, 7):
        cdf = np.cumsum(_cpmf_np(float(th[e]), lo, n_levels, d32, a32))
        ref = lo + min(int(np.searchsorted(cdf, float(u[e]), side="right")), n_levels - 1)
        if margin[e] > 1e-12:
            assert idx[e] == ref, (e, idx[e], ref, margin[e])


def test_draw_frequencies_are_the_cpmf(oracle):
    """With u on a regular grid of N points every level is drawn round(N * P) times up to one."""
    lo, n, d, a = -4, 8, 0.1, 150.0
    N = 100000
    u = ((np.arange(N) + 0.5) / N).astype(np.float32)
    for theta in (0.03, -0.17, 0.249, 0.5):
        th = np.full(N, theta, dtype=np.float32)
        idx, _ = oracle.quantize_draw(th, u, lo, n, d, a)
        P, _, _ = oracle.cpmf(float(np.float32(theta)), lo, n, float(np.float32(d)), float(np.float32(a)))
        counts = np.bincount(idx - lo, minlength=n)
        assert np.all(np.abs(counts - N * P) <= 2.0), (counts, N * P)
        assert np.all(np.diff(idx) >= 0)            # monotone in u


def test_draw_tends_to_the_nearest_level_as_sharpness_grows(oracle):
    """Remark after eq. Qprob: Q_p equals the uniformly quantized value with probability -> 1."""
    rng = np.random.default_rng(9)
    lo, n, d = -7, 15, 0.02
    th = rng.normal(0, 0.05, 20000).astype(np.float32)
    u = rng.random(20000, dtype=np.float32)
    mode, _, _ = oracle.quantize_fwd(th, lo, n, d, 1e4 / d ** 2)
    frac = []
    for kappa in (1.0, 10.0, 100.0, 1e4):
        idx, _ = oracle.quantize_draw(th, u, lo, n, d, kappa / d ** 2)
        frac.append(np.mean(idx == mode))
    assert frac[0] < frac[1] < frac[2] <= frac[3] and frac[3] > 0.999
    # u = 0 picks the lowest level with positive probability, u just below 1 the highest
    idx, _ = oracle.quantize_draw(np.float32([0.011]), np.float32([0.0]), lo, n, d, 1.0 / d ** 2)
    assert idx[0] < 0
    idx, _ = oracle.quantize_draw(np.float32([0.011]), np.float32([1.0 - 2.0 ** -24]), lo, n, d, 1.0 / d ** 2)
    assert idx[0] > 1


def test_draw_with_truncated_cpmf_stays_inside_the_kept_levels(oracle):
    rng = np.random.default_rng(2)
    th = np.abs(rng.normal(0, 1, 5000)).astype(np.float32)
    u = rng.random(5000, dtype=np.float32)
    idx, _ = oracle.quantize_draw(th, u, 0, 16, 0.25, 0.8, top_k=5)
    near = np.clip(np.rint(th / np.float32(0.25)), 0, 15)
    win_lo = np.clip(near - 2, 0, 11)
    assert np.all((idx >= win_lo) & (idx <= win_lo + 4))
    full, _ = oracle.quantize_draw(th, u, 0, 16, 0.25, 0.8)
    assert np.any(full != idx)                         # kappa = 0.05: the full CPMF reaches further


# ------------------------------------------------------------------ gradient of the entropy term (Sec. IV-D)

def _entropy_np(th, lo, n_levels, delta, alpha):
    m = np.mean([_cpmf_np(float(t), lo, n_levels, delta, alpha) for t in th], axis=0)
    return -float(np.sum(np.where(m > 0, m * np.log2(np.maximum(m, 1e-300)), 0.0))), m


@pytest.mark.parametrize("lo,n_levels,delta,alpha", [(-4, 8, 0.1, 100.0), (0, 16, 0.25, 20.0), (-7, 15, 0.02, 6000.0), (-15, 31, 0.004, 500.0)])
def test_entropy_gradient_matches_finite_differences(oracle, lo, n_levels, delta, alpha):
    rng = np.random.default_rng(n_levels)
    d32, a32 = float(np.float32(delta)), float(np.float32(alpha))
    th = (rng.normal(0, 2.5 * delta, 24)).astype(np.float32)
    if lo == 0:
        th = np.abs(th)
    H, m = _entropy_np(th, lo, n_levels, d32, a32)
    r = oracle.entropy_bwd(th, m, lo, n_levels, delta, alpha)
    # wrt every entry
    for e in range(th.size):
        h = 1e-6 * delta
        tp, tm = th.astype(np.float64).copy(), th.astype(np.float64).copy()
        tp[e] += h
        tm[e] -= h
        fd = (_entropy_np(tp, lo, n_levels, d32, a32)[0] - _entropy_np(tm, lo, n_levels, d32, a32)[0]) / (2 * h)
        assert r["dtheta"][e] == pytest.approx(fd, rel=2e-5, abs=1e-7 / delta)
    h = 1e-6 * d32
    fd = (_entropy_np(th, lo, n_levels, d32 + h, a32)[0] - _entropy_np(th, lo, n_levels, d32 - h, a32)[0]) / (2 * h)
    assert r["d_delta"] == pytest.approx(fd, rel=2e-5, abs=1e-7 / delta)
    h = 1e-5 * a32
    fd = (_entropy_np(th, lo, n_levels, d32, a32 + h)[0] - _entropy_np(th, lo, n_levels, d32, a32 - h)[0]) / (2 * h)
    assert r["d_alpha"] == pytest.approx(fd, rel=2e-5, abs=1e-9 / alpha)


def test_entropy_gradient_obeys_the_scaling_identity(oracle):
    """H is unchanged under (theta, q, alpha) -> (c theta, c q, alpha / c^2), hence
    sum_e theta_e dH/dtheta_e + q dH/dq - 2 alpha dH/dalpha = 0."""
    rng = np.random.default_rng(3)
    for lo, n, d, a in ((-7, 15, 0.02, 3000.0), (0, 16, 0.25, 9.0), (-127, 255, 0.15, 40.0)):
        th = rng.normal(0, 4 * d, 200).astype(np.float32)
        m, _ = oracle.marginal_entropy(th, lo, n, d, a)
        r = oracle.entropy_bwd(th, m, lo, n, d, a)
        d32, a32 = float(np.float32(d)), float(np.float32(a))
        resid = float(np.dot(th.astype(np.float64), r["dtheta"])) + d32 * r["d_delta"] - 2 * a32 * r["d_alpha"]
        size = float(np.abs(th.astype(np.float64) * r["dtheta"]).sum()) + abs(d32 * r["d_delta"]) + abs(2 * a32 * r["d_alpha"])
        assert abs(resid) < 1e-11 * max(size, 1.0)


def test_entropy_gradient_special_cases(oracle):
    rng = np.random.default_rng(4)
    lo, n, d = -4, 8, 0.1
    th = rng.normal(0, 0.2, 50).astype(np.float32)
    # a uniform marginal has constant log: the gradient vanishes identically
    r = oracle.entropy_bwd(th, np.full(n, 1.0 / n), lo, n, d, 100.0)
    assert np.abs(r["dtheta"]).max() < 1e-12 and abs(r["d_delta"]) < 1e-10 and abs(r["d_alpha"]) < 1e-12
    # scale multiplies everything
    m, _ = oracle.marginal_entropy(th, lo, n, d, 100.0)
    r1 = oracle.entropy_bwd(th, m, lo, n, d, 100.0)
    r3 = oracle.entropy_bwd(th, m, lo, n, d, 100.0, scale=3.0)
    np.testing.assert_allclose(r3["dtheta"], 3.0 * r1["dtheta"], rtol=1e-14)
    assert r3["d_delta"] == pytest.approx(3.0 * r1["d_delta"], rel=1e-14)
    # the entries' gradients sum to zero when every entry is shifted together with the level grid... (translation by
    # one whole step permutes interior levels): moving all entries far inside a long level set by exactly one step
    # leaves H unchanged, so the directional derivative along (1, ..., 1) is not zero in general, but it is odd
    # under reflection: H(theta) = H(-theta) on a symmetric set
    lo, n = -7, 15
    m_p, _ = oracle.marginal_entropy(th, lo, n, d, 60.0)
    m_n, _ = oracle.marginal_entropy(-th, lo, n, d, 60.0)
    np.testing.assert_allclose(m_p, m_n[::-1], rtol=1e-12)
    g_p = oracle.entropy_bwd(th, m_p, lo, n, d, 60.0)
    g_n = oracle.entropy_bwd(-th, m_n, lo, n, d, 60.0)
    np.testing.assert_allclose(g_p["dtheta"], -g_n["dtheta"], rtol=1e-10, atol=1e-14)
    assert g_p["d_delta"] == pytest.approx(g_n["d_delta"], rel=1e-10)


def test_entropy_gradient_with_truncated_cpmf_matches_finite_differences(oracle):
    lo, n, d, a, k = 0, 16, 0.25, 2.0, 5
    rng = np.random.default_rng(8)
    th = np.abs(rng.normal(0, 1, 20)).astype(np.float32)
    th = th[np.abs(th / 0.25 - np.rint(th / 0.25)) < 0.45]          # stay away from the points where the kept set switches

    def H_of(tt, dd, aa):
        m = np.mean([oracle.cpmf(float(t), lo, n, dd, aa, top_k=k)[0] for t in tt], axis=0)
        return -float(np.sum(np.where(m > 0, m * np.log2(np.maximum(m, 1e-300)), 0.0))), m
    _, m = H_of(th, d, a)
    r = oracle.entropy_bwd(th, m, lo, n, d, a, top_k=k)
    for e in range(th.size):
        h = 1e-7
        tp, tm = th.astype(np.float64).copy(), th.astype(np.float64).copy()
        tp[e] += h
        tm[e] -= h
        fd = (H_of(tp, d, a)[0] - H_of(tm, d, a)[0]) / (2 * h)
        assert r["dtheta"][e] == pytest.approx(fd, rel=1e-5, abs=1e-8)
    h = 1e-7
    assert r["d_delta"] == pytest.approx((H_of(th, d + h, a)[0] - H_of(th, d - h, a)[0]) / (2 * h), rel=1e-5, abs=1e-7)
    assert r["d_alpha"] == pytest.approx((H_of(th, d, a + h)[0] - H_of(th, d, a - h)[0]) / (2 * h), rel=1e-5, abs=1e-8)


# ------------------------------------------------------------------ Huffman-coded size (Sec. V-A, eq. Nofbits)

def _huffman_total_heapq(counts):
    """Independent restatement with the standard library's heap: total code length = sum of merged weights."""
    import heapq
    h = [int(c) for c in counts if c > 0]
    if len(h) == 1:
        return h[0]
    heapq.heapify(h)
    total = 0
    while len(h) > 1:
        a, b = heapq.heappop(h), heapq.heappop(h)
        total += a + b
        heapq.heappush(h, a + b)
    return total


def test_huffman_textbook_example(oracle):
    # the classic six-symbol example (tests/golden/huffman_six_symbols.txt): frequencies 45, 13, 12, 16, 9, 5 have
    # optimal code lengths 1, 3, 3, 3, 4, 4, i.e. 224 bits
    import os
    freq, lengths, want_total = [], [], None
    for line in open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "huffman_six_symbols.txt")):
        f = line.split("#")[0].split()
        if len(f) == 2 and f[0] == "total_bits":
            want_total = int(f[1])
        elif len(f) == 2:
            freq.append(int(f[0]))
            lengths.append(int(f[1]))
    assert want_total == sum(a * b for a, b in zip(freq, lengths)) == 224
    idx = np.concatenate([np.full(f, k - 3, np.int8) for k, f in enumerate(freq)])
    counts, total, avg = oracle.huffman_bits(idx, -3, 6)
    assert list(counts) == freq and total == want_total and avg == pytest.approx(want_total / sum(freq))


def test_huffman_bounds_and_special_cases(oracle):
    rng = np.random.default_rng(0)
    for lo, n_levels in ((-7, 15), (0, 16), (-127, 255)):
        p = rng.dirichlet(np.full(n_levels, 0.3))
        idx = (rng.choice(n_levels, size=20000, p=p) + lo).astype(np.int8)
        counts, total, avg = oracle.huffman_bits(idx, lo, n_levels)
        assert counts.sum() == idx.size and np.array_equal(counts, np.bincount(idx.astype(int) - lo, minlength=n_levels))
        assert total == _huffman_total_heapq(counts)
        q = counts[counts > 0] / idx.size
        H = -np.sum(q * np.log2(q))
        assert H <= avg + 1e-12 and avg < H + 1.0          # Shannon's bounds for an optimal prefix code
    # dyadic distribution: the code meets the entropy exactly
    idx = np.concatenate([np.full(8, 0), np.full(4, 1), np.full(2, 2), np.full(1, 3), np.full(1, 4)]).astype(np.int8)
    _, total, avg = oracle.huffman_bits(idx, 0, 16)
    assert total == 8 * 1 + 4 * 2 + 2 * 3 + 4 + 4 and avg == pytest.approx(30 / 16)
    # two equally likely levels: one bit each; a single level: one bit each (reading); nothing: zero
    assert oracle.huffman_bits(np.int8([1, 2, 1, 2]), 0, 4)[1:] == (4.0, 1.0)
    assert oracle.huffman_bits(np.int8([3, 3, 3]), 0, 4)[1:] == (3.0, 1.0)
    assert oracle.huffman_bits(np.zeros(0, np.int8), 0, 4)[1:] == (0.0, 0.0)

"""Pins of the CPU oracle's quantizer against things other than itself.

Each test states what in the paper or in mathematics fixes the expected value:
closed forms (the two-level quantizer is the logistic function), invariants
(probabilities sum to one, Proposition 1, a scaling identity), limits in the
sharpness, exact rational arithmetic for the nearest level, and central finite
differences of Q_d for Lemma 1 and the alpha derivative.
"""
import math
from fractions import Fraction

import numpy as np
import pytest
from scipy.special import expit

LEVEL_SETS = [(-4, 8), (-8, 16), (-7, 15), (0, 16), (-15, 31), (0, 2), (-127, 255)]


def _fd(f, x, h):
    return (f(x + h) - f(x - h)) / (2.0 * h)


# ---------------------------------------------------------------- CPMF (eq. CPMF / eq. PMF, Sec. III-A)

@pytest.mark.parametrize("lo,L", LEVEL_SETS)
def test_cpmf_is_a_distribution(oracle, lo, L):
    rng = np.random.default_rng(1)
    for kappa in (0.01, 1.0, 4.0, 30.0, 1e4):
        delta = 0.1
        alpha = kappa / delta ** 2
        for theta in rng.uniform((lo - 2) * delta, (lo + L + 1) * delta, size=20):
            P, mode, gap = oracle.cpmf(theta, lo, L, delta, alpha)
            assert abs(P.sum() - 1.0) < 1e-14
            assert np.all(P >= 0.0) and P.max() > 0.0
            assert gap >= 0.0
            assert lo <= mode <= lo + L - 1
            assert P[mode - lo] == P.max()


def test_cpmf_matches_textbook_softmax_of_negative_scaled_squared_distance(oracle):
    # eq. PMF: the CPMF is softmax(-alpha (theta - levels)^2); scipy's softmax is the library routine
    from scipy.special import softmax
    lo, L, delta, alpha = -4, 8, 0.1, 300.0
    for theta in (-0.37, -0.05, 0.0, 0.012, 0.26, 0.31):
        P, _, _ = oracle.cpmf(theta, lo, L, delta, alpha)
        levels = delta * np.arange(lo, lo + L)
        ref = softmax(-alpha * (theta - levels) ** 2)
        np.testing.assert_allclose(P, ref, rtol=1e-12, atol=1e-300)


def test_cpmf_mirror_symmetry_on_symmetric_level_set(oracle):
    lo, L, delta, alpha = -7, 15, 0.02, 1e4
    for theta in (0.0131, -0.0777, 0.14, 0.2):
        P, _, _ = oracle.cpmf(theta, lo, L, delta, alpha)
        Pm, _, _ = oracle.cpmf(-theta, lo, L, delta, alpha)
        np.testing.assert_allclose(P, Pm[::-1], rtol=1e-12, atol=1e-300)


def test_two_level_quantizer_is_the_logistic_function(oracle):
    # levels {0, delta}: P(delta|theta) = 1/(1+exp(-alpha(theta^2-(theta-delta)^2))) = expit(alpha*delta*(2 theta - delta))
    lo, L = 0, 2
    rng = np.random.default_rng(2)
    for _ in range(50):
        delta = rng.uniform(0.05, 2.0)
        alpha = rng.uniform(0.1, 20.0) / delta ** 2
        theta = rng.uniform(-0.5 * delta, 1.5 * delta)
        z = alpha * delta * (2 * theta - delta)
        s = expit(z)
        e = oracle.element(theta, lo, L, delta, alpha)
        P, _, _ = oracle.cpmf(theta, lo, L, delta, alpha)
        assert P[1] == pytest.approx(s, rel=1e-12)
        assert e["soft"] == pytest.approx(delta * s, rel=1e-12)
        # derivatives of delta*expit(z) by the chain rule on z
        assert e["dtheta"] == pytest.approx(2 * alpha * delta ** 2 * s * (1 - s), rel=1e-10)
        assert e["ddelta"] == pytest.approx(s + 2 * alpha * delta * s * (1 - s) * (theta - delta), rel=1e-9, abs=1e-12)
        assert e["dalpha"] == pytest.approx(delta ** 2 * s * (1 - s) * (2 * theta - delta), rel=1e-9, abs=1e-14)


# ---------------------------------------------------------------- hard index = nearest level (Remark in Sec. III-A)

def _nearest_level_exact(theta: float, delta: float, lo: int, hi: int) -> int:
    """argmin_i |theta - i delta| in exact rational arithmetic, lowest index on ties."""
    t, d = Fraction(theta), Fraction(delta)
    best, best_dist = lo, None
    for i in range(lo, hi + 1):
        dist = abs(t - i * d)
        if best_dist is None or dist < best_dist:
            best, best_dist = i, dist
    return best


def test_hard_index_is_nearest_level_with_clamping(oracle):
    rng = np.random.default_rng(3)
    for lo, L in [(-4, 8), (-7, 15), (0, 16), (-127, 255), (0, 256), (130, 126)]:
        delta = float(np.float32(0.0731))
        alpha = float(np.float32(4.0 / delta ** 2))
        theta = rng.uniform((lo - 3) * delta, (lo + L + 2) * delta, size=300).astype(np.float32)
        idx, soft, gap = oracle.quantize_fwd(theta, lo, L, delta, alpha)
        for t, i, g in zip(theta, idx, gap):
            if g > 1e-9:  # away from an exact tie of the double-precision scores
                assert i == _nearest_level_exact(float(t), delta, lo, lo + L - 1)
    # far outside the range: clamps to the end levels
    idx, _, _ = oracle.quantize_fwd(np.array([-1e3, 1e3, -0.6, 5.0], np.float32), -7, 15, 0.02, 1e4)
    assert idx.tolist() == [-7, 7, -7, 7]


def test_unsigned_8_bit_alphabet_end_levels_and_softmax(oracle):
    """Level set {0, ..., 255} (eq. repo_alphabet with b = 8): clamping at 0 and 255, the CPMF against scipy's softmax,
    and the two-level logistic closed form shifted to the top pair of levels (254, 255)."""
    from scipy.special import softmax
    delta, alpha = float(np.float32(0.05)), float(np.float32(900.0))
    idx, soft, _ = oracle.quantize_fwd(np.array([-3.0, 0.0, 12.7499, 12.75, 100.0, 6.3751], np.float32), 0, 256, delta, alpha)
    assert idx.tolist() == [0, 0, 255, 255, 255, 128]
    theta = 11.93
    P, mode, _ = oracle.cpmf(theta, 0, 256, delta, alpha)
    ref = softmax(-alpha * (theta - np.arange(256) * delta) ** 2)
    np.testing.assert_allclose(P, ref, rtol=1e-12, atol=1e-300)
    assert mode == int(np.argmax(ref)) == 239
    # far above the set only the top two levels matter: P(255) = expit(alpha delta (2 theta - (254 + 255) delta))
    # (at theta = 12.9 level 253 carries e^-36 of the top level's weight)
    theta = 12.9
    P, _, _ = oracle.cpmf(theta, 0, 256, delta, alpha)
    assert P[254] == pytest.approx(expit(-alpha * delta * (2 * theta - 509 * delta)), rel=1e-9)
    assert P[255] == pytest.approx(expit(alpha * delta * (2 * theta - 509 * delta)), rel=1e-12)
    el = oracle.element(theta, 0, 256, delta, alpha)
    assert el["soft"] == pytest.approx(delta * (254 + P[255]), rel=1e-12)


def test_hard_index_tie_goes_to_lower_level(oracle):
    # theta exactly halfway between levels 1 and 2 (binary-exact values)
    idx, soft, gap = oracle.quantize_fwd(np.array([0.375, -0.375, 0.125], np.float32), -4, 8, 0.25, 64.0)
    assert idx.tolist() == [1, -2, 0]
    assert np.all(gap == 0.0)


# ---------------------------------------------------------------- soft value Q_d (eq. softQ) and its limits

def test_soft_value_tends_to_hard_value_as_alpha_grows(oracle):
    # Sec. III-B, last paragraph: Q_d converges to the uniform quantizer as alpha grows
    rng = np.random.default_rng(4)
    lo, L, delta = -7, 15, 0.02
    theta = rng.normal(0, 0.05, size=2000).astype(np.float32)
    prev = None
    for kappa in (1.0, 10.0, 100.0, 1e4):
        idx, soft, gap = oracle.quantize_fwd(theta, lo, L, delta, kappa / delta ** 2)
        err = np.abs(soft - idx * float(np.float32(delta)))
        if prev is not None:
            assert err.mean() < prev
        prev = err.mean()
    # at kappa = 1e4 everything at least 1% of a step from a midpoint is hard to 1e-12*delta
    r = theta.astype(np.float64) / float(np.float32(delta))
    inside = (np.abs(r) < L // 2)
    away = np.abs(np.abs(r - np.floor(r)) - 0.5) > 0.01
    assert np.all(err[inside & away] < 1e-12 * delta)


def test_soft_value_limits(oracle):
    lo, L, delta = -8, 16, 0.1
    # alpha -> 0: uniform CPMF, Q_d = mean of the alphabet
    e = oracle.element(0.123, lo, L, delta, 1e-12)
    assert e["soft"] == pytest.approx(delta * (lo + lo + L - 1) / 2.0, abs=1e-9)
    # exact midpoint of a deep-interior pair at large sharpness: two equal masses
    e = oracle.element(0.25 + 0.125, -20, 41, 0.25, 400.0 / 0.0625)
    assert e["soft"] == pytest.approx(0.375, abs=1e-13)
    # on a level with large sharpness: that level
    e = oracle.element(0.5, -20, 41, 0.25, 400.0 / 0.0625)
    assert e["soft"] == pytest.approx(0.5, abs=1e-13) and e["idx"] == 2


def test_soft_value_is_odd_on_symmetric_set_and_monotone(oracle):
    lo, L, delta, alpha = -7, 15, 0.02, 1e4
    theta = np.linspace(-0.2, 0.2, 801).astype(np.float32)
    _, soft, _ = oracle.quantize_fwd(theta, lo, L, delta, alpha)
    _, softm, _ = oracle.quantize_fwd(-theta, lo, L, delta, alpha)
    np.testing.assert_allclose(soft, -softm, rtol=0, atol=1e-15)
    assert np.all(np.diff(soft) >= -1e-15)  # dQd/dtheta = 2 alpha Var >= 0


# ---------------------------------------------------------------- Proposition 1 (Sec. III-B, proof in App. A)

@pytest.mark.parametrize("lo,L", [(-4, 8), (0, 16), (-15, 31)])
def test_proposition_1_distortion_decomposition(oracle, lo, L):
    rng = np.random.default_rng(5)
    delta = 0.1
    for kappa in (0.3, 1.0, 5.0, 30.0):
        alpha = kappa / delta ** 2
        for theta in rng.uniform((lo - 1) * delta, (lo + L) * delta, size=25):
            P, _, _ = oracle.cpmf(theta, lo, L, delta, alpha)
            levels = delta * np.arange(lo, lo + L)
            lhs = float(np.sum(P * (theta - levels) ** 2))       # E{(theta - Q_p)^2 | theta} by enumeration
            e = oracle.element(theta, lo, L, delta, alpha)
            var = e["dtheta"] / (2 * alpha)                        # Lemma 1 first line
            assert lhs == pytest.approx((theta - e["soft"]) ** 2 + var, rel=1e-11, abs=1e-15)


# ---------------------------------------------------------------- Lemma 1 and d/dalpha by finite differences

def _paper_parameter_sets(prefix):
    """(lo, n_levels, delta, alpha) of the rows of tests/golden/paper_parameters.txt whose name starts with prefix."""
    import os
    rows = []
    for line in open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_parameters.txt")):
        f = line.split("#")[0].split()
        if len(f) == 5 and f[0].startswith(prefix):
            rows.append((int(f[1]), int(f[2]), float(f[3]), float(f[4])))
    return rows


FIG1 = _paper_parameter_sets("fig1_")   # the parameter set of Figs. 1-2: b=3, q=0.1, four sharpness values
assert len(FIG1) == 4
OTHER = [(-7, 15, 0.02, 1e4), (0, 16, 0.25, 64.0), (0, 16, 0.25, 500.0), (-15, 31, 0.004, 2.5e5),
         (-15, 31, 0.004, 500.0), (-127, 255, 0.15, 4 / 0.15 ** 2), (-8, 16, 0.3, 0.7)]


@pytest.mark.parametrize("lo,L,delta,alpha", FIG1 + OTHER)
def test_analytic_gradients_match_central_finite_differences(oracle, lo, L, delta, alpha):
    rng = np.random.default_rng(6)
    soft = lambda th, dl, al: oracle.element(th, lo, L, dl, al)["soft"]
    thetas = list(rng.uniform((lo - 0.7) * delta, (lo + L - 0.3) * delta, size=40))
    thetas += [lo * delta, (lo + L - 1) * delta, (lo + 0.5) * delta, 0.0]
    for theta in thetas:
        e = oracle.element(theta, lo, L, delta, alpha)
        scale = abs(e["soft"]) + delta
        fd_t = _fd(lambda x: soft(x, delta, alpha), theta, 1e-6 * delta)
        fd_d = _fd(lambda x: soft(theta, x, alpha), delta, 1e-6 * delta)
        fd_a = _fd(lambda x: soft(theta, delta, x), alpha, 1e-5 * alpha)
        assert e["dtheta"] == pytest.approx(fd_t, rel=2e-6, abs=1e-8)
        assert e["ddelta"] == pytest.approx(fd_d, rel=2e-6, abs=1e-7 * max(1.0, abs(lo), abs(lo + L)))
        assert e["dalpha"] == pytest.approx(fd_a, rel=2e-6, abs=1e-9 * scale / alpha + 1e-16)


def test_cpmf_partials_match_appendix_b_identities(oracle):
    # eq. partialw2 and eq. partialq2 (App. B): dP_i/dtheta and dP_i/dq in terms of P itself
    lo, L, delta, alpha = -4, 8, 0.1, 300.0
    idx = np.arange(lo, lo + L)
    for theta in (-0.33, -0.049, 0.02, 0.151, 0.29):
        P, _, _ = oracle.cpmf(theta, lo, L, delta, alpha)
        d = theta - idx * delta
        want_t = -2 * alpha * P * d + 2 * alpha * P * np.sum(d * P)
        want_q = 2 * alpha * idx * P * d - 2 * alpha * P * np.sum(idx * d * P)
        h = 1e-7
        fd_t = (oracle.cpmf(theta + h, lo, L, delta, alpha)[0] - oracle.cpmf(theta - h, lo, L, delta, alpha)[0]) / (2 * h)
        fd_q = (oracle.cpmf(theta, lo, L, delta + h, alpha)[0] - oracle.cpmf(theta, lo, L, delta - h, alpha)[0]) / (2 * h)
        np.testing.assert_allclose(fd_t, want_t, rtol=1e-6, atol=1e-8)
        np.testing.assert_allclose(fd_q, want_q, rtol=1e-6, atol=1e-8)


def test_dsoft_dtheta_grows_away_from_the_nearest_level(oracle):
    # Sec. III-B, text after Lemma 1: the derivative increases as theta moves away from its nearest level
    # (checked for alpha >= 300: at alpha = 100, i.e. alpha q^2 = 1, the derivative stays within 1% of 1 and the
    #  edge of the 8-level alphabet already bends the curve, so the statement is not a strict inequality there)
    lo, L, delta = -4, 8, 0.1
    for alpha in (300.0, 500.0, 700.0):
        for k in (-2, 0, 1):
            up = [oracle.element(k * delta + f * delta, lo, L, delta, alpha)["dtheta"] for f in np.linspace(0, 0.5, 26)]
            dn = [oracle.element(k * delta - f * delta, lo, L, delta, alpha)["dtheta"] for f in np.linspace(0, 0.5, 26)]
            assert np.all(np.diff(up) > 0) and np.all(np.diff(dn) > 0)


def test_scaling_identity_ties_the_three_partials_together(oracle):
    # Q_d(c theta; c delta, alpha/c^2) = c Q_d(theta; delta, alpha)  =>  theta d/dtheta + delta d/ddelta - 2 alpha d/dalpha = Q_d
    rng = np.random.default_rng(7)
    for lo, L in [(-4, 8), (0, 16), (-127, 255)]:
        for _ in range(30):
            delta = rng.uniform(0.01, 1.0)
            alpha = rng.uniform(0.05, 40.0) / delta ** 2
            theta = rng.uniform((lo - 1) * delta, (lo + L) * delta)
            e = oracle.element(theta, lo, L, delta, alpha)
            lhs = theta * e["dtheta"] + delta * e["ddelta"] - 2 * alpha * e["dalpha"]
            assert lhs == pytest.approx(e["soft"], rel=1e-9, abs=1e-9 * delta * L)
            assert oracle.element(3 * theta, lo, L, 3 * delta, alpha / 9)["soft"] == pytest.approx(3 * e["soft"], rel=1e-12, abs=1e-15)


def test_lemma_1_as_printed_with_raw_powers_agrees_where_it_is_well_conditioned(oracle):
    rng = np.random.default_rng(8)
    for lo, L, delta, alpha in [(-4, 8, 0.1, 300.0), (0, 16, 0.25, 64.0), (-7, 15, 0.02, 2500.0)]:
        for theta in rng.uniform(lo * delta, (lo + L - 1) * delta, size=20):
            e = oracle.element(theta, lo, L, delta, alpha)
            raw_t, raw_q = oracle.lemma1_raw(theta, lo, L, delta, alpha)
            assert e["dtheta"] == pytest.approx(raw_t, rel=1e-8, abs=1e-12)
            assert e["ddelta"] == pytest.approx(raw_q, rel=1e-8, abs=1e-10)


# ---------------------------------------------------------------- tensor backward: chain rule and scalar sums (Sec. IV-B)

def test_tensor_backward_is_elementwise_product_and_sum_of_element_partials(oracle):
    rng = np.random.default_rng(9)
    lo, L, delta, alpha = -7, 15, float(np.float32(0.02)), float(np.float32(1e4))
    theta = rng.normal(0, 0.05, 64).astype(np.float32)
    g = rng.normal(0, 1, 64).astype(np.float32)
    out = oracle.quantize_bwd(theta, g, lo, L, delta, alpha)
    # finite differences of the scalar function F = sum_e g_e Q_d(theta_e) in theta_e, delta, alpha
    F = lambda th, dl, al: sum(float(ge) * oracle.element(float(t), lo, L, dl, al)["soft"] for t, ge in zip(th, g))
    th64 = theta.astype(np.float64)
    assert out["d_delta"] == pytest.approx(_fd(lambda x: F(th64, x, alpha), delta, 1e-7 * delta), rel=1e-6, abs=1e-6)
    assert out["d_alpha"] == pytest.approx(_fd(lambda x: F(th64, delta, x), alpha, 1e-5 * alpha), rel=1e-5, abs=1e-12)
    for j in (0, 17, 63):
        def Fj(x):
            t = th64.copy(); t[j] = x
            return F(t, delta, alpha)
        assert out["dtheta"][j] == pytest.approx(_fd(Fj, th64[j], 1e-6 * delta), rel=1e-6, abs=1e-9)


def test_per_entry_moments_of_lemma_1(oracle):
    """oracle.moments returns E, Var, Skew_u per entry.  Pinned by: the raw-power definitions of Lemma 1 written out
    with numpy on the CPMF (small indices, where raw powers are well conditioned); the two-level closed form
    (Bernoulli: E = q s, Var = q^2 s (1 - s), Skew_u = E X^3 - E X E X^2 = q^3 s (1 - s)); and Lemma 1 itself,
    which turns them into the partials that finite differences pin elsewhere in this file."""
    rng = np.random.default_rng(21)
    lo, L, delta, alpha = -4, 8, 0.1, 300.0
    theta = rng.uniform(-0.5, 0.45, 40).astype(np.float32)
    E, V, S = oracle.moments(theta, lo, L, delta, alpha)
    v = (lo + np.arange(L)) * np.float64(np.float32(delta))
    for e, t in enumerate(theta):
        P, _, _ = oracle.cpmf(float(t), lo, L, float(np.float32(delta)), float(np.float32(alpha)))
        e1, e2, e3 = np.sum(P * v), np.sum(P * v ** 2), np.sum(P * v ** 3)
        assert E[e] == pytest.approx(e1, rel=1e-12, abs=1e-15)
        assert V[e] == pytest.approx(e2 - e1 ** 2, rel=1e-9, abs=1e-15)
        assert S[e] == pytest.approx(e3 - e1 * e2, rel=1e-9, abs=1e-15)
        el = oracle.element(float(t), lo, L, float(np.float32(delta)), float(np.float32(alpha)))
        a64, d64 = float(np.float32(alpha)), float(np.float32(delta))
        assert el["dtheta"] == pytest.approx(2.0 * a64 * V[e], rel=1e-12)
        assert el["ddelta"] == pytest.approx((E[e] + 2.0 * a64 * float(t) * V[e] - 2.0 * a64 * S[e]) / d64, rel=1e-9, abs=1e-12)
    # two levels {0, q}
    q, al = float(np.float32(0.3)), float(np.float32(25.0))
    th = np.array([0.05, 0.15, 0.2, -0.4, 0.9], np.float32)
    E, V, S = oracle.moments(th, 0, 2, q, al)
    s = expit(al * q * (2.0 * th.astype(np.float64) - q))
    np.testing.assert_allclose(E, q * s, rtol=1e-12)
    np.testing.assert_allclose(V, q * q * s * (1 - s), rtol=1e-10, atol=1e-18)
    np.testing.assert_allclose(S, q ** 3 * s * (1 - s), rtol=1e-10, atol=1e-18)


def test_size_measure_of_the_scalar_sums_in_closed_form_cases(oracle):
    """The size of what the two scalar sums add up, as the GPU tests form it from the oracle's per-entry moments
    (tests/gpu_util.py), where it has a closed form.
    Sharp regime, theta on a level: the CPMF is one-hot, variance and third moment vanish, dQd/dq is the index
    itself, so the size is sum |g| |index| and that of the alpha sum is 0.  Soft regime, level set far from
    zero: E is about theta and 2 alpha Var about 1, so the three pieces of dQd/dq are E/q, -E/q and ~0 and the
    size is about 2 sum |g theta| / q while the sum itself is far smaller."""
    import gpu_util as gu
    delta = float(np.float32(0.25))
    idx = np.array([3, -5, 0, 7], dtype=np.float64)
    theta = (idx * delta).astype(np.float32)
    g = np.array([1.5, -2.0, 4.0, 0.5], dtype=np.float32)
    args = (-8, 16, delta, float(np.float32(1e4 / delta ** 2)))
    out = oracle.quantize_bwd(theta, g, *args)
    size_d, size_a = gu.scalar_sum_sizes(oracle, theta, g, *args)
    assert size_d == pytest.approx(float(np.sum(np.abs(g) * np.abs(idx))), rel=1e-12)
    assert size_a == pytest.approx(0.0, abs=1e-12)
    assert out["d_delta"] == pytest.approx(float(np.sum(g * idx)), rel=1e-12)

    # sharp regime, theta on a midpoint: P = (1/2, 1/2), Var = q^2 / 4, C3 = 0, E = theta: the term vanishes, and
    # its size is 2 (q/2 + q/2) q^2/4 = q^3 / 2 per unit of |g|
    mid = np.array([2.5 * delta], dtype=np.float32)
    g1 = np.array([3.0], np.float32)
    out = oracle.quantize_bwd(mid, g1, *args)
    assert gu.scalar_sum_sizes(oracle, mid, g1, *args)[1] == pytest.approx(3.0 * delta ** 3 / 2.0, rel=1e-9)
    assert abs(out["d_alpha"]) < 1e-12

    rng = np.random.default_rng(4)
    lo, L = 60, 60                                             # levels 60 .. 119
    theta = (rng.uniform(80.0, 100.0, 500) * delta).astype(np.float32)
    g = rng.normal(0, 1, 500).astype(np.float32)
    args = (lo, L, delta, float(np.float32(0.3 / delta ** 2)))
    out = oracle.quantize_bwd(theta, g, *args)
    size = 2.0 * float(np.sum(np.abs(g.astype(np.float64) * theta.astype(np.float64)))) / delta
    size_d, _ = gu.scalar_sum_sizes(oracle, theta, g, *args)
    assert size_d == pytest.approx(size, rel=1e-3)
    assert abs(out["d_delta"]) < 1e-6 * size_d


def test_scalar_sum_check_takes_the_stated_tolerance_first():
    """The helper of the GPU tests: inside 1e-6 + 1e-5|ref| passes; outside it fails unless the sum has cancelled
    to under a thousandth of its size and the error is under 2e-7 of that size."""
    import gpu_util as gu
    assert gu.check_scalar_sum("t", "x", 1.0 + 5e-6, 1.0) <= 1.0
    with pytest.raises(AssertionError):
        gu.check_scalar_sum("t", "x", 1.0 + 5e-5, 1.0, lambda: 100.0)            # not cancelled: 1 > 1e-3 * 100
    with pytest.raises(AssertionError):
        gu.check_scalar_sum("t", "x", 1.0 + 5e-5, 1.0, lambda: 1e6, strict_only=True)
    assert gu.check_scalar_sum("t", "x", 1.0 + 5e-5, 1.0, lambda: 1e4) > 1.0     # cancelled, 5e-5 < 2e-7 * 1e4
    with pytest.raises(AssertionError):
        gu.check_scalar_sum("t", "x", 1.0 + 5e-2, 1.0, lambda: 1e4)              # cancelled, but beyond 2e-7 of the size
    del gu.SCALAR_LOG[:]

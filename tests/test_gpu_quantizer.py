"""GPU parity of the quantizer entry points against the CPU oracle, element by element.

Sizes are chosen so that the oracle finishes in seconds while the GPU launch
still spans many blocks and ends in a ragged tail (n not a multiple of 4).
"""
import numpy as np
import pytest

import cdl_inputs
from cdl_inputs import QuantSpec
import gpu_util as gu

pytestmark = pytest.mark.gpu

KAPPAS = (0.01, 0.2, 1.0, 4.0, 30.0, 1e4)
SETS = [(-7, 15), (0, 16), (-15, 31), (-8, 16), (-127, 255)]


def _spec(lo, L, delta, kappa):
    d = float(np.float32(delta))
    return QuantSpec(lo, L, d, float(np.float32(kappa / (d * d))))


def _theta(lo, L, delta, n, seed):
    """Values spread over the whole alphabet plus some beyond both ends, midpoints and exact levels."""
    hi = lo + L - 1
    rng = np.random.default_rng(seed)
    th = rng.uniform((lo - 1.5) * delta, (hi + 1.5) * delta, size=n)
    th[: n // 8] = rng.normal(0.0, 2.5 * delta, size=n // 8)
    k = rng.integers(lo, hi + 1, size=64)
    th[-64:-32] = k[:32] * np.float64(np.float32(delta))                    # on a level
    th[-32:] = (k[32:] + 0.5) * np.float64(np.float32(delta))               # on a midpoint (up to fp32 rounding)
    th[-70:-64] = [1e3 * delta, -1e3 * delta, 1e6 * delta, -1e6 * delta, 0.0, -0.0]
    return th.astype(np.float32)


@pytest.mark.parametrize("lo,L", SETS)
@pytest.mark.parametrize("kappa", KAPPAS)
def test_quantize_fwd_matches_oracle(oracle, lo, L, kappa):
    n = 20011 if L <= 31 or kappa >= 1.0 else 6007
    spec = _spec(lo, L, 0.0731, kappa)
    theta = _theta(lo, L, spec.delta, n, seed=abs(lo) * 131 + L)
    q = gu.Quantizer(spec)
    idx, soft, marg, H = q.fwd(gu.dev(theta))
    r_idx, r_soft, r_gap = oracle.quantize_fwd(theta, *q.args)
    r_marg, r_H = oracle.marginal_entropy(theta, *q.args)
    gu.assert_indices(idx, r_idx, r_gap, "idx")
    gu.assert_close(soft, r_soft, "soft")
    gu.assert_close(marg, r_marg, "marg")
    gu.assert_close([H], [r_H], "entropy")
    assert marg.sum() == pytest.approx(1.0, abs=2e-6)


@pytest.mark.parametrize("lo,L", SETS)
@pytest.mark.parametrize("kappa", KAPPAS)
def test_quantize_bwd_matches_oracle(oracle, lo, L, kappa):
    n = 20011 if L <= 31 or kappa >= 1.0 else 6007
    spec = _spec(lo, L, 0.0731, kappa)
    theta = _theta(lo, L, spec.delta, n, seed=abs(lo) * 17 + L)
    g = np.random.default_rng(5).standard_normal(n).astype(np.float32)
    q = gu.Quantizer(spec)
    dth, dd, da = q.bwd(gu.dev(theta), gu.dev(g))
    ref = oracle.quantize_bwd(theta, g, *q.args)
    gu.assert_close(dth, ref["dtheta"], "dtheta")
    gu.check_quantizer_scalars(oracle, "bwd levels %d..%d kappa %g" % (lo, lo + L - 1, kappa), theta, g, q.args, dd, da, ref)


@pytest.mark.parametrize("lo,L", [(0, 2), (-1, 3), (-128, 256), (100, 28), (-128, 9)])
@pytest.mark.parametrize("kappa", (0.05, 4.0, 1e4))
def test_smallest_widest_and_off_centre_level_sets(oracle, lo, L, kappa):
    """Two levels, three levels, all 256 int8 levels, and sets that sit at either end of the int8 range."""
    n = 12007 if L < 256 or kappa >= 1.0 else 4003
    spec = _spec(lo, L, 0.0731, kappa)
    theta = _theta(lo, L, spec.delta, n, seed=abs(lo) * 7 + L)
    g = np.random.default_rng(8).standard_normal(n).astype(np.float32)
    q = gu.Quantizer(spec)
    idx, soft, marg, H = q.fwd(gu.dev(theta))
    r_idx, r_soft, r_gap = oracle.quantize_fwd(theta, *q.args)
    r_marg, r_H = oracle.marginal_entropy(theta, *q.args)
    gu.assert_indices(idx, r_idx, r_gap, "idx")
    gu.assert_close(soft, r_soft, "soft")
    gu.assert_close(marg, r_marg, "marg")
    gu.assert_close([H], [r_H], "entropy")
    dth, dd, da = q.bwd(gu.dev(theta), gu.dev(g))
    ref = oracle.quantize_bwd(theta, g, *q.args)
    gu.assert_close(dth, ref["dtheta"], "dtheta")
    gu.check_quantizer_scalars(oracle, "edge sets levels %d..%d kappa %g" % (lo, lo + L - 1, kappa), theta, g, q.args, dd, da, ref)


@pytest.mark.parametrize("lo,L", [(0, 6), (-3, 7), (-4, 8), (100, 9), (-128, 10), (-8, 17), (0, 18), (95, 32), (-16, 33), (-128, 33)])
@pytest.mark.parametrize("kappa,delta", [(0.004, 0.9), (0.05, 0.0731), (0.25, 0.011)])
def test_soft_regime_on_small_level_sets(oracle, lo, L, kappa, delta):
    """At most 33 levels, all of them live (the regime of the paper's initial sharpness, Sec. V-B): the kernels
    that evaluate every entry about the centre of the level set.  Even and odd level counts, every padded loop
    length, sets at either end of the int8 range, a large step (where a soft value next to zero has only the absolute
    tolerance), values far outside the set, exact levels and midpoints, a ragged tail."""
    n = 9001 + L
    spec = _spec(lo, L, delta, kappa)
    theta = _theta(lo, L, spec.delta, n, seed=L * 31 + abs(lo))
    g = np.random.default_rng(L).standard_normal(n).astype(np.float32)
    q = gu.Quantizer(spec)
    th_d, g_d = gu.dev(theta), gu.dev(g)
    idx, soft, marg, H = q.fwd(th_d)
    r_idx, r_soft, r_gap = oracle.quantize_fwd(theta, *q.args)
    r_marg, r_H = oracle.marginal_entropy(theta, *q.args)
    gu.assert_indices(idx, r_idx, r_gap, "idx")
    gu.assert_close(soft, r_soft, "soft")
    gu.assert_close(marg, r_marg, "marg")
    gu.assert_close([H], [r_H], "entropy")
    marg2, H2 = q.marginal(th_d)
    assert np.array_equal(marg2, marg) and H2 == H
    _, soft_only, _, _ = q.fwd(th_d, marg=False)
    assert np.array_equal(soft_only, soft)
    dth, dd, da = q.bwd(th_d, g_d)
    ref = oracle.quantize_bwd(theta, g, *q.args)
    gu.assert_close(dth, ref["dtheta"], "dtheta")
    gu.check_quantizer_scalars(oracle, "soft regime levels %d..%d kappa %g delta %g" % (lo, lo + L - 1, kappa, delta),
                               theta, g, q.args, dd, da, ref)
    dth_only, _, _ = q.bwd(th_d, g_d, scalars=False)
    assert np.array_equal(dth_only, dth)
    _, dd2, da2 = q.bwd(th_d, g_d, dtheta=False)
    assert dd2 == dd and da2 == da


@pytest.mark.parametrize("lo,L,kappa", [(-7, 15, 4.0), (0, 16, 31.25), (-15, 31, 0.008), (-127, 255, 4.0)])
def test_marginal_entropy_entry_point_matches_oracle(oracle, lo, L, kappa):
    spec = _spec(lo, L, 0.02, kappa)
    theta = (np.random.default_rng(3).standard_normal(30001) * 0.05).astype(np.float32)
    q = gu.Quantizer(spec)
    marg, H = q.marginal(gu.dev(theta))
    r_marg, r_H = oracle.marginal_entropy(theta, *q.args)
    gu.assert_close(marg, r_marg, "marg")
    gu.assert_close([H], [r_H], "entropy")
    # the fused and the stand-alone path agree with each other too
    _, _, marg2, H2 = q.fwd(gu.dev(theta))
    gu.assert_close(marg2, r_marg, "marg (fused)")


def test_workload_1_weights_and_activations(oracle):
    wl = cdl_inputs.workload(1)
    for theta, spec in ((cdl_inputs.draw_w(wl), wl.w_spec), (cdl_inputs.draw_x(wl), wl.x_spec)):
        for sp in (spec, spec.with_alpha(cdl_inputs.ALPHA_PAPER)):
            q = gu.Quantizer(sp)
            flat = theta.reshape(-1)
            idx, soft, marg, H = q.fwd(gu.dev(flat))
            r_idx, r_soft, r_gap = oracle.quantize_fwd(flat, *q.args)
            r_marg, r_H = oracle.marginal_entropy(flat, *q.args)
            gu.assert_indices(idx, r_idx, r_gap, "idx")
            gu.assert_close(soft, r_soft, "soft")
            gu.assert_close(marg, r_marg, "marg")
            gu.assert_close([H], [r_H], "H")


@pytest.mark.parametrize("n", [0, 1, 2, 3, 4, 5, 255, 1024, 1027])
def test_tiny_and_empty_tensors(oracle, n):
    torch = gu.torch_mod()
    spec = _spec(-7, 15, 0.02, 4.0)
    q = gu.Quantizer(spec)
    theta = (np.random.default_rng(n).standard_normal(n) * 0.05).astype(np.float32)
    g = np.random.default_rng(n + 1).standard_normal(n).astype(np.float32)
    th_d = gu.dev(theta) if n else torch.empty(0, dtype=torch.float32, device="cuda")
    g_d = gu.dev(g) if n else torch.empty(0, dtype=torch.float32, device="cuda")
    idx, soft, marg, H = q.fwd(th_d)
    dth, dd, da = q.bwd(th_d, g_d)
    if n == 0:
        assert np.all(marg == 0.0) and H == 0.0 and dd == 0.0 and da == 0.0
        return
    r_idx, r_soft, r_gap = oracle.quantize_fwd(theta, *q.args)
    r_marg, r_H = oracle.marginal_entropy(theta, *q.args)
    ref = oracle.quantize_bwd(theta, g, *q.args)
    gu.assert_indices(idx, r_idx, r_gap, "idx")
    gu.assert_close(soft, r_soft, "soft")
    gu.assert_close(marg, r_marg, "marg")
    gu.assert_close([H], [r_H], "H")
    gu.assert_close(dth, ref["dtheta"], "dtheta")
    gu.assert_close([dd], [ref["d_delta"]], "d_delta")
    gu.assert_close([da], [ref["d_alpha"]], "d_alpha")


def test_exact_ties_go_to_the_lower_level():
    # delta = 0.25: midpoints are exactly representable
    spec = QuantSpec(-4, 8, 0.25, 64.0)
    q = gu.Quantizer(spec)
    theta = np.array([0.375, -0.375, 0.125, -0.125, 0.625, -1.125, 0.875, 5.0], np.float32)
    idx, soft, _, _ = q.fwd(gu.dev(theta))
    assert idx.tolist() == [1, -2, 0, -1, 2, -4, 3, 3]


def test_results_are_reproducible_bit_for_bit():
    spec = _spec(-15, 31, 0.004, 4.0)
    q = gu.Quantizer(spec)
    theta = (np.random.default_rng(9).standard_normal(300007) * 0.02).astype(np.float32)
    g = np.random.default_rng(10).standard_normal(300007).astype(np.float32)
    th_d, g_d = gu.dev(theta), gu.dev(g)
    a = q.bwd(th_d, g_d)
    b = q.bwd(th_d, g_d)
    assert np.array_equal(a[0], b[0]) and a[1] == b[1] and a[2] == b[2]
    f1 = q.fwd(th_d)
    f2 = q.fwd(th_d)
    assert np.array_equal(f1[0], f2[0]) and np.array_equal(f1[1], f2[1])


def test_outputs_are_optional():
    torch = gu.torch_mod()
    spec = _spec(0, 16, 0.25, 4.0)
    q = gu.Quantizer(spec)
    theta = np.abs(np.random.default_rng(2).standard_normal(5003)).astype(np.float32)
    g = np.random.default_rng(3).standard_normal(5003).astype(np.float32)
    th_d, g_d = gu.dev(theta), gu.dev(g)
    full = q.fwd(th_d)
    only_idx = q.fwd(th_d, soft=False, marg=False)
    assert np.array_equal(full[0], only_idx[0]) and only_idx[1] is None
    b_full = q.bwd(th_d, g_d)
    b_t = q.bwd(th_d, g_d, scalars=False)
    b_s = q.bwd(th_d, g_d, dtheta=False)
    assert np.array_equal(b_full[0], b_t[0]) and b_full[1] == b_s[1] and b_full[2] == b_s[2]


def _sweep_cases():
    """Thirty seeded parameter sets: level sets anywhere in the int8 range, step sizes over three decades,
    sharpness either side of every band width the kernels are specialised for, odd tensor lengths."""
    rng = np.random.default_rng(2501)
    edges = [1.25, 1.3, 1.35, 1.85, 1.9, 1.95, 3.7, 3.8, 3.9, 10.7, 10.9, 11.1]
    cases = []
    for i in range(30):
        L = int(rng.integers(2, 257))
        lo = int(rng.integers(-128, 128 - L + 1))
        delta = float(10.0 ** rng.uniform(-3, 0))
        kappa = float(edges[i // 2]) if i < 24 else float(10.0 ** rng.uniform(-1.7, 4))
        n = int(rng.integers(1, 9000))
        cases.append((lo, L, delta, kappa, n))
    return cases


@pytest.mark.parametrize("lo,L,delta,kappa,n", _sweep_cases())
def test_forward_and_backward_on_seeded_random_parameters(oracle, lo, L, delta, kappa, n):
    spec = _spec(lo, L, delta, kappa)
    n = max(n, 80)   # the input recipe plants 70 special values
    theta = _theta(lo, L, spec.delta, n, seed=n + L)
    g = np.random.default_rng(n).standard_normal(n).astype(np.float32)
    q = gu.Quantizer(spec)
    idx, soft, marg, H = q.fwd(gu.dev(theta))
    r_idx, r_soft, r_gap = oracle.quantize_fwd(theta, *q.args)
    r_marg, r_H = oracle.marginal_entropy(theta, *q.args)
    gu.assert_indices(idx, r_idx, r_gap, "idx")
    gu.assert_close(soft, r_soft, "soft")
    gu.assert_close(marg, r_marg, "marg")
    gu.assert_close([H], [r_H], "entropy")
    dth, dd, da = q.bwd(gu.dev(theta), gu.dev(g))
    ref = oracle.quantize_bwd(theta, g, *q.args)
    gu.assert_close(dth, ref["dtheta"], "dtheta")
    gu.check_quantizer_scalars(oracle, "sweep levels %d..%d delta %.3g kappa %.3g n %d" % (lo, lo + L - 1, delta, kappa, n),
                               theta, g, q.args, dd, da, ref)

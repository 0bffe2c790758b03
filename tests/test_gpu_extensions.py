"""GPU parity of the extensions of the path: truncated (top-k) CPMF, the probabilistic draw Q_p, and the
gradient of the entropy term, each against the CPU oracle on the same seeded inputs.

Tolerances as for the core path.  The draw is an integer decision made on fp32 cumulative sums: entries
whose uniform number lies within 1e-6 of a boundary of the oracle's cumulative distribution are exempt
(counted, and still have to be a neighbouring level).
"""
import numpy as np
import pytest

import cdl_inputs
import gpu_util as gu

pytestmark = pytest.mark.gpu

SPECS = [(-7, 15, 0.02), (0, 16, 0.25), (-15, 31, 0.004), (-127, 255, 0.15092)]


def _theta(lo, n_levels, delta, n, seed):
    rng = np.random.default_rng(seed)
    th = rng.normal(0.0, 0.3 * n_levels * delta, n)
    if lo == 0:
        th = np.abs(th)
    th[:16] = np.linspace((lo - 3) * delta, (lo + n_levels + 2) * delta, 16)      # beyond both ends
    th[16:32] = (np.arange(16) + lo + 0.5) * delta                                  # exact midpoints
    return th.astype(np.float32)


def _call(fn, *a, **kw):
    fn(*a, **kw)
    gu.torch_mod().cuda.synchronize()


@pytest.mark.parametrize("lo,n_levels,delta", SPECS)
@pytest.mark.parametrize("kappa", [0.05, 0.7, 4.0, 50.0])
@pytest.mark.parametrize("top_k", [1, 3, 5])
def test_truncated_cpmf_forward_backward_marginal(oracle, lo, n_levels, delta, kappa, top_k):
    import paper_2501_09849_amd as cdl
    torch = gu.torch_mod()
    n = 20003
    spec = cdl_inputs.QuantSpec(lo, n_levels, float(np.float32(delta)), float(np.float32(kappa / np.float32(delta) ** 2)))
    a = (spec.lo, spec.n_levels, spec.delta, spec.alpha)
    th = _theta(lo, n_levels, spec.delta, n, seed=n_levels + top_k)
    g = np.random.default_rng(1).normal(0, 1, n).astype(np.float32)
    th_d, g_d = gu.dev(th), gu.dev(g)
    idx, soft, dth = gu.empty((n,), torch.int8), gu.empty((n,), torch.float32), gu.empty((n,), torch.float32)
    marg, sc = gu.empty((n_levels,), torch.float32), gu.empty((4,), torch.float32)
    ws = gu.workspace(cdl.quantize_workspace_bytes(n, n_levels))
    _call(cdl.cdl_quantize_fwd, th_d, n, *a, idx, soft, marg, sc[0:1], ws, top_k=top_k)
    _call(cdl.cdl_quantize_bwd, th_d, g_d, n, *a, dth, sc[1:2], sc[2:3], ws, top_k=top_k)
    r_idx, r_soft, gap = oracle.quantize_fwd(th, *a, top_k=top_k)
    gu.assert_indices(idx.cpu().numpy(), r_idx, gap, "idx")
    gu.assert_close(soft.cpu().numpy(), r_soft, "soft")
    r_m, r_h = oracle.marginal_entropy(th, *a, top_k=top_k)
    gu.assert_close(marg.cpu().numpy(), r_m, "marginal")
    gu.assert_close([float(sc[0])], [r_h], "entropy")
    rb = oracle.quantize_bwd(th, g, *a, top_k=top_k)
    gu.assert_close(dth.cpu().numpy(), rb["dtheta"], "dtheta")
    gu.check_quantizer_scalars(oracle, "top-%d levels %d..%d delta %g kappa %g" % (top_k, lo, lo + n_levels - 1, delta, kappa),
                               th, g, a, float(sc[1]), float(sc[2]), rb, top_k=top_k)
    # marginal-only entry point
    m2, h2 = gu.empty((n_levels,), torch.float32), gu.empty((1,), torch.float32)
    _call(cdl.cdl_marginal_entropy, th_d, n, *a, m2, h2, ws, top_k=top_k)
    gu.assert_close(m2.cpu().numpy(), r_m, "marginal (marginal-only call)")


def test_truncation_wider_than_the_level_set_is_the_full_cpmf(oracle):
    import paper_2501_09849_amd as cdl
    torch = gu.torch_mod()
    n = 4099
    a = (-2, 5, 0.1, 3.0)
    th = _theta(-2, 5, 0.1, n, seed=3)
    th_d = gu.dev(th)
    idx, s5, s0 = gu.empty((n,), torch.int8), gu.empty((n,), torch.float32), gu.empty((n,), torch.float32)
    _call(cdl.cdl_quantize_fwd, th_d, n, *a, idx, s5, top_k=5)
    _call(cdl.cdl_quantize_fwd, th_d, n, *a, idx, s0)
    assert torch.equal(s5, s0)
    with pytest.raises(cdl.CdlError):
        cdl.cdl_quantize_fwd(th_d, n, *a, idx, s5, top_k=4)


@pytest.mark.parametrize("lo,n_levels,delta", SPECS)
@pytest.mark.parametrize("kappa", [0.05, 0.7, 4.0, 30.0, 1e4])
@pytest.mark.parametrize("top_k", [0, 5])
def test_draw_matches_oracle(oracle, lo, n_levels, delta, kappa, top_k):
    import paper_2501_09849_amd as cdl
    torch = gu.torch_mod()
    n = 50003
    spec = cdl_inputs.QuantSpec(lo, n_levels, float(np.float32(delta)), float(np.float32(kappa / np.float32(delta) ** 2)))
    a = (spec.lo, spec.n_levels, spec.delta, spec.alpha)
    th = _theta(lo, n_levels, spec.delta, n, seed=7 + n_levels)
    u = np.random.default_rng(2).random(n, dtype=np.float32)
    u[:4] = [0.0, 1.0 - 2.0 ** -24, 0.5, 0.25]
    idx = gu.empty((n,), torch.int8)
    _call(cdl.cdl_quantize_draw, gu.dev(th), gu.dev(u), n, *a, idx, top_k=top_k)
    got = idx.cpu().numpy().astype(np.int64)
    ref, margin = oracle.quantize_draw(th, u, *a, top_k=top_k)
    diff = got != ref
    exempt = diff & (margin < 1e-6)
    assert not (diff & ~exempt).any(), "%d draws differ with a margin >= 1e-6 (first %d: gpu %d ref %d margin %.3g)" % (
        int((diff & ~exempt).sum()), int(np.argmax(diff & ~exempt)), got[np.argmax(diff & ~exempt)],
        ref[np.argmax(diff & ~exempt)], margin[np.argmax(diff & ~exempt)])
    assert np.all(np.abs(got[exempt] - ref[exempt]) == 1)
    assert exempt.sum() <= 20
    assert got.min() >= lo and got.max() <= lo + n_levels - 1


def test_draw_frequencies_follow_the_cpmf(oracle):
    import paper_2501_09849_amd as cdl
    torch = gu.torch_mod()
    lo, n_levels, d, a = -4, 8, 0.1, 150.0
    N = 200000
    u = ((np.arange(N) + 0.5) / N).astype(np.float32)
    for theta in (0.03, -0.17, 0.249):
        idx = gu.empty((N,), torch.int8)
        _call(cdl.cdl_quantize_draw, gu.dev(np.full(N, theta, np.float32)), gu.dev(u), N, lo, n_levels, d, a, idx)
        counts = np.bincount(idx.cpu().numpy().astype(np.int64) - lo, minlength=n_levels)
        P, _, _ = oracle.cpmf(float(np.float32(theta)), lo, n_levels, float(np.float32(d)), float(np.float32(a)))
        assert np.all(np.abs(counts - N * P) <= 3.0), (counts, N * P)


@pytest.mark.parametrize("lo,n_levels,delta", SPECS)
@pytest.mark.parametrize("kappa", [0.2, 1.0, 4.0, 30.0])
@pytest.mark.parametrize("top_k", [0, 5])
def test_entropy_gradient_matches_oracle(oracle, lo, n_levels, delta, kappa, top_k):
    import paper_2501_09849_amd as cdl
    torch = gu.torch_mod()
    n = 30001
    spec = cdl_inputs.QuantSpec(lo, n_levels, float(np.float32(delta)), float(np.float32(kappa / np.float32(delta) ** 2)))
    a = (spec.lo, spec.n_levels, spec.delta, spec.alpha)
    th = _theta(lo, n_levels, spec.delta, n, seed=11 + n_levels)
    g = np.random.default_rng(3).normal(0, 1, n).astype(np.float32)
    th_d, g_d = gu.dev(th), gu.dev(g)
    marg, H = gu.empty((n_levels,), torch.float32), gu.empty((1,), torch.float32)
    ws = gu.workspace(cdl.quantize_workspace_bytes(n, n_levels))
    _call(cdl.cdl_marginal_entropy, th_d, n, *a, marg, H, ws, top_k=top_k)
    # lambda * n for the total-bits term, with lambda chosen so that the entry gradients are of order one
    # (dH/dtheta = -(2 alpha delta / n) Cov(k, log2 m), and the covariance is of order one)
    scale = n / (2.0 * spec.alpha * spec.delta)
    dth, dth_add, sc = gu.empty((n,), torch.float32), gu.empty((n,), torch.float32), gu.empty((2,), torch.float32)
    _call(cdl.cdl_entropy_bwd, th_d, marg, n, *a, scale, None, dth, sc[0:1], sc[1:2], ws, top_k=top_k)
    _call(cdl.cdl_entropy_bwd, th_d, marg, n, *a, scale, g_d, dth_add, None, None, None, top_k=top_k)
    r = oracle.entropy_bwd(th, marg.cpu().numpy().astype(np.float64), *a, scale=scale, top_k=top_k, want_terms=True)
    gu.assert_close(dth.cpu().numpy(), r["dtheta"], "dH/dtheta")
    gu.assert_close(dth_add.cpu().numpy(), g.astype(np.float64) + r["dtheta"], "g + dH/dtheta")
    label = "dH levels %d..%d delta %g kappa %g top_k %d" % (lo, lo + n_levels - 1, delta, kappa, top_k)
    gu.check_scalar_sum(label, "d_delta", float(sc[0]), r["d_delta"], lambda: np.abs(r["term_delta"]).sum())
    gu.check_scalar_sum(label, "d_alpha", float(sc[1]), r["d_alpha"], lambda: np.abs(r["term_alpha"]).sum())
    # scalars only
    sc2 = gu.empty((2,), torch.float32)
    _call(cdl.cdl_entropy_bwd, th_d, marg, n, *a, scale, None, None, sc2[0:1], sc2[1:2], ws, top_k=top_k)
    assert torch.equal(sc, sc2)


def test_extension_entry_points_on_tiny_and_empty_tensors(oracle):
    import paper_2501_09849_amd as cdl
    torch = gu.torch_mod()
    a = (-7, 15, 0.02, 1e4)
    for n in (0, 1, 3, 5):
        th = _theta(-7, 15, 0.02, 64, seed=n)[32:32 + n]
        u = np.random.default_rng(n).random(n, dtype=np.float32)
        th_d, u_d = gu.dev(np.ascontiguousarray(th)) if n else gu.empty((4,), torch.float32), gu.dev(u) if n else gu.empty((4,), torch.float32)
        idx = gu.empty((max(n, 4),), torch.int8)
        _call(cdl.cdl_quantize_draw, th_d, u_d, n, *a, idx)
        marg = gu.dev(np.full(15, 1 / 15, np.float32))
        dth, sc = gu.empty((max(n, 4),), torch.float32), gu.empty((2,), torch.float32).fill_(7.0)
        ws = gu.workspace(cdl.quantize_workspace_bytes(n, 15))
        _call(cdl.cdl_entropy_bwd, th_d, marg, n, *a, 1.0, None, dth, sc[0:1], sc[1:2], ws)
        if n:
            ref, margin = oracle.quantize_draw(th, u, *a)
            ok = (idx.cpu().numpy()[:n] == ref) | (margin < 1e-6)
            assert ok.all()
            assert float(dth[:n].abs().max()) < 1e-6        # uniform marginal: zero gradient
        assert abs(float(sc[0])) < 1e-6 and abs(float(sc[1])) < 1e-6


def _huffman_gpu(idx_h, lo, n_levels):
    import paper_2501_09849_amd as cdl
    torch = gu.torch_mod()
    n = idx_h.size
    idx_d = gu.dev(idx_h) if n else gu.empty((16,), torch.int8)
    counts = gu.empty((n_levels,), torch.int64)
    total = gu.empty((1,), torch.int64)
    avg = gu.empty((1,), torch.float32)
    ws = gu.workspace(cdl.huffman_workspace_bytes(n))
    cdl.cdl_huffman_bits(idx_d, n, lo, n_levels, counts, total, avg, ws)
    torch.cuda.synchronize()
    return counts.cpu().numpy(), int(total.item()), float(avg.item())


@pytest.mark.parametrize("lo,n_levels", [(-7, 15), (0, 16), (-15, 31), (-127, 255), (-128, 256)])
@pytest.mark.parametrize("n", [0, 1, 17, 4099, 1_000_003])
def test_huffman_bits_match_oracle(oracle, lo, n_levels, n):
    rng = np.random.default_rng(n_levels * 7 + n % 1000)
    p = rng.dirichlet(np.full(n_levels, 0.25))
    idx = (rng.choice(n_levels, size=n, p=p) + lo).astype(np.int8)
    counts, total, avg = _huffman_gpu(idx, lo, n_levels)
    r_counts, r_total, r_avg = oracle.huffman_bits(idx, lo, n_levels)
    assert np.array_equal(counts, r_counts)
    assert total == int(r_total)
    assert abs(avg - r_avg) <= 1e-6 + 1e-5 * r_avg


def test_huffman_bits_degenerate_and_out_of_set_entries(oracle):
    # a single level; two levels; entries outside the level set are ignored
    assert _huffman_gpu(np.full(1000, 3, np.int8), 0, 16)[1:] == (1000, 1.0)
    assert _huffman_gpu(np.int8([1, 2] * 500), 0, 16)[1] == 1000
    idx = np.int8([0, 1, 1, 2, 2, 2, 40, -40] * 64)
    counts, total, _ = _huffman_gpu(idx, 0, 4)
    r_counts, r_total, _ = oracle.huffman_bits(idx, 0, 4)
    assert np.array_equal(counts, r_counts) and total == int(r_total)


def test_huffman_bits_of_the_quantized_flat_tensor(oracle):
    """Workload 4 at full size: bits per weight of the hard indices, against the oracle on the same indices,
    and between the entropy of the index histogram and that entropy plus one."""
    import paper_2501_09849_amd as cdl
    torch = gu.torch_mod()
    wl = cdl_inputs.workload(4)
    spec = wl.w_spec
    W = cdl_inputs.draw_w(wl)
    n = W.size
    idx = gu.empty((n,), torch.int8)
    cdl.cdl_quantize_fwd(gu.dev(W), n, spec.lo, spec.n_levels, spec.delta, spec.alpha, idx)
    torch.cuda.synchronize()
    idx_h = idx.cpu().numpy()
    counts, total, avg = _huffman_gpu(idx_h, spec.lo, spec.n_levels)
    r_counts, r_total, r_avg = oracle.huffman_bits(idx_h, spec.lo, spec.n_levels)
    assert np.array_equal(counts, r_counts) and total == int(r_total)
    q = counts[counts > 0] / n
    H = -np.sum(q * np.log2(q))
    assert H <= avg + 1e-6 < H + 1.0


def _sweep_cases():
    """Twenty-four seeded parameter sets for the extensions: level sets anywhere in the int8 range, step sizes
    over three decades, sharpness either side of the band widths the kernels are specialised for, every
    truncation width, odd tensor lengths."""
    rng = np.random.default_rng(985)
    edges = [1.3, 1.9, 3.8, 10.9]
    cases = []
    for i in range(24):
        L = int(rng.integers(2, 257))
        lo = int(rng.integers(-128, 128 - L + 1))
        delta = float(10.0 ** rng.uniform(-3, 0))
        kappa = float(edges[i % 4] * (0.97 if i % 8 < 4 else 1.03)) if i < 16 else float(10.0 ** rng.uniform(-1.5, 3.5))
        top_k = int(rng.choice([0, 1, 3, 5, 7, 9]))   # (the widths the boundary accepts)
        if top_k >= L:
            top_k = 0
        cases.append((lo, L, delta, kappa, top_k, int(rng.integers(100, 7000))))
    return cases


@pytest.mark.parametrize("lo,n_levels,delta,kappa,top_k,n", _sweep_cases())
def test_extensions_on_seeded_random_parameters(oracle, lo, n_levels, delta, kappa, top_k, n):
    import paper_2501_09849_amd as cdl
    torch = gu.torch_mod()
    spec = cdl_inputs.QuantSpec(lo, n_levels, float(np.float32(delta)), float(np.float32(kappa / np.float32(delta) ** 2)))
    a = (spec.lo, spec.n_levels, spec.delta, spec.alpha)
    rng = np.random.default_rng(n)
    hi = lo + n_levels - 1
    th = rng.uniform((lo - 2.5) * spec.delta, (hi + 2.5) * spec.delta, n)
    th[:4] = [(hi + 40.0) * spec.delta, (lo - 40.0) * spec.delta, (hi + 1e5) * spec.delta, (lo - 1e5) * spec.delta]
    th = th.astype(np.float32)
    g = rng.normal(0, 1, n).astype(np.float32)
    u = rng.random(n, dtype=np.float32)
    th_d, g_d = gu.dev(th), gu.dev(g)
    ws = gu.workspace(cdl.quantize_workspace_bytes(n, n_levels))
    # truncated (or full) forward, marginal, backward
    idx, soft, dth = gu.empty((n,), torch.int8), gu.empty((n,), torch.float32), gu.empty((n,), torch.float32)
    marg, sc = gu.empty((n_levels,), torch.float32), gu.empty((6,), torch.float32)
    _call(cdl.cdl_quantize_fwd, th_d, n, *a, idx, soft, marg, sc[0:1], ws, top_k=top_k)
    _call(cdl.cdl_quantize_bwd, th_d, g_d, n, *a, dth, sc[1:2], sc[2:3], ws, top_k=top_k)
    r_idx, r_soft, gap = oracle.quantize_fwd(th, *a, top_k=top_k)
    gu.assert_indices(idx.cpu().numpy(), r_idx, gap, "idx")
    gu.assert_close(soft.cpu().numpy(), r_soft, "soft")
    r_m, r_h = oracle.marginal_entropy(th, *a, top_k=top_k)
    gu.assert_close(marg.cpu().numpy(), r_m, "marginal")
    gu.assert_close([float(sc[0])], [r_h], "entropy")
    rb = oracle.quantize_bwd(th, g, *a, top_k=top_k)
    gu.assert_close(dth.cpu().numpy(), rb["dtheta"], "dtheta")
    label = "ext sweep levels %d..%d delta %.3g kappa %.3g top_k %d n %d" % (lo, lo + n_levels - 1, spec.delta, spec.alpha * spec.delta ** 2, top_k, n)
    gu.check_quantizer_scalars(oracle, label, th, g, a, float(sc[1]), float(sc[2]), rb, top_k=top_k)
    # the draw
    didx = gu.empty((n,), torch.int8)
    _call(cdl.cdl_quantize_draw, th_d, gu.dev(u), n, *a, didx, top_k=top_k)
    got = didx.cpu().numpy().astype(np.int64)
    ref, margin = oracle.quantize_draw(th, u, *a, top_k=top_k)
    diff = got != ref
    assert not (diff & (margin >= 1e-6)).any(), "draws differ with a margin >= 1e-6"
    assert np.all(np.abs(got[diff] - ref[diff]) == 1) and diff.sum() <= 20
    # the gradient of the entropy term
    scale = n / (2.0 * spec.alpha * spec.delta)
    eth = gu.empty((n,), torch.float32)
    _call(cdl.cdl_entropy_bwd, th_d, marg, n, *a, scale, None, eth, sc[3:4], sc[4:5], ws, top_k=top_k)
    r = oracle.entropy_bwd(th, marg.cpu().numpy().astype(np.float64), *a, scale=scale, top_k=top_k, want_terms=True)
    gu.assert_close(eth.cpu().numpy(), r["dtheta"], "dH/dtheta")
    gu.check_scalar_sum(label + " dH", "d_delta", float(sc[3]), r["d_delta"], lambda: np.abs(r["term_delta"]).sum())
    gu.check_scalar_sum(label + " dH", "d_alpha", float(sc[4]), r["d_alpha"], lambda: np.abs(r["term_alpha"]).sum())


def _indices_with_counts(counts, lo, seed):
    idx = np.repeat(np.arange(len(counts)) + lo, counts).astype(np.int8)
    np.random.default_rng(seed).shuffle(idx)
    return idx


@pytest.mark.parametrize("shape", ["equal", "fibonacci", "powers_of_two", "one_heavy", "two_symbols_of_256"])
def test_huffman_bits_on_count_profiles_that_stress_the_merge(oracle, shape):
    """Equal counts on all 256 levels (every merge is a tie: the coded size is unique even where the tree is
    not); Fibonacci counts (the deepest tree a given total allows, codes longer than 32 bits); powers of two
    (a comb); one level holding almost everything; two used levels of 256."""
    lo, n_levels = -128, 256
    if shape == "equal":
        counts = np.full(256, 37)
    elif shape == "fibonacci":
        f = [1, 1]
        while len(f) < 40:
            f.append(f[-1] + f[-2])          # 40 levels, 267 914 295 entries in all would be too many: scale down
        counts = np.zeros(256, dtype=np.int64)
        counts[100:100 + 32] = f[:32]        # 32 levels, total 5 702 886, code lengths up to 31
        counts[10:14] = [1, 1, 1, 1]         # and a few more leaves at the bottom: lengths beyond 32
    elif shape == "powers_of_two":
        counts = np.zeros(256, dtype=np.int64)
        counts[:21] = 2 ** np.arange(21)
    elif shape == "one_heavy":
        counts = np.ones(256, dtype=np.int64)
        counts[77] = 3_000_000
    else:
        counts = np.zeros(256, dtype=np.int64)
        counts[3], counts[250] = 12345, 678
    idx = _indices_with_counts(counts, lo, seed=len(shape))
    got_counts, total, avg = _huffman_gpu(idx, lo, n_levels)
    r_counts, r_total, r_avg = oracle.huffman_bits(idx, lo, n_levels)
    assert np.array_equal(got_counts, counts) and np.array_equal(r_counts, counts)
    assert total == int(r_total)
    assert abs(avg - r_avg) <= 1e-6 + 1e-5 * r_avg
    if shape == "equal":
        assert total == 8 * idx.size             # 256 equal counts: every code has 8 bits
    if shape == "two_symbols_of_256":
        assert total == idx.size                 # one bit each

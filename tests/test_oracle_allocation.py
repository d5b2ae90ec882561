"""Pins of the oracle's cosine-similarity closed forms and heterogeneous sparsity allocation
(appendix "Cosine similarity and heterogeneous stochastic pruning")."""
import math

import numpy as np
import pytest
from scipy import integrate

import oracle as O
import synth_inputs as SI


def truncated_lognormal(n, sigma, cutoff, seed):
    """ln|x| ~ N(0, sigma^2) conditioned on ln|x| <= cutoff, random signs (rejection sampling)."""
    rng = np.random.default_rng(seed)
    z = rng.normal(0.0, sigma, int(n * 1.3) + 1000)
    z = z[z <= cutoff][:n]
    assert z.size == n
    return (np.exp(z) * rng.choice([-1.0, 1.0], n)).astype(np.float32)


def quadrature_cosine(sigma, L, c):
    """The definitions integrated numerically in the log domain: no closed form involved."""
    pdf = lambda y: math.exp(-0.5 * (y / sigma) ** 2) / (sigma * math.sqrt(2 * math.pi))
    lo = -12 * sigma
    xx = integrate.quad(lambda y: math.exp(2 * y) * pdf(y), lo, c, limit=400)[0]              # E[x^2] = E[x T(x)]
    kept = integrate.quad(lambda y: math.exp(2 * y) * pdf(y), min(L, c), c, limit=400)[0]      # |x| > alpha
    # |x| <= alpha: T = +-alpha with probability |x| / alpha, so E[T^2 | x] = alpha |x|
    small = integrate.quad(lambda y: math.exp(L + y) * pdf(y), lo, min(L, c), limit=400)[0]
    return xx / math.sqrt(xx * (kept + small))


@pytest.mark.parametrize("sigma", [1.0, 1.5, 2.0, 3.0, 5.0])
@pytest.mark.parametrize("k", [2.0, 2.75, 4.0])
def test_cosine_closed_form_equals_quadrature_of_the_definition(sigma, k):
    c = k * sigma
    for L in (-3 * sigma, -sigma, 0.0, 0.5 * sigma, sigma, 1.5 * sigma, min(2.5 * sigma, c)):
        assert O.cosine_similarity(sigma, L, c) == pytest.approx(quadrature_cosine(sigma, L, c), rel=2e-9)


@pytest.mark.parametrize("sigma,k", [(1.5, 2.75), (2.0, 3.0), (3.0, 3.0)])
def test_cosine_closed_form_against_simulated_pruning(sigma, k):
    """Simulation as in the paper's comparison figure: prune a truncated lognormal sample with the
    stochastic operator and measure the angle."""
    c = k * sigma
    x = truncated_lognormal(1 << 22, sigma, c, seed=int(sigma * 10))
    xd = x.astype(np.float64)
    for L in (0.0, 0.8 * sigma, 1.4 * sigma):
        t = O.prune(x, math.exp(L), 1234, 0).astype(np.float64)
        measured = float(xd @ t / math.sqrt((xd @ xd) * (t @ t)))
        want = O.cosine_similarity(sigma, L, c)
        assert 1 - measured == pytest.approx(1 - want, rel=0.08, abs=2e-4), (L, measured, want)


def test_cosine_limits_and_monotonicity():
    for sigma in (1.0, 2.0, 4.0, 9.0, 14.0):
        c = 3 * sigma
        assert O.cosine_similarity(sigma, -60 * sigma, c) == pytest.approx(1.0, abs=1e-12)
        grid = np.linspace(-4 * sigma, c, 60)
        vals = [O.cosine_similarity(sigma, L, c) for L in grid]
        assert all(np.isfinite(vals)) and all(0 < v <= 1 + 1e-15 for v in vals)
        assert all(b <= a + 1e-15 for a, b in zip(vals, vals[1:]))        # more pruning, smaller cosine
    # removing the largest components lowers the similarity (the section on truncated lognormals)
    assert O.cosine_similarity(2.0, 2.0, 5.0) < O.cosine_similarity(2.0, 2.0, 8.0)


def test_threshold_for_a_minimum_cosine():
    for sigma, k, cmin in ((1.5, 2.75, 0.98), (2.0, 3.0, 0.95), (3.0, 3.0, 0.999)):
        c = k * sigma
        L = O.log_alpha_for_cosine(sigma, c, cmin)
        assert O.cosine_similarity(sigma, L, c) == pytest.approx(cmin, abs=1e-12)
        assert O.cosine_similarity(sigma, L + 1e-6, c) < cmin
    assert O.log_alpha_for_cosine(2.0, 6.0, 0.0) == 6.0                   # never binding: up to the cut-off


def test_histogram_bins_bracket_the_values():
    g = SI.lognormal_tensor(200_000, seed=4, mu=-11.0, sigma=3.0, zero_frac=0.25)
    g[:6] = [np.inf, -np.inf, np.nan, 1e-45, -3e-39, 3.4e38]
    h = O.log_histogram(g)
    a = np.abs(g[np.isfinite(g) & (g != 0)])
    assert int(h.sum()) == a.size
    # independent route: the bin is the top eleven bits of the magnitude pattern
    by_bits = np.bincount((a.view(np.uint32) >> 20).astype(np.int64), minlength=O.HIST_BINS)
    assert np.array_equal(h, by_bits.astype(np.uint64))
    # and the edges of a normal-range bin, computed as powers of two, bracket its members
    b = np.nonzero(h)[0]
    b = b[b >= 8]
    lower = 2.0 ** (b // 8 - 127.0) * (1 + (b % 8) / 8.0)
    upper = 2.0 ** ((b + 1) // 8 - 127.0) * (1 + ((b + 1) % 8) / 8.0)
    for lo, hi, cnt in zip(lower, upper, h[b]):
        assert int(np.sum((a >= lo) & (a < hi))) == int(cnt)
    bf = SI.f32_to_bf16_bits(g)
    hb = O.log_histogram(bf)
    ab = np.abs(SI.bf16_bits_to_f32(bf))
    ab = ab[np.isfinite(ab) & (ab != 0)]
    assert np.array_equal(hb, np.bincount((ab.view(np.uint32) >> 20).astype(np.int64), minlength=O.HIST_BINS).astype(np.uint64))


def test_truncation_point_from_the_histogram():
    sigma = 2.0
    g = SI.lognormal_tensor(1 << 20, seed=8, mu=-9.0, sigma=sigma, zero_frac=0.3)
    st = O.stats(g)
    k = O.truncation_k(O.log_histogram(g), st.mu, st.sigma, 0.997)
    logs = np.log(np.abs(g[g != 0]).astype(np.float64))
    exact = (np.quantile(logs, 0.997, method="inverted_cdf") - st.mu) / st.sigma
    assert abs(k - exact) <= math.log(9 / 8) / sigma                     # within one bin
    assert abs(k - 2.748) < 0.08                                          # the normal quantile: nothing is cut
    assert O.truncation_k(None, st.mu, st.sigma, 0.997) == pytest.approx(2.7477813854, rel=1e-9)
    # a sample cut at 2 sigma: the estimate sees it
    cut = g.copy()
    cut[np.abs(cut) > math.exp(-9.0 + 2.0 * sigma)] = 0
    stc = O.stats(cut)
    kc = O.truncation_k(O.log_histogram(cut), -9.0, sigma, 0.997)
    assert 1.85 < kc < 2.0


def layer_stats(seed=2):
    """Stats of twenty layers, deepest first: small late layers first, large early layers last."""
    rng = np.random.default_rng(seed)
    sizes = [256 * c * h * w for c, h, w in ([(512, 7, 7)] * 5 + [(256, 14, 14)] * 5 + [(128, 28, 28)] * 5
                                             + [(64, 56, 56)] * 4 + [(64, 112, 112)])]
    out = []
    for n in sizes:
        nnz = int(n * rng.uniform(0.4, 0.7))
        out.append(O.make_stats(n, nnz, rng.uniform(-16, -8), rng.uniform(1.2, 2.2), 1.0, 1e-30))
    return out


def test_allocation_invariants():
    stats = layer_stats()
    total = sum(s.n for s in stats)
    S = 0.9
    # no deep layers, or minima that never bind: the homogeneous scheme
    for min_cos in ([], [0.0] * 10):
        p, a = O.sparsity_allocate(stats, None, S, min_cos, 0.98)
        for st, pi, ai in zip(stats, p, a):
            ref = O.threshold(st, S)
            assert pi.alpha == ref.alpha and ai.status == 0
            assert ai.sparsity == pytest.approx(S, abs=1e-6)
    # ten deep layers with a demanding minimum: their thresholds drop, the others make up for it
    min_cos = [0.98] * 5 + [0.95] * 5
    p, a = O.sparsity_allocate(stats, None, S, min_cos, 0.98)
    lowered = [i for i in range(10) if a[i].status & 1]
    assert lowered, "the scenario must bind somewhere"
    for i in range(10):
        assert a[i].cosine >= min_cos[i] - 1e-6
        if a[i].status & 1:
            assert a[i].cosine == pytest.approx(min_cos[i], abs=1e-6)
            assert a[i].sparsity < S and p[i].alpha < O.threshold(stats[i], S).alpha
            k = a[i].k
            L = math.log(p[i].alpha) - stats[i].mu
            assert O.cosine_similarity(stats[i].sigma, L, k * stats[i].sigma) == pytest.approx(a[i].cosine, abs=1e-12)
    rest = a[10:]
    assert all(r.sparsity == pytest.approx(rest[0].sparsity, abs=1e-6) for r in rest)
    assert rest[0].sparsity > S and not any(r.status & 2 for r in rest)
    budget = sum(s.n * ai.sparsity for s, ai in zip(stats, a)) / total
    assert budget == pytest.approx(S, abs=2e-6)                            # the mean over elements is kept
    # a cap that binds: the rest sits at the cap, the budget is missed from below
    p2, a2 = O.sparsity_allocate(stats, None, S, min_cos, rest[0].sparsity - 0.004)
    assert all(r.status & 2 for r in a2[10:])
    assert all(r.sparsity == pytest.approx(rest[0].sparsity - 0.004, abs=1e-6) for r in a2[10:])
    assert sum(s.n * ai.sparsity for s, ai in zip(stats, a2)) / total < S

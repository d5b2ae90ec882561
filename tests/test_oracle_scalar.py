"""Pins for the oracle's scalar mathematics: random words, sparsity/threshold closed form,
expected relative error and the format / scale choice.  None of the expected values here comes
from the oracle itself: they are the paper's printed table, published known-answer vectors,
numerical quadrature of the defining integral, Monte-Carlo on exact lognormal samples, and
closed-form limits."""
import math
import os

import numpy as np
import pytest
from scipy import integrate, special, stats as sps

import oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------------------- random words
def _kat_rows():
    rows = []
    with open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) as fh:
        for line in fh:
            if line.strip() and not line.startswith("#"):
                v = [int(t, 16) for t in line.split()]
                rows.append((v[0:4], v[4:6], v[6:10]))
    return rows


@pytest.mark.parametrize("ctr,key,want", _kat_rows())
def test_philox_known_answers(ctr, key, want):
    assert O.philox4x32_10(ctr, key) == want


def test_random_word_layout():
    """Word of element j = output[j & 3] of the block with counter (lo(j>>2), hi(j>>2), 0, 0)."""
    seed = 0x0123456789ABCDEF
    for j in (0, 1, 2, 3, 4, 7, 12345, (1 << 34) + 5, (1 << 40) + 2):
        q = j >> 2
        blk = O.philox4x32_10([q & 0xFFFFFFFF, q >> 32, 0, 0], [seed & 0xFFFFFFFF, seed >> 32])
        assert O.random_word(seed, j) == blk[j & 3]


def test_random_words_look_uniform():
    w = np.array([O.random_word(7, j) for j in range(20000)], dtype=np.uint64)
    # the two halves of a word (pruning variable, rounding variable) are each uniform ...
    for half in (w >> 16, w & 0xFFFF):
        u = (half.astype(np.float64) + 0.5) / 2 ** 16
        assert abs(u.mean() - 0.5) < 5 * math.sqrt(1 / 12 / u.size)
        assert sps.kstest(u, "uniform").pvalue > 1e-4
    # ... and uncorrelated with each other
    a, b = (w >> 16).astype(np.float64), (w & 0xFFFF).astype(np.float64)
    assert abs(np.corrcoef(a, b)[0, 1]) < 5 / math.sqrt(w.size)
    # another seed is another stream
    w1 = np.array([O.random_word(8, j) for j in range(2000)], dtype=np.uint64)
    assert (w1 != w[:2000]).mean() > 0.99


# ---------------------------------------------------------------------- sparsity closed form
def _sparsity_by_quadrature(mu, sigma, alpha):
    """The definition: S = E_eps[ F(alpha * eps) ], F the lognormal CDF, eps ~ U[0,1]."""
    f = lambda e: sps.norm.cdf((math.log(alpha * e) - mu) / sigma) if e > 0 else 0.0
    val, _ = integrate.quad(f, 0.0, 1.0, epsabs=1e-13, epsrel=1e-13, limit=400,
                            points=[1e-9, 1e-6, 1e-3, 1e-1])
    return val


@pytest.mark.parametrize("mu,sigma", [(0.0, 1.0), (-12.0, 2.0), (-14.0, 2.5), (-20.0, 3.5),
                                      (3.0, 0.3), (-8.0, 5.5)])
@pytest.mark.parametrize("zq", [-2.5, -1.0, 0.0, 0.7, 1.5, 3.0])
def test_sparsity_closed_form_matches_definition(mu, sigma, zq):
    alpha = math.exp(mu + zq * sigma)
    want = _sparsity_by_quadrature(mu, sigma, alpha)
    got = O.sparsity_of_alpha(mu, sigma, alpha)
    assert got == pytest.approx(want, abs=2e-10)


def test_sparsity_printed_erf_form():
    """The closed form exactly as the paper prints it (with erf, no rearrangement)."""
    for mu, sigma, alpha in [(0.0, 1.0, 2.0), (-12.0, 2.0, 3e-5), (1.0, 0.5, 4.0)]:
        r = alpha / math.exp(mu)
        L = math.log(r)
        printed = 0.5 + (1 / (2 * r)) * (
            math.exp(sigma ** 2 / 2) * math.erf(sigma / math.sqrt(2) - L / (math.sqrt(2) * sigma))
            + r * math.erf(L / (math.sqrt(2) * sigma)) - math.exp(sigma ** 2 / 2))
        assert O.sparsity_of_alpha(mu, sigma, alpha) == pytest.approx(printed, abs=1e-12)


def test_sparsity_monotone_and_below_hard_threshold():
    mu, sigma = -3.0, 2.0
    prev = -1.0
    for v in np.linspace(mu - 6 * sigma, mu + 12 * sigma, 200):
        s = O.sparsity_of_alpha(mu, sigma, math.exp(v))
        assert 0.0 <= s <= 1.0
        assert s >= prev
        # stochastic pruning zeroes less than hard thresholding at the same alpha
        assert s <= sps.norm.cdf((v - mu) / sigma) + 1e-15
        prev = s
    assert O.sparsity_of_alpha(mu, sigma, math.exp(mu + 60 * sigma)) == pytest.approx(1.0, abs=1e-12)
    # extreme arguments neither overflow nor produce NaN
    for v in (mu - 40 * sigma, mu + 40 * sigma + 60):
        assert math.isfinite(O.sparsity_of_alpha(mu, sigma, math.exp(v)))
    assert math.isfinite(O.lib().orc_sparsity_of_log_alpha(0.0, 15.0, -600.0))


# --------------------------------------------------------------------------------- threshold
@pytest.mark.parametrize("mu,sigma,s", [(0.0, 1.0, 0.1), (0.0, 1.0, 0.5), (0.0, 1.0, 0.9),
                                        (-12.0, 2.0, 0.785), (-20.0, 3.5, 0.9), (-9.0, 1.5, 0.99),
                                        (-14.0, 2.5, 0.001)])
def test_threshold_inverts_definition(mu, sigma, s):
    st = O.make_stats(10 ** 6, 10 ** 6, mu, sigma)
    p = O.threshold(st, s)
    assert p.status == 0
    assert p.s_eff == pytest.approx(s, abs=1e-15)
    # alpha reproduces the asked sparsity under the defining integral (fp32 rounding of alpha
    # moves S by < 1e-7)
    assert _sparsity_by_quadrature(mu, sigma, p.alpha) == pytest.approx(s, abs=3e-7)
    assert p.s_pred == pytest.approx(_sparsity_by_quadrature(mu, sigma, p.alpha), abs=2e-10)
    # the hard-threshold quantile is a strict lower bound
    assert p.alpha > math.exp(mu + sigma * sps.norm.ppf(s))


def test_threshold_accounts_for_existing_zeros():
    """Target is the zero fraction of the whole tensor: S' = (S - l) / (1 - l)."""
    n, nnz = 1000, 700
    st = O.make_stats(n, nnz, -12.0, 2.0)
    p = O.threshold(st, 0.85)
    assert p.s_eff == pytest.approx((0.85 - 0.3) / 0.7, rel=1e-14)
    q = O.threshold(O.make_stats(nnz, nnz, -12.0, 2.0), (0.85 - 0.3) / 0.7)
    assert p.alpha == pytest.approx(q.alpha, rel=1e-6)
    # already sparse enough: nothing to prune
    z = O.threshold(st, 0.3)
    assert z.alpha == 0.0 and z.status & O.ST_NOTHING_TO_PRUNE
    z = O.threshold(st, 0.2)
    assert z.alpha == 0.0 and z.status & O.ST_NOTHING_TO_PRUNE


def test_threshold_degenerate_inputs():
    e = O.threshold(O.make_stats(100, 0, float("nan"), float("nan"), status=O.ST_EMPTY), 0.9)
    assert e.alpha == 0.0 and e.status & O.ST_EMPTY
    # point mass at c: fraction zeroed is 1 - c/alpha
    c = 3e-4
    p = O.threshold(O.make_stats(100, 100, math.log(c), 0.0, c, c, status=O.ST_SIGMA0), 0.75)
    assert p.alpha == pytest.approx(c / 0.25, rel=1e-6)
    assert p.status & O.ST_SIGMA0
    # the general formula tends to the same limit
    q = O.threshold(O.make_stats(100, 100, math.log(c), 1e-4), 0.75)
    assert q.alpha == pytest.approx(c / 0.25, rel=1e-4)


def test_threshold_bf16_rounding():
    st = O.make_stats(1000, 1000, -20.0, 3.5)
    a32 = O.threshold(st, 0.9, O.F32).alpha
    p = O.threshold(st, 0.9, O.BF16)
    bits = np.float32(p.alpha).view(np.uint32)
    assert bits & 0xFFFF == 0
    assert abs(p.alpha - a32) <= a32 * 2 ** -8
    assert p.s_pred == pytest.approx(O.sparsity_of_alpha(-20.0, 3.5, p.alpha), abs=1e-15)


def test_threshold_monte_carlo_on_exact_lognormal():
    """Apply the three-case pruning rule with fresh uniforms (plain numpy, not the oracle's
    operator) to an exact lognormal sample: the zero fraction must hit the target."""
    rng = np.random.default_rng(5)
    mu, sigma, s, n = -12.0, 2.0, 0.8, 2_000_000
    x = np.exp(mu + sigma * rng.standard_normal(n))
    alpha = O.threshold(O.make_stats(n, n, mu, sigma), s).alpha
    eps = rng.random(n)
    zeroed = np.mean(x < alpha * eps)
    assert abs(zeroed - s) < 5 * math.sqrt(s * (1 - s) / n)


def test_normal_quantile():
    for q in (1e-9, 0.003, 0.3, 0.5, 0.9, 0.997, 0.99999):
        assert O.normal_quantile(q) == pytest.approx(special.ndtri(q), abs=1e-11)


# ----------------------------------------------------------------- expected relative error
def _table2():
    rows = []
    with open(os.path.join(GOLDEN, "table2_formats.txt")) as fh:
        for line in fh:
            if line.strip() and not line.startswith("#"):
                t = line.split()
                fmts = [tuple(int(v) for v in f.split("-")) for f in t[3:8]]
                rows.append((t[0], float(t[1]), float(t[2]), fmts))
    return rows


@pytest.mark.parametrize("name,lo,hi,fmts", _table2())
def test_format_choice_reproduces_paper_table2(name, lo, hi, fmts):
    """Each row of the paper's table of ideal formats is reproduced by one sigma of its range
    (the row's upper sigma for ImageNet, sigma = 4 for Cifar100)."""
    sigma = {"Cifar100": 4.0, "ImageNet": 5.5}[name]
    assert lo <= sigma <= hi
    for n_bits, (sgn, e, m) in zip((4, 5, 6, 7, 8), fmts):
        f = O.fp_params(O.make_stats(10, 10, 0.0, sigma), n_bits)
        assert (1, f.e_bits, f.m_bits) == (sgn, e, m), (n_bits, sigma)
        assert f.n_bits == n_bits


def _eta_direct(sigma, e, m):
    """The paper's expression, summed from its three parts with scipy (2^m mantissa levels)."""
    emax = 2.0 ** (e - 1)
    p_in = 2 * sps.norm.cdf(emax / sigma) - 1
    mant = p_in / (8 * math.log(2) * 2 ** m)
    # overflow part: integral of (1 - 2^(Emax - E)) over E > Emax, E ~ N(0, sigma^2)
    over, _ = integrate.quad(lambda E: (1 - 2.0 ** (emax - E)) * sps.norm.pdf(E / sigma) / sigma,
                             emax, emax + 60 * sigma, epsabs=1e-14, epsrel=1e-12, limit=400)
    under = sps.norm.cdf(-emax / sigma)
    return mant + over + under


@pytest.mark.parametrize("sigma", [0.7, 1.0, 3.0, 5.0, 8.0])
@pytest.mark.parametrize("e,m", [(1, 6), (2, 5), (3, 2), (4, 3), (5, 2), (5, 0), (7, 0)])
def test_expected_relative_error_three_parts(sigma, e, m):
    assert O.expected_relative_error(sigma, e, m) == pytest.approx(_eta_direct(sigma, e, m),
                                                                   rel=1e-8, abs=1e-12)


def test_expected_relative_error_limits():
    # range never exceeded: only mantissa noise, 1 / (8 ln2 2^m)
    for m in range(0, 7):
        assert O.expected_relative_error(0.5, 6, m) == pytest.approx(
            1 / (8 * math.log(2) * 2 ** m), rel=1e-12)
    # range always exceeded: half the mass flushes (error 1), half saturates (error -> 1)
    assert O.expected_relative_error(1e4, 1, 3) == pytest.approx(1.0, abs=2e-3)
    # huge E_max with small sigma must not overflow
    assert math.isfinite(O.expected_relative_error(0.3, 7, 0))
    assert math.isfinite(O.expected_relative_error(50.0, 7, 0))


def test_optimal_exponent_bits_grow_with_sigma():
    for n_bits in (4, 5, 6, 7, 8):
        prev = 1
        for sigma in np.linspace(0.3, 12, 60):
            f = O.fp_params(O.make_stats(10, 10, 0.0, float(sigma)), n_bits)
            assert f.e_bits >= prev
            assert f.e_bits + f.m_bits == n_bits - 1
            etas = [O.expected_relative_error(sigma, e, n_bits - 1 - e) for e in range(1, n_bits)]
            assert f.eta == pytest.approx(min(etas), rel=1e-15)
            assert f.e_bits == 1 + int(np.argmin(etas))
            prev = f.e_bits


def test_sigma_units_and_fixed_split():
    st = O.make_stats(10, 10, -12.0, 2.0)
    a = O.fp_params(st, 6, sigma_units=O.SIGMA_BASE2)
    b = O.fp_params(O.make_stats(10, 10, -12.0, 2.0 / math.log(2)), 6)
    assert (a.e_bits, a.m_bits, a.eta) == (b.e_bits, b.m_bits, b.eta)
    f = O.fp_params(st, 6, e_bits=5)
    assert (f.e_bits, f.m_bits) == (5, 0)
    assert f.eta == pytest.approx(O.expected_relative_error(2.0, 5, 0))


# ------------------------------------------------------------------------------------ scale
def test_scale_rules():
    mu, sigma = -12.0, 2.0
    st = O.make_stats(1000, 1000, mu, sigma, max_abs=0.0811, min_abs_nz=1e-10)
    for e in (2, 3, 4, 5):
        etop = 2 ** (e - 1) - 1
        f = O.fp_params(st, 6, e_bits=e, scale_mode=O.SCALE_MAX)
        # the maximum falls in the top binade [2^(s+etop), 2^(s+etop+1))
        assert 2.0 ** (f.scale_exp + etop) <= 0.0811 < 2.0 ** (f.scale_exp + etop + 1)
        f = O.fp_params(st, 6, e_bits=e, scale_mode=O.SCALE_QUANTILE, scale_arg=0.997)
        top = math.exp(mu + sigma * special.ndtri(0.997))
        assert 2.0 ** (f.scale_exp + etop) <= top < 2.0 ** (f.scale_exp + etop + 1)
        f = O.fp_params(st, 6, e_bits=e, scale_mode=O.SCALE_CENTER)
        assert f.scale_exp == round(mu / math.log(2))
    # exact powers of two as maximum
    for k in (-20, -1, 0, 5):
        st = O.make_stats(10, 10, 0.0, 1.0, max_abs=2.0 ** k, min_abs_nz=2.0 ** k)
        assert O.fp_params(st, 8, e_bits=4, scale_mode=O.SCALE_MAX).scale_exp == k - 7
    # empty tensor
    f = O.fp_params(O.make_stats(5, 0, float("nan"), float("nan"), status=O.ST_EMPTY), 6)
    assert f.scale_exp == 0 and f.status & O.ST_EMPTY

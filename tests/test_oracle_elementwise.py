"""Pins for the oracle's per-element operators: statistics, stochastic pruning, the FP-n
quantizer, their composition and the bit packing.  Expected values are exact results on
hand-checkable tensors, exhaustive enumeration of the FP-n code table, the paper's stated
properties (unbiasedness, achieved = required sparsity, in-range relative error) and invariants.
"""
import math

import numpy as np
import pytest

import oracle as O
import synth_inputs as SI


def _f32(x):
    return np.asarray(x, dtype=np.float32)


# -------------------------------------------------------------------------------- statistics
def test_stats_powers_of_two_exact():
    """ln 2^k = k ln 2: mean and population std follow by hand; zeros are excluded."""
    ks = np.array([-20, -18, -18, -10, 3, 0, -7], dtype=np.float64)
    g = np.concatenate([2.0 ** ks * np.array([1, -1, 1, -1, 1, -1, 1]), [0.0, -0.0, 0.0]])
    st = O.stats(_f32(g))
    assert (st.n, st.nnz, st.n_nonfinite, st.status) == (10, 7, 0, 0)
    assert st.mu == pytest.approx(ks.mean() * math.log(2), rel=1e-15)
    assert st.sigma == pytest.approx(ks.std() * math.log(2), rel=1e-14)   # population (ddof=0)
    assert st.max_abs == 8.0 and st.min_abs_nz == 2.0 ** -20


def test_stats_population_not_sample_std():
    st = O.stats(_f32([1.0, math.e ** 2]))     # ln = 0, 2 -> mean 1, population std 1
    assert st.mu == pytest.approx(1.0, rel=1e-7)
    assert st.sigma == pytest.approx(1.0, rel=1e-7)


def test_stats_invariances_and_scaling():
    g = SI.lognormal_tensor(50_000, seed=11, mu=-9.0, sigma=2.2, zero_frac=0.25)
    a = O.stats(g)
    rng = np.random.default_rng(0)
    b = O.stats(rng.permutation(g))
    c = O.stats(-g)
    d = O.stats(g * np.float32(2.0 ** 7))
    for o in (b, c):
        assert o.nnz == a.nnz
        assert o.mu == pytest.approx(a.mu, rel=1e-13)
        assert o.sigma == pytest.approx(a.sigma, rel=1e-13)
    assert d.mu == pytest.approx(a.mu + 7 * math.log(2), rel=1e-13)
    assert d.sigma == pytest.approx(a.sigma, rel=1e-12)
    # against the textbook definition evaluated with numpy in float64
    nz = np.abs(g[g != 0]).astype(np.float64)
    assert a.nnz == nz.size
    assert a.mu == pytest.approx(np.log(nz).mean(), rel=1e-13)
    assert a.sigma == pytest.approx(np.log(nz).std(), rel=1e-12)


def test_stats_recovers_population_parameters():
    n, mu, sigma, z = 1 << 20, -12.0, 2.0, 0.3
    st = O.stats(SI.lognormal_tensor(n, seed=0, mu=mu, sigma=sigma, zero_frac=z))
    assert abs(st.nnz / n - (1 - z)) < 5 * math.sqrt(z * (1 - z) / n)
    assert abs(st.mu - mu) < 5 * sigma / math.sqrt(st.nnz)
    assert abs(st.sigma - sigma) < 5 * sigma / math.sqrt(2 * st.nnz)


def test_stats_special_values_and_bf16():
    g = _f32([np.inf, -np.inf, np.nan, 0.0, 1e-40, -2.0, 1e-45])     # two subnormals
    st = O.stats(g)
    assert (st.n, st.nnz, st.n_nonfinite) == (7, 3, 3)
    assert st.status & O.ST_HAS_NONFINITE
    want = np.log(np.abs(g[[4, 5, 6]]).astype(np.float64))
    assert st.mu == pytest.approx(want.mean(), rel=1e-14)
    assert st.sigma == pytest.approx(want.std(), rel=1e-14)
    assert st.max_abs == 2.0 and st.min_abs_nz == np.float32(1e-45)
    e = O.stats(_f32([0.0, -0.0]))
    assert e.nnz == 0 and e.status & O.ST_EMPTY and math.isnan(e.mu) and math.isnan(e.sigma)
    assert O.stats(_f32([])).status & O.ST_EMPTY
    s0 = O.stats(_f32([3.0, -3.0, 0.0, 3.0]))
    assert s0.sigma < 1e-15 and s0.status & O.ST_SIGMA0
    assert s0.mu == pytest.approx(math.log(3.0), rel=1e-15)
    # bf16 input is widened exactly
    x = _f32([0.5, -3.0, 0.0, 2.0 ** -130, 1.5 * 2.0 ** 100])
    hb = SI.f32_to_bf16_bits(x)
    a, b = O.stats(hb), O.stats(SI.bf16_bits_to_f32(hb))
    assert (a.nnz, a.mu, a.sigma, a.max_abs, a.min_abs_nz) == (b.nnz, b.mu, b.sigma, b.max_abs,
                                                              b.min_abs_nz)


# ----------------------------------------------------------------------- stochastic pruning
def test_prune_three_cases_by_hand():
    alpha = np.float32(1.0)
    w_of_k = lambda k: int(k) << 16           # u = (k + 1/2) / 2^16
    half = w_of_k(1 << 15)                    # u = 0.5 + 2^-17
    u_half = np.float32(0.5 + 2.0 ** -17)
    assert O.prune_one(1.5, alpha, half) == 1.5            # above: untouched
    assert O.prune_one(-1.5, alpha, half) == -1.5
    assert O.prune_one(1.0, alpha, half) == 1.0            # |x| = alpha -> sign * alpha = x
    assert O.prune_one(0.75, alpha, half) == 1.0           # alpha*u <= |x| <= alpha
    assert O.prune_one(-0.75, alpha, half) == -1.0
    assert O.prune_one(u_half, alpha, half) == 1.0         # |x| = alpha*u belongs to the middle case
    assert O.prune_one(0.5, alpha, half) == 0.0            # just below alpha*u
    assert O.prune_one(0.25, alpha, half) == 0.0           # |x| < alpha*u
    assert O.prune_one(-0.25, alpha, half) == 0.0
    # zeros stay zeros for the smallest u; the low 16 bits of the word (the rounding variable) are not used
    assert O.prune_one(0.0, alpha, 0) == 0.0
    assert O.prune_one(-0.0, alpha, 0) == 0.0 and not math.copysign(1, O.prune_one(-0.0, alpha, 0)) < 0
    assert O.prune_one(0.25, alpha, half | 0xFFFF) == 0.0
    assert O.prune_one(u_half, alpha, half | 0xFFFF) == 1.0
    assert O.prune_one(2.0 ** -17, alpha, 0) == 1.0        # smallest u = 2^-17
    assert O.prune_one(2.0 ** -18, alpha, 0) == 0.0        # u is never 0: tiny values can vanish
    assert O.prune_one(1.0 - 2.0 ** -17, alpha, 0xFFFFFFFF) == 1.0   # largest u = 1 - 2^-17
    assert O.prune_one(np.nextafter(np.float32(1.0 - 2.0 ** -17), np.float32(0)), alpha, 0xFFFFFFFF) == 0.0
    assert math.isnan(O.prune_one(float("nan"), alpha, half))
    assert O.prune_one(float("inf"), alpha, half) == float("inf")
    # alpha = 0 prunes nothing
    assert O.prune_one(1e-30, 0.0, 0xFFFFFFFF) == np.float32(1e-30)


def test_prune_threshold_product_is_single_precision():
    """alpha * u is rounded once to fp32 before the comparison."""
    alpha = np.float32(1.0 + 2.0 ** -23)
    k = (1 << 16) - 1
    u = (k + 0.5) / 2.0 ** 16
    t = np.float32(np.float64(alpha) * u)                   # exact product rounded once
    assert float(t) != float(np.float64(alpha) * u)         # the product really needs rounding
    below = np.nextafter(t, np.float32(0))
    assert O.prune_one(t, alpha, k << 16) == alpha
    assert O.prune_one(below, alpha, k << 16) == 0.0


def test_prune_outputs_sparsity_and_mean():
    cfg = SI.config_c1()
    g = SI.make(cfg)
    st = O.stats(g)
    p = O.threshold(st, cfg["sparsity"])
    y = O.prune(g, p.alpha, cfg["rng_seed"])
    a = np.abs(g)
    big = a > p.alpha
    assert np.array_equal(y[big], g[big])
    small = ~big
    assert np.all((y[small] == 0) | (np.abs(y[small]) == p.alpha))
    keep = small & (y != 0)
    assert np.array_equal(np.sign(y[keep]), np.sign(g[keep]))
    assert np.all(y[g == 0] == 0)
    # data-conditional zero count: element i is zeroed with probability 1 - |x_i|/alpha
    pz = np.where(small & (a > 0), 1.0 - a.astype(np.float64) / p.alpha, 0.0)
    new_zeros = np.count_nonzero(y == 0) - np.count_nonzero(g == 0)
    assert abs(new_zeros - pz.sum()) < 6 * math.sqrt((pz * (1 - pz)).sum())
    # achieved = required sparsity (the paper's claim), within binomial noise + estimation error
    achieved = np.mean(y == 0)
    assert abs(achieved - cfg["sparsity"]) < 6 * math.sqrt(0.85 * 0.15 / g.size) + 3 / math.sqrt(st.nnz)
    # unbiased: sum changes by a zero-mean amount with variance sum |x|(alpha-|x|)
    aa = a[small].astype(np.float64)
    var = (aa * (p.alpha - aa)).sum()
    assert abs(y.astype(np.float64).sum() - g.astype(np.float64).sum()) < 6 * math.sqrt(var)
    assert abs(np.abs(y).astype(np.float64).sum() - a.astype(np.float64).sum()) < 6 * math.sqrt(var)


def test_prune_keep_probability_exact():
    """Over ALL 2^16 grid values of u, P(keep) = |x|/alpha rounded to the grid."""
    alpha, x = np.float32(0.8), np.float32(0.3)
    kept = sum(O.prune_one(x, alpha, k << 16) != 0 for k in range(1 << 16))
    assert abs(kept - float(x) / float(alpha) * 2 ** 16) <= 1.0
    # threshold index: kept iff alpha*u <= x
    k_star = int(math.floor(float(x) / float(alpha) * 2 ** 16))
    assert O.prune_one(x, alpha, (k_star - 2) << 16) != 0
    assert O.prune_one(x, alpha, (k_star + 2) << 16) == 0


def test_prune_elem_offset_and_bf16():
    g = SI.lognormal_tensor(4099, seed=3, mu=-10, sigma=2, zero_frac=0.2)
    whole = O.prune(g, 1e-4, 99)
    parts = np.concatenate([O.prune(g[:1001], 1e-4, 99, 0), O.prune(g[1001:], 1e-4, 99, 1001)])
    assert np.array_equal(whole.view(np.uint32), parts.view(np.uint32))
    assert not np.array_equal(whole, O.prune(g, 1e-4, 100))
    hb = SI.f32_to_bf16_bits(g)
    alpha = SI.bf16_bits_to_f32(SI.f32_to_bf16_bits(_f32([1e-4])))[0]
    yb = O.prune(hb, alpha, 99)
    yf = O.prune(SI.bf16_bits_to_f32(hb), alpha, 99)
    assert np.array_equal(SI.bf16_bits_to_f32(yb), yf)


# ----------------------------------------------------------------------------- FP-n quantizer
FORMATS = [(1, 2), (2, 1), (3, 0), (1, 4), (3, 2), (4, 1), (5, 0), (4, 3), (5, 2), (7, 0), (2, 5),
           (1, 6), (1, 0), (2, 0)]


def _table(e, m, s):
    n_codes = 1 << (e + m)
    return np.array([O.decode(c, e, m, s) for c in range(n_codes)])


@pytest.mark.parametrize("e,m", FORMATS)
def test_code_table_structure(e, m):
    """Positive codes enumerate (2^e - 1) binades of 2^m values: (1 + k/2^m) 2^(c - 2^(e-1))."""
    s = -3
    emax = 2 ** (e - 1)
    t = _table(e, m, s)
    assert np.all(t[: 1 << m] == 0)                      # exponent field 0 is zero
    pos = t[1 << m:]
    assert pos.size == (2 ** e - 1) * 2 ** m
    assert np.all(np.diff(pos) > 0)                      # codes are ordered like their values
    assert pos[0] == 2.0 ** (1 - emax + s)
    assert pos[-1] == (2 - 2.0 ** -m) * 2.0 ** (emax - 1 + s)
    want = [(1 + k / 2 ** m) * 2.0 ** (c - emax + s) for c in range(1, 2 ** e) for k in range(2 ** m)]
    assert np.array_equal(pos, np.array(want))
    # sign bit
    assert O.decode((1 << (e + m)) | ((1 << m) + 1 if m else 1 << m), e, m, s) == -t[(1 << m) + (1 if m else 0)]


def test_code_table_examples_from_the_format_definition():
    t = _table(3, 2, 0)          # FP6 1-3-2: 28 positive values from 0.125 to 14
    pos = t[t > 0]
    assert pos.size == 28 and pos.min() == 0.125 and pos.max() == 14.0
    t = _table(5, 0, 0)          # FP6 1-5-0: 31 powers of two 2^-15 .. 2^15
    pos = t[t > 0]
    assert np.array_equal(pos, 2.0 ** np.arange(-15, 16))


@pytest.mark.parametrize("e,m", FORMATS)
def test_nearest_rounding_against_enumeration(e, m):
    s = -2
    t = _table(e, m, s)
    pos = t[1 << m:]
    codes_pos = np.arange(1 << m, 1 << (e + m))
    rng = np.random.default_rng(e * 16 + m)
    lo, hi = pos[0], pos[-1]
    xs = np.exp(rng.uniform(math.log(lo) - 2, math.log(hi) + 2, 4000)).astype(np.float32)
    mids = ((pos[:-1] + pos[1:]) / 2).astype(np.float32)        # exact ties
    xs = np.concatenate([xs, pos.astype(np.float32), mids, np.nextafter(mids, np.float32(0)),
                         np.nextafter(mids, np.float32(np.inf)),
                         np.nextafter(np.float32(lo), np.float32(0))[None]])
    for x in xs:
        for sgn in (1.0, -1.0):
            code = O.quantize_one(sgn * x, e, m, s)
            mag = code & ((1 << (e + m)) - 1)
            xd = float(x)
            if xd < lo:                                  # below the smallest binade: flushed
                assert code == 0
                continue
            assert (code >> (e + m)) == (1 if sgn < 0 else 0)
            if xd >= hi:
                assert mag == codes_pos[-1]
                continue
            d = np.abs(pos - xd)
            best = d.min()
            cands = codes_pos[d == best]
            if cands.size == 1:
                assert mag == cands[0], (x, e, m)
            else:                                        # tie: the even code
                assert mag in cands and mag % 2 == 0, (x, e, m)
            # idempotent
            assert O.quantize_one(sgn * t[mag], e, m, s) == code


@pytest.mark.parametrize("e,m", [(3, 2), (5, 0), (4, 3), (2, 1)])
def test_stochastic_rounding_against_enumeration(e, m):
    s = 1
    t = _table(e, m, s)
    pos = t[1 << m:]
    rng = np.random.default_rng(7)
    xs = np.exp(rng.uniform(math.log(pos[0]), math.log(pos[-1]), 60)).astype(np.float32)
    nbits = 23 - m
    for x in xs:
        xd = float(x)
        i = np.searchsorted(pos, xd, side="right") - 1
        lo_v = pos[i]
        hi_v = pos[i + 1] if i + 1 < pos.size else None
        # fraction of the way up, in units of 2^-nbits of the local spacing: exact integer
        step = 2.0 ** (math.floor(math.log2(xd)) - m)
        f = (xd - lo_v) / step * 2 ** nbits
        assert f == int(f)
        f = int(f)
        # r is the lower half of the word; up iff f / 2^nbits + (r + 1/2) / 2^16 >= 1, i.e. (exact
        # integers) iff  f * 2^17 + (2 r + 1) * 2^nbits >= 2^(nbits + 17)
        r_star = ((1 << (nbits + 17)) - f * (1 << 17) - (1 << nbits) + (1 << (nbits + 1)) - 1) >> (nbits + 1)
        for r in (0, 1, r_star - 1, r_star, r_star + 1, 0xFFFF):
            if r < 0 or r > 0xFFFF:
                continue
            w = r | 0xFFFF0000                  # the upper half (pruning variable) is not used
            val = O.decode(O.quantize_one(x, e, m, s, O.ROUND_STOCHASTIC, w), e, m, s)
            up = f * (1 << 17) + (2 * r + 1) * (1 << nbits) >= (1 << (nbits + 17))
            assert up == (r >= r_star)
            if up:
                assert val == (hi_v if hi_v is not None else pos[-1])
            else:
                assert val == lo_v
        # the up-probability over all 2^16 values of r is the cut-off fraction rounded to the grid
        ups = (1 << 16) - min(max(r_star, 0), 1 << 16)
        assert abs(ups - f / 2 ** nbits * 2 ** 16) <= 0.5
        # exactly representable values never move
        assert O.decode(O.quantize_one(np.float32(lo_v), e, m, s, O.ROUND_STOCHASTIC, 0xFFFFFFFF),
                        e, m, s) == lo_v


def test_stochastic_rounding_is_unbiased_in_range():
    e, m, s = 3, 2, -12
    rng = np.random.default_rng(3)
    x = np.exp(rng.uniform(math.log(2.0 ** -14), math.log(2.0 ** -10), 400_000)).astype(np.float32)
    q = O.fp_quantize(x, e, m, s, O.ROUND_STOCHASTIC, seed=5)
    err = (q.astype(np.float64) - x.astype(np.float64))
    spacing = 2.0 ** (np.floor(np.log2(x.astype(np.float64))) - m)
    assert abs(err.sum()) < 6 * math.sqrt((spacing ** 2 / 4).sum())
    assert np.all(np.abs(err) < spacing)
    qn = O.fp_quantize(x, e, m, s, O.ROUND_NEAREST_EVEN)
    assert np.all(np.abs(qn.astype(np.float64) - x) <= spacing / 2)


def test_quantizer_special_values_and_flush_before_rounding():
    e, m, s = 3, 2, 0          # range 0.125 .. 14
    assert O.quantize_one(0.0, e, m, s) == 0 and O.quantize_one(-0.0, e, m, s) == 0
    assert O.quantize_one(float("nan"), e, m, s) == 0b011111      # not finite: saturates like Inf
    assert O.quantize_one(float("inf"), e, m, s) == 0b011111
    assert O.quantize_one(float("-inf"), e, m, s) == 0b111111
    assert O.quantize_one(1e30, e, m, s) == 0b011111
    assert O.quantize_one(14.9, e, m, s) == 0b011111          # carry out of the top binade clamps
    assert O.quantize_one(15.9, e, m, s, O.ROUND_STOCHASTIC, 0xFFFFFFFF) == 0b011111
    just_below = np.nextafter(np.float32(0.125), np.float32(0))
    assert O.quantize_one(just_below, e, m, s) == 0          # no round-up out of the flushed zone
    assert O.quantize_one(just_below, e, m, s, O.ROUND_STOCHASTIC, 0xFFFFFFFF) == 0
    assert O.quantize_one(0.125, e, m, s) == 0b000100
    assert O.quantize_one(-0.125, e, m, s) == 0b100100
    assert O.quantize_one(1.0, e, m, s) == (4 << 2)           # E = 0 -> field 4
    # mantissa carry into the exponent: 1.9 -> 2.0
    assert O.decode(O.quantize_one(1.9, e, m, s), e, m, s) == 2.0
    # m = 0: ties go to the even exponent field
    assert O.decode(O.quantize_one(1.5, 3, 0, 0), 3, 0, 0) == 1.0     # fields 4 (even) vs 5
    assert O.decode(O.quantize_one(3.0, 3, 0, 0), 3, 0, 0) == 4.0     # fields 5 vs 6 (even)
    # subnormal fp32 inputs are ordinary numbers once the scale brings them in range
    tiny = np.float32(3 * 2.0 ** -149)
    assert O.decode(O.quantize_one(tiny, 3, 2, -148), 3, 2, -148) == 3 * 2.0 ** -149
    assert O.decode(O.quantize_one(np.float32(2.0 ** -149), 5, 0, -140), 5, 0, -140) == 2.0 ** -149


def test_in_range_relative_error_matches_the_paper_term():
    """Centred log2-normal data well inside the range: mean |x_q - x|/x = 1/(8 ln2 2^m)."""
    rng = np.random.default_rng(2)
    x = (2.0 ** (1.0 * rng.standard_normal(200_000))).astype(np.float32)
    for e, m in [(4, 1), (4, 2), (4, 3)]:
        q = O.fp_quantize(x, e, m, 0)
        rel = np.mean(np.abs(q.astype(np.float64) - x) / x)
        assert rel == pytest.approx(1 / (8 * math.log(2) * 2 ** m), rel=0.03)


def test_simulated_relative_error_tracks_the_closed_form():
    """The protocol of the paper's figure on analysis vs simulation (lognormal samples, FP8,
    sigma in {1, 3, 5}).  The closed form treats the exponent as continuous, so it is compared
    (i) with the real quantizer where clipping is rare (E_max >= 5 sigma), and (ii) everywhere
    with a Monte-Carlo of the idealisation it was derived for: saturate to 2^E_max when
    log2 x > E_max, flush when log2 x < -E_max, nearest mantissa on 2^m levels in between."""
    rng = np.random.default_rng(4)
    for sigma in (1.0, 3.0, 5.0):
        x = (2.0 ** (sigma * rng.standard_normal(200_000))).astype(np.float32)
        xd = x.astype(np.float64)
        for e in (2, 3, 4, 5, 6):
            m, emax = 7 - e, 2.0 ** (e - 1)
            eta = O.expected_relative_error(sigma, e, m)
            if emax >= 5 * sigma:
                q = O.fp_quantize(x, e, m, 0).astype(np.float64)
                assert np.mean(np.abs(q - xd) / xd) == pytest.approx(eta, rel=0.05)
            lg = np.log2(xd)
            E = np.floor(lg)
            mq = np.round((xd / 2.0 ** E - 1) * 2 ** m) / 2 ** m + 1
            ideal = np.where(lg > emax, 2.0 ** emax, np.where(lg < -emax, 0.0, mq * 2.0 ** E))
            sim = np.mean(np.abs(ideal - xd) / xd)
            assert sim == pytest.approx(eta, rel=0.04, abs=1e-3), (sigma, e)


def test_value_output_equals_decoded_codes_and_dtypes():
    g = SI.lognormal_tensor(30_000, seed=8, mu=-12, sigma=2.5, zero_frac=0.1)
    g[:3] = [np.nan, np.inf, -np.inf]
    for rounding in (O.ROUND_NEAREST_EVEN, O.ROUND_STOCHASTIC):
        codes = O.fp_quantize(g, 4, 1, -20, rounding, 17, 0, O.OUT_CODE8)
        vals = O.fp_quantize(g, 4, 1, -20, rounding, 17, 0, O.OUT_VALUE)
        deq = O.dequantize(codes, 4, 1, -20)
        assert np.isnan(vals[0]) and deq[0] == O.decode(codes[0], 4, 1, -20) and (codes[0] & 31) == 31
        assert np.array_equal(vals[1:], deq[1:])
        assert codes.max() < 64
        # bf16 input gives the same codes as its widened values
        hb = SI.f32_to_bf16_bits(g)
        cb = O.fp_quantize(hb, 4, 1, -20, rounding, 17, 0, O.OUT_CODE8)
        cf = O.fp_quantize(SI.bf16_bits_to_f32(hb), 4, 1, -20, rounding, 17, 0, O.OUT_CODE8)
        assert np.array_equal(cb, cf)
        vb = O.fp_quantize(hb, 4, 1, -20, rounding, 17, 0, O.OUT_VALUE)
        assert np.array_equal(SI.bf16_bits_to_f32(vb)[1:], O.dequantize(cb, 4, 1, -20)[1:])


# ------------------------------------------------------------------- composition and packing
@pytest.mark.parametrize("rounding", [O.ROUND_NEAREST_EVEN, O.ROUND_STOCHASTIC])
def test_fused_is_quantize_after_prune(rounding):
    cfg = SI.config_c1()
    g = SI.make(cfg, n=100_003)
    st = O.stats(g)
    p = O.threshold(st, 0.85)
    f = O.fp_params(st, 6)
    assert (f.e_bits, f.m_bits) == (3, 2)
    two = O.fp_quantize(O.prune(g, p.alpha, 5), f.e_bits, f.m_bits, f.scale_exp, rounding, 5, 0,
                        O.OUT_CODE8)
    one = O.prune_quantize(g, p.alpha, f.e_bits, f.m_bits, f.scale_exp, rounding, 5, 0, O.OUT_CODE8)
    assert np.array_equal(one, two)
    # sharding with elem_offset reproduces the whole
    cut = 40_001
    parts = np.concatenate([
        O.prune_quantize(g[:cut], p.alpha, 3, 2, f.scale_exp, rounding, 5, 0, O.OUT_CODE8),
        O.prune_quantize(g[cut:], p.alpha, 3, 2, f.scale_exp, rounding, 5, cut, O.OUT_CODE8)])
    assert np.array_equal(one, parts)
    # packed output is the packed code stream
    pk = O.prune_quantize(g, p.alpha, 3, 2, f.scale_exp, rounding, 5, 0, O.OUT_PACKED)
    assert np.array_equal(pk, O.pack(one, 6))


def test_pack_layout_by_hand():
    # three 6-bit codes 0b000001, 0b100000, 0b111111 -> bits 0, 11, 12..17
    pk = O.pack(np.array([1, 32, 63], dtype=np.uint8), 6)
    assert pk.tolist() == [0b00000001, 0b11111000, 0b00000011]
    assert O.packed_bytes(3, 6) == 3 and O.packed_bytes(0, 6) == 0 and O.packed_bytes(5, 5) == 4
    for n_bits in range(2, 9):
        rng = np.random.default_rng(n_bits)
        codes = rng.integers(0, 1 << n_bits, 1237, dtype=np.uint8)
        pk = O.pack(codes, n_bits)
        assert pk.size == (1237 * n_bits + 7) // 8
        assert np.array_equal(O.unpack(pk, 1237, n_bits), codes)
        bits = np.unpackbits(pk, bitorder="little")[: 1237 * n_bits].reshape(1237, n_bits)
        assert np.array_equal((bits * (1 << np.arange(n_bits))).sum(1), codes)


# ------------------------------------------------------------------------ stochastic underflow
def test_threshold_floor_is_the_smallest_magnitude_of_the_format():
    for e, m, s in ((3, 2, -14), (2, 1, 0), (5, 2, -30), (4, 1, 7)):
        p = O.threshold_floor(e, s)
        # the smallest non-zero code decodes to the floor
        assert p.alpha == O.decode(1 << m, e, m, s) and p.status == 16
        big = O.PruneParams(alpha=np.float32(2.0 * p.alpha), s_eff=0.5, s_pred=0.5, status=0)
        kept = O.threshold_floor(e, s, big)
        assert kept.alpha == big.alpha and kept.status == 0 and kept.s_pred == 0.5
        small = O.PruneParams(alpha=np.float32(0.25 * p.alpha), s_eff=0.5, s_pred=0.5, status=0)
        raised = O.threshold_floor(e, s, small)
        assert raised.alpha == p.alpha and raised.status == 16
    assert O.threshold_floor(3, -200).alpha == 0.0        # below the fp32 normal range: no floor


def test_stochastic_underflow_keeps_the_mean_where_flushing_loses_it():
    e, m, s = 3, 2, -10
    floor = O.threshold_floor(e, s).alpha                 # 2^-13
    n = 1 << 20
    for frac in (0.9, 0.5, 0.1, 0.01):
        x = np.full(n, frac * floor, np.float32)
        flushed = O.dequantize(O.fp_quantize(x, e, m, s, O.ROUND_STOCHASTIC, 3, 0, O.OUT_CODE8), e, m, s)
        assert np.all(flushed == 0)                       # Section 4.1: underflow goes to zero
        codes = O.prune_quantize(x, floor, e, m, s, O.ROUND_STOCHASTIC, 3, 0, O.OUT_CODE8)
        y = O.dequantize(codes, e, m, s)
        assert set(np.unique(y)) <= {0.0, np.float32(floor)}
        keep = float(np.mean(y != 0))
        assert abs(keep - frac) < 5 * math.sqrt(frac * (1 - frac) / n) + 1e-6
        assert abs(float(y.mean()) - frac * floor) < 6 * floor * math.sqrt(frac * (1 - frac) / n) + 1e-12


# --------------------------------------------------- random-variable grids, composition status
@pytest.mark.parametrize("e,m", [(4, 1), (3, 2), (5, 0)])
def test_stochastic_rounding_probability_is_exact_for_16_bit_inputs(e, m):
    """A bf16 value has 7 - m cut-off bits: over all 2^16 values of the rounding variable the number
    of round-ups is exactly (cut-off fraction) * 2^16 (brute force over the whole grid)."""
    s = -3
    for bits in (0x3E13, 0x3DFF, 0x3E80, 0x3D55, 0xBE2B):          # bf16 patterns inside the range
        x = SI.bf16_bits_to_f32(np.array([bits], np.uint16))[0]
        lo_code = O.quantize_one(x, e, m, s, O.ROUND_STOCHASTIC, 0)       # r = 0 never goes up ...
        lo_v = O.decode(lo_code, e, m, s)
        ups = sum(O.quantize_one(x, e, m, s, O.ROUND_STOCHASTIC, r) != lo_code for r in range(1 << 16))
        spacing = 2.0 ** (math.floor(math.log2(abs(float(x)))) - m)
        frac = (abs(float(x)) - abs(lo_v)) / spacing                      # exact in binary
        assert ups == frac * 2 ** 16
        if frac == 0:
            assert O.quantize_one(x, e, m, s, O.ROUND_STOCHASTIC, 0xFFFF) == lo_code


def test_pruning_and_rounding_use_disjoint_halves_of_the_word():
    """The pruning decision depends on the upper half only, the rounding decision on the lower half."""
    alpha, x = np.float32(0.8), np.float32(0.3)
    for w in (0x00000000, 0x5A5A0000, 0x60000000, 0xFFFF0000):
        assert all(O.prune_one(x, alpha, w | lo) == O.prune_one(x, alpha, w) for lo in (1, 0x8000, 0xFFFF))
    for w in (0x0000, 0x1234, 0x8000, 0xFFFF):
        assert all(O.quantize_one(0.3, 3, 2, 0, O.ROUND_STOCHASTIC, w | (hi << 16)) ==
                   O.quantize_one(0.3, 3, 2, 0, O.ROUND_STOCHASTIC, w) for hi in (1, 0x8000, 0xFFFF))


def test_alpha_below_fp_range_is_where_the_quantizer_flushes_alpha():
    """Pruning turns every survivor at or below alpha into +-alpha; the flag must be set exactly when
    the quantizer (pinned by enumeration above) sends alpha itself to code 0."""
    for e, m, s in ((3, 2, -14), (2, 1, 0), (5, 2, -30), (4, 1, 7), (1, 6, -5), (7, 0, -60)):
        edge = np.float32(2.0 ** (1 - 2 ** (e - 1) + s))           # smallest representable magnitude
        below = np.nextafter(edge, np.float32(0))
        above = np.nextafter(edge, np.float32(1e30))
        assert O.alpha_below_fp_range(below, e, s) is True
        assert O.alpha_below_fp_range(edge, e, s) is False
        assert O.alpha_below_fp_range(above, e, s) is False
        assert O.alpha_below_fp_range(0.0, e, s) is False          # no pruning: nothing to lose
        for a in (below, edge, above, np.float32(edge * 0.01), np.float32(edge * 37.0)):
            for rounding, w in ((O.ROUND_NEAREST_EVEN, 0), (O.ROUND_STOCHASTIC, 0xFFFFFFFF)):
                flushed = O.quantize_one(a, e, m, s, rounding, w) == 0
                assert flushed == O.alpha_below_fp_range(a, e, s)


def test_pruning_bias_of_the_16_bit_grid_is_bounded():
    """Averaged over ALL 2^16 values of the pruning variable, T(x) differs from x by at most
    alpha * 2^-17 (half a grid step), except below alpha * 2^-17 where an element is always dropped
    and the bias is the element itself -- the bound the design quotes for this reading."""
    alpha = np.float32(0.8)
    for x in (0.3, -0.3, 0.799, 1e-3, 0.123456, 0.5 * 0.8, 0.8 * 2.0 ** -16, 0.8 * 2.0 ** -18):
        x = np.float32(x)
        total = sum(float(O.prune_one(x, alpha, k << 16)) for k in range(1 << 16))
        mean = total / 2 ** 16
        assert abs(mean - float(x)) <= float(alpha) * 2.0 ** -17 * (1 + 1e-6), (x, mean)


def test_value_output_is_the_exact_value_rounded_to_the_type():
    """2^s q written out from the code's fields in exact arithmetic (Fraction), then rounded to the
    output type by numpy: at scales near 2^-149 the value needs more bits than an fp32 subnormal
    has, and the de-quantizer's output is the nearest fp32 (ties to even), not a truncation; the
    16-bit types round the same value once more."""
    from fractions import Fraction
    for e, m in ((1, 5), (2, 5), (3, 4), (4, 3), (1, 2)):
        nb = 1 + e + m
        codes = np.arange(1 << nb, dtype=np.uint8)
        emax = 1 << (e - 1)
        for s in (-150, -149, -148, -147, -140, -127, -20, 0, 100):
            exact = []
            for c in range(1 << nb):
                mag = c & ((1 << (e + m)) - 1)
                cexp, k = mag >> m, mag & ((1 << m) - 1)
                # exponent codes 1 .. 2^e - 1 stand for 2^(1 - emax) .. 2^(emax - 1): symmetric about 1
                v = Fraction(0) if cexp == 0 else (1 + Fraction(k, 1 << m)) * Fraction(2) ** (cexp - emax + s)
                exact.append(-v if c >> (e + m) else v)
            as_double = np.array([float(v) for v in exact])            # exact: at most 9 significant bits
            assert all(Fraction(d) == v for d, v in zip(as_double, exact))
            with np.errstate(over="ignore", under="ignore"):
                want32 = as_double.astype(np.float32)
            got32 = O.dequantize(codes, e, m, s, O.F32)
            assert np.array_equal(got32.view(np.uint32) & 0x7FFFFFFF, want32.view(np.uint32) & 0x7FFFFFFF), (e, m, s)
            assert np.array_equal(np.signbit(got32)[want32 != 0], np.signbit(want32)[want32 != 0])
            got16 = O.dequantize(codes, e, m, s, O.F16)
            with np.errstate(over="ignore", under="ignore"):
                want16 = want32.astype(np.float16)
            assert np.array_equal(got16.view(np.uint16) & 0x7FFF, want16.view(np.uint16) & 0x7FFF), (e, m, s)

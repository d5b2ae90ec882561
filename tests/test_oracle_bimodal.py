"""Pins of the oracle's masked statistics and of the bi-modal pruning procedure (appendix
"Algorithm for bi-Modal lognormal pruning"): the numpy definition on the selected entries, step 2's
S' = (S - l) / (1 - l), and the paper's claim that the required sparsity is achieved for S >= 0.7
and undershot below."""
import math

import numpy as np
import pytest

import oracle as O
import synth_inputs as SI


def pair(n=1 << 20, left_frac=0.6, dtype=SI.F32, seed=21):
    return SI.bimodal_pair(n, seed=seed, left_frac=left_frac, mu_right=-9.0, sigma_right=2.0,
                           mu_left=-16.0, sigma_left=1.2, dtype=dtype)


@pytest.mark.parametrize("dtype", [SI.F32, SI.BF16])
def test_masked_statistics_are_the_numpy_definition_on_the_selection(dtype):
    x, m = pair(1 << 18, dtype=dtype)
    xv = x if dtype == SI.F32 else SI.bf16_bits_to_f32(x)
    mv = m if dtype == SI.F32 else SI.bf16_bits_to_f32(m)
    sel = (mv != 0) & (xv != 0)
    logs = np.log(np.abs(xv[sel].astype(np.float64)))
    st = O.stats_masked(x, m)
    assert st.n == x.size and st.nnz == int(sel.sum())
    assert st.mu == pytest.approx(float(logs.mean()), rel=1e-12)
    assert st.sigma == pytest.approx(float(logs.std()), rel=1e-11)
    assert np.float32(st.max_abs) == np.abs(xv[sel]).max() and np.float32(st.min_abs_nz) == np.abs(xv[sel]).min()
    # a byte mask selecting the same entries gives the same numbers; an all-ones mask is plain stats
    st8 = O.stats_masked(x, (mv != 0).astype(np.uint8))
    assert bytes(st8) == bytes(st)
    assert bytes(O.stats_masked(x, np.ones(x.size, np.uint8))) == bytes(O.stats(x))
    # the right mode's parameters are recovered, the left mode's are not mixed in
    assert abs(st.mu + 9.0) < 0.02 and abs(st.sigma - 2.0) < 0.02
    assert abs(O.stats(x).mu + 9.0) > 3.0


def test_masked_statistics_special_entries():
    x = np.array([1.0, np.nan, 0.0, -4.0, np.inf, 16.0, 2.0], np.float32)
    m = np.array([1.0, 1.0, 1.0, -0.0, 0.0, np.nan, 3.0], np.float32)   # -0 is zero, NaN is not
    st = O.stats_masked(x, m)
    # fit: 1.0, 16.0, 2.0; the NaN of x is counted, its zero skipped, -4 and inf are masked out
    assert (st.n, st.nnz, st.n_nonfinite) == (7, 3, 1)
    logs = np.log([1.0, 16.0, 2.0])
    assert st.mu == pytest.approx(logs.mean(), rel=1e-14) and st.sigma == pytest.approx(logs.std(), rel=1e-14)
    assert (st.max_abs, st.min_abs_nz) == (16.0, 1.0)
    none = O.stats_masked(x, np.zeros(7, np.uint8))
    assert none.nnz == 0 and none.status & O.ST_EMPTY


def test_step_two_is_the_zero_credit():
    x, m = pair()
    st = O.stats_masked(x, m)
    l = 1.0 - st.nnz / st.n
    for s in (0.7, 0.8, 0.9, 0.97):
        p = O.threshold(st, s)
        assert p.s_eff == pytest.approx((s - l) / (1.0 - l), rel=1e-12)


@pytest.mark.parametrize("left_frac", [0.5, 0.8])
def test_required_sparsity_is_achieved_above_and_undershot_below(left_frac):
    """Prune the WHOLE tensor with the threshold of the right mode."""
    x, m = pair(left_frac=left_frac)
    st = O.stats_masked(x, m)
    achieved = {}
    for s in (left_frac + 0.03, 0.9, 0.97):
        p = O.threshold(st, s)
        y = O.prune(x, p.alpha, 99, 0)
        achieved[s] = float(np.mean(y == 0))
        assert achieved[s] <= s + 2e-3                       # never more than asked for
    # high sparsity: accurate (left-mode values are far below alpha * eps and all go)
    assert abs(achieved[0.97] - 0.97) < 2e-3
    assert abs(achieved[0.9] - 0.9) < 4e-3
    # barely above the left fraction: alpha is small, part of the left mode survives
    low = left_frac + 0.03
    assert achieved[low] < low - 2e-3

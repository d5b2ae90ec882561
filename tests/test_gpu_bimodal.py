"""Parity of the masked statistics (right mode of a bi-modal gradient) with the oracle, and the
bi-modal pruning procedure end to end on the device."""
import math

import numpy as np
import pytest

import oracle as O
import synth_inputs as SI

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lgn():
    import paper_2006_08173_amd as m
    m.load()
    return m


def to_dev(a: np.ndarray):
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda()
    return torch.from_numpy(a).cuda()


def assert_stats_match(got, want, rel=1e-6):
    assert (got.n, got.nnz, got.n_nonfinite, got.status) == (want.n, want.nnz, want.n_nonfinite, want.status)
    assert np.float32(got.max_abs) == np.float32(want.max_abs)
    assert np.float32(got.min_abs_nz) == np.float32(want.min_abs_nz)
    if want.nnz == 0:
        assert math.isnan(got.mu) and math.isnan(got.sigma)
        return
    assert abs(got.mu - want.mu) <= rel * abs(want.mu) + 1e-12
    assert abs(got.sigma - want.sigma) <= rel * want.sigma + 1e-12


def pair(n, dtype, seed=31, left_frac=0.6):
    return SI.bimodal_pair(n, seed=seed, left_frac=left_frac, mu_right=-9.0, sigma_right=2.0,
                           mu_left=-16.0, sigma_left=1.2, dtype=dtype)


@pytest.mark.parametrize("dtype", [SI.F32, SI.BF16])
@pytest.mark.parametrize("byte_mask", [False, True])
def test_masked_stats_parity_sizes(lgn, dtype, byte_mask):
    for n in (0, 1, 3, 5, 255, 257, 1023, 4099, 262_147, 2_000_003):
        x, m = pair(n, dtype, seed=31 + n % 13)
        if n > 40:                                        # special entries on both sides
            xf = x.view(np.uint32 if dtype == SI.F32 else np.uint16)
            mf = m.view(np.uint32 if dtype == SI.F32 else np.uint16)
            nan, inf, negz = (0x7FC00000, 0x7F800000, 0x80000000) if dtype == SI.F32 else (0x7FC0, 0x7F80, 0x8000)
            xf[3], mf[3] = nan, mf[3] | 1                 # NaN inside the fit: counted as non-finite
            xf[5], mf[5] = inf, 0                         # Inf outside the fit: ignored
            mf[7] = negz                                  # -0 in the mask is a zero
            mf[9] = nan                                   # NaN in the mask is not
            xf[11] = 1                                    # subnormal value
        if byte_mask:
            mv = m if dtype == SI.F32 else SI.bf16_bits_to_f32(m)
            with np.errstate(invalid="ignore"):
                m = (~(mv == 0)).astype(np.uint8) * np.uint8(1 + n % 200)
        want = O.stats_masked(x, m)
        got = lgn.read_stats(lgn.lgn_stats_masked(to_dev(x), to_dev(m)))
        assert_stats_match(got, want)
        st, _, _ = lgn.lgn_stats_solve(to_dev(x), mask=to_dev(m))
        assert bytes(lgn.read_stats(st)) == bytes(got), n  # the one-launch form gives the same bits


def test_mask_argument_errors(lgn):
    x = torch.zeros(1024, device="cuda")
    with pytest.raises(ValueError):
        lgn.lgn_stats_masked(x, torch.zeros(1000, device="cuda"))
    with pytest.raises(TypeError):
        lgn.lgn_stats_masked(x, torch.zeros(1024, dtype=torch.bfloat16, device="cuda"))
    with pytest.raises(lgn.LgnError):
        lgn.lgn_stats_masked(x, torch.zeros(1040, dtype=torch.uint8, device="cuda")[1:1025])  # misaligned


@pytest.mark.parametrize("left_frac", [0.5, 0.8])
def test_bimodal_pruning_on_device(lgn, left_frac):
    """Appendix "Algorithm for bi-Modal lognormal pruning", steps 1-4 with nothing leaving the device:
    fit the right mode, credit the left mode, prune the whole tensor."""
    n = 1 << 22
    x, m = pair(n, SI.F32, seed=77, left_frac=left_frac)
    dx, dm = to_dev(x), to_dev(m)
    ost = O.stats_masked(x, m)
    for s in (0.9, 0.97):
        st, p, _ = lgn.lgn_stats_solve(dx, s, mask=dm)
        hs, hp = lgn.read_stats(st), lgn.read_prune_params(p)
        assert_stats_match(hs, ost)
        same_in = O.make_stats(hs.n, hs.nnz, hs.mu, hs.sigma, hs.max_abs, hs.min_abs_nz, hs.n_nonfinite, hs.status)
        want_p = O.threshold(same_in, s)
        assert np.float32(hp.alpha) == np.float32(want_p.alpha)
        l = 1.0 - hs.nnz / hs.n
        assert hp.s_eff == pytest.approx((s - l) / (1 - l), rel=1e-12)
        y = lgn.lgn_prune(dx, p, 4242, 0).cpu().numpy()
        assert np.array_equal(y.view(np.uint32), O.prune(x, hp.alpha, 4242, 0).view(np.uint32))
        achieved = float(np.mean(y == 0))
        assert abs(achieved - s) < 4e-3                   # "very accurate above 0.7"

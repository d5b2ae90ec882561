"""Parity of every entry point on half-precision (fp16) tensors with the oracle."""
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


def dev(a):
    return torch.from_numpy(a).cuda()


def u16(a):
    return a.view(np.uint16)


SPECIALS = np.array([0, 0x8000, 0x7C00, 0xFC00, 0x7E00, 0x0001, 0x8001, 0x03FF, 0x0400, 0x7BFF, 0xFBFF, 0x3C00,
                     0xBC00, 0x0200], dtype=np.uint16).view(np.float16)   # zeros, inf, nan, subnormals, extremes


def tensor(n, seed, mu=-7.0, sigma=2.0, zero_frac=0.3):
    g = SI.lognormal_tensor(n, seed=seed, mu=mu, sigma=sigma, zero_frac=zero_frac, dtype=SI.F16)
    k = min(n, SPECIALS.size)
    if k:
        g[np.random.default_rng(seed).choice(n, k, replace=False)] = SPECIALS[:k]
    return g


def stats_match(got, want, rel=1e-6):
    assert (got.n, got.nnz, got.n_nonfinite, got.status) == (want.n, want.nnz, want.n_nonfinite, want.status)
    assert np.float32(got.max_abs) == np.float32(want.max_abs)
    assert np.float32(got.min_abs_nz) == np.float32(want.min_abs_nz)
    if want.nnz:
        assert abs(got.mu - want.mu) <= rel * abs(want.mu) + 1e-12
        assert abs(got.sigma - want.sigma) <= rel * want.sigma + 1e-12


def test_stats_threshold_histogram(lgn):
    for n in (0, 1, 7, 8, 9, 511, 4099, 262_147, 3_000_001):
        g = tensor(n, 70 + n % 17)
        d = dev(g)
        hs = lgn.read_stats(lgn.lgn_stats(d))
        stats_match(hs, O.stats(g))
        assert np.array_equal(lgn.lgn_log_histogram(d).cpu().numpy().view(np.uint64), O.log_histogram(g))
        if hs.nnz:
            same_in = O.make_stats(hs.n, hs.nnz, hs.mu, hs.sigma, hs.max_abs, hs.min_abs_nz, hs.n_nonfinite, hs.status)
            st, p, f = lgn.lgn_stats_solve(d, 0.8, lgn.LGN_F16, 6)
            hp = lgn.read_prune_params(p)
            want = O.threshold(same_in, 0.8, O.F16)
            assert np.float32(hp.alpha) == np.float32(want.alpha)
            assert np.float32(hp.alpha) == np.float32(np.float16(hp.alpha))       # a half-precision value
    # masks: a half tensor of its own type, and bytes
    x, m = SI.bimodal_pair(500_003, seed=5, left_frac=0.6, mu_right=-5.0, sigma_right=1.5, mu_left=-11.0,
                           sigma_left=1.0, dtype=SI.F16)
    stats_match(lgn.read_stats(lgn.lgn_stats_masked(dev(x), dev(m))), O.stats_masked(x, m))
    bm = (m != 0).astype(np.uint8)
    stats_match(lgn.read_stats(lgn.lgn_stats_masked(dev(x), dev(bm))), O.stats_masked(x, bm))


def test_prune_quantize_fused(lgn):
    alpha = float(np.float16(2.5e-4))
    p = lgn.upload_struct(lgn.LgnPruneParams(alpha, 0, 0.0, 0.0))
    for n in (0, 1, 3, 4, 5, 255, 257, 1023, 4099, 300_001):
        g = tensor(n, 20 + n % 13)
        d = dev(g)
        for off in (0, 8, 3):
            y = lgn.lgn_prune(d, p, 11, off).cpu().numpy()
            assert np.array_equal(u16(y), u16(O.prune(g, alpha, 11, off))), (n, off)
        for e, m, s in ((3, 2, -12), (5, 2, -17), (2, 1, -9), (4, 3, -14)):
            f = lgn.upload_struct(lgn.LgnFpParams(1 + e + m, e, m, s, 0.0, 0, 0))
            for rounding in (O.ROUND_NEAREST_EVEN, O.ROUND_STOCHASTIC):
                want = O.prune_quantize(g, alpha, e, m, s, rounding, 11, 0, O.OUT_CODE8)
                got = lgn.lgn_prune_quantize_fused(d, p, f, rounding, 11, 0, out_kind=O.OUT_CODE8).cpu().numpy()
                assert np.array_equal(got, want), (n, e, m, rounding)
                qw = O.fp_quantize(g, e, m, s, rounding, 11, 0, O.OUT_CODE8)
                qg = lgn.lgn_fp_quantize(d, f, rounding, 11, 0, out_kind=O.OUT_CODE8).cpu().numpy()
                assert np.array_equal(qg, qw)
                pk = lgn.lgn_prune_quantize_fused(d, p, f, rounding, 11, 0, out_kind=O.OUT_PACKED,
                                                  n_bits=1 + e + m).cpu().numpy()
                assert np.array_equal(pk, O.pack(want, 1 + e + m))
            # values: 2^s q rounded to half precision (exact here except below the half subnormal range)
            vw = O.fp_quantize(g, e, m, s, O.ROUND_NEAREST_EVEN, 0, 0, O.OUT_VALUE)
            vg = lgn.lgn_fp_quantize(d, f, O.ROUND_NEAREST_EVEN, 0, 0, out_kind=O.OUT_VALUE).cpu().numpy()
            assert np.array_equal(u16(vg), u16(vw)), (n, e, m, s)
            codes = O.fp_quantize(g, e, m, s, O.ROUND_NEAREST_EVEN, 0, 0, O.OUT_CODE8)
            deq = lgn.lgn_dequantize(dev(codes), n, O.OUT_CODE8, f, lgn.LGN_F16).cpu().numpy()
            assert np.array_equal(u16(deq), u16(O.dequantize(codes, e, m, s, O.F16)))


def test_prefix_code_of_half_values(lgn):
    alpha = float(np.float16(2.5e-4))
    p = lgn.upload_struct(lgn.LgnPruneParams(alpha, 0, 0.0, 0.0))
    g = tensor(3 * 4096 + 77, 3)
    y = O.prune(g, alpha, 5, 0)
    d = dev(y)
    buf, table = lgn.lgn_prefix_encode(d, lgn.LGN_OUT_VALUE, p)
    nchunks = 4
    t = table.cpu().numpy().view(np.uint64)[: nchunks + 2]
    want, wt = O.prefix_encode(y, O.prefix_special_of_alpha(alpha, 16, fp16=True))
    assert np.array_equal(t, wt)
    assert np.array_equal(buf.cpu().numpy()[: int(t[-2]) * 4], want)
    back = lgn.lgn_prefix_decode(buf, table, y.size, lgn.LGN_OUT_VALUE, p, dtype=lgn.LGN_F16).cpu().numpy()
    assert np.array_equal(u16(back), u16(y))
    assert int(np.sum(np.abs(y) == np.float16(alpha))) > 100     # the special class is in use


def test_chain_on_half_tensor(lgn):
    g = SI.lognormal_tensor(1 << 20, seed=44, mu=-6.0, sigma=1.8, zero_frac=0.3, dtype=SI.F16)
    d = dev(g)
    st, p, f = lgn.lgn_stats_solve(d, 0.85, lgn.LGN_F16, 6)
    hs, hp, hf = lgn.read_stats(st), lgn.read_prune_params(p), lgn.read_fp_params(f)
    stats_match(hs, O.stats(g))
    codes = lgn.lgn_prune_quantize_fused(d, p, f, O.ROUND_STOCHASTIC, 8, 0, out_kind=O.OUT_CODE8).cpu().numpy()
    want = O.prune_quantize(g, hp.alpha, hf.e_bits, hf.m_bits, hf.scale_exp, O.ROUND_STOCHASTIC, 8, 0, O.OUT_CODE8)
    assert np.array_equal(codes, want)
    achieved = float(np.mean((codes & 0x1F) == 0))
    assert abs(achieved - 0.85) < 6 * math.sqrt(0.85 * 0.15 / g.size) + 3 / math.sqrt(hs.nnz) + 2e-3

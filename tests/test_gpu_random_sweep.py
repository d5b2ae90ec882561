"""Seeded random sweep of the streaming entry points: every argument drawn at random within its
documented range (size, element type, threshold, format, scale, rounding, seed, element offset,
output kind), the result compared bit for bit with the CPU oracle.  The fixed grids of the other
parity files cover the corners; this one covers combinations nobody thought of.
LGN_SWEEP_SEED (environment, an integer) moves every sweep to other draws."""
import os

import numpy as np
import pytest

import oracle as O
import synth_inputs as SI

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

SEED_SHIFT = 1_000_003 * int(os.environ.get("LGN_SWEEP_SEED", "0"))


@pytest.fixture(scope="module")
def lgn():
    import paper_2006_08173_amd as m
    m.load()
    return m


def to_dev(a):
    return torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).cuda()


def raw(t, like):
    a = t.cpu().numpy()
    if like.dtype == np.uint16:
        return a.view(np.uint16)
    if like.dtype == np.float16:
        return a.view(np.uint16)
    return a.view(np.uint32) if a.dtype == np.float32 else a


def alpha_in_dtype(alpha, dtype):
    """A threshold that is a value of the tensor's element type (as lgn_threshold would produce)."""
    if dtype == SI.BF16:
        return float(SI.bf16_bits_to_f32(SI.f32_to_bf16_bits(np.float32([alpha])))[0])
    if dtype == SI.F16:
        return float(np.float16(alpha))
    return float(np.float32(alpha))


def draw_case(rng):
    dtype = (SI.F32, SI.BF16, SI.F16)[int(rng.integers(0, 3))]
    n = int(rng.choice([rng.integers(1, 600), rng.integers(600, 70_000), rng.integers(70_000, 400_000)]))
    mu = float(rng.uniform(-14.0, -4.0)) if dtype != SI.F16 else float(rng.uniform(-9.0, -3.0))
    sigma = float(rng.uniform(0.3, 3.0))
    g = SI.lognormal_tensor(n, seed=int(rng.integers(0, 1 << 30)), mu=mu, sigma=sigma,
                            zero_frac=float(rng.uniform(0.0, 0.6)), dtype=dtype)
    nb = int(rng.integers(2, 9))
    e = int(rng.integers(1, nb))
    m = nb - 1 - e
    # scale so that the bulk of the tensor lands inside, below or above the format's range
    s = int(round(mu / np.log(2.0))) + int(rng.integers(-6, 7)) - (1 << (e - 1)) // 2
    alpha = alpha_in_dtype(float(np.exp(mu + sigma * rng.uniform(-1.5, 2.5))), dtype) if rng.random() < 0.9 else 0.0
    rounding = int(rng.integers(0, 2))
    seed = int(rng.integers(0, 1 << 62))
    offset = int(rng.choice([0, 4 * rng.integers(0, 1 << 40), rng.integers(0, 1 << 34),
                             (1 << 34) - 4 * rng.integers(1, 2000)]))   # aligned, unaligned, near a counter carry
    return dtype, g, alpha, e, m, s, rounding, seed, offset


def test_random_sweep_of_the_streaming_calls(lgn):
    rng = np.random.default_rng(777 + SEED_SHIFT)
    lgn_dtype = {SI.F32: lgn.LGN_F32, SI.BF16: lgn.LGN_BF16, SI.F16: lgn.LGN_F16}
    for case in range(160):
        dtype, g, alpha, e, m, s, rounding, seed, offset = draw_case(rng)
        ctx = (case, dtype, g.size, alpha, e, m, s, rounding, seed, offset)
        d = to_dev(g)
        if dtype == SI.F16:
            d = d.view(torch.float16) if d.dtype != torch.float16 else d
        p = lgn.upload_struct(lgn.LgnPruneParams(alpha, 0, 0.0, 0.0))
        f = lgn.upload_struct(lgn.LgnFpParams(1 + e + m, e, m, s, 0.0, 0, 0))
        kind = (O.OUT_CODE8, O.OUT_PACKED, O.OUT_VALUE)[case % 3]
        want = O.prune_quantize(g, alpha, e, m, s, rounding, seed, offset, kind)
        got = lgn.lgn_prune_quantize_fused(d, p, f, rounding, seed, offset, out_kind=kind, n_bits=1 + e + m,
                                           dtype=lgn_dtype[dtype])
        if kind == O.OUT_VALUE:
            assert np.array_equal(raw(got, g), raw(_as_tensor(want), g)), ctx
        else:
            assert np.array_equal(got.cpu().numpy(), want), ctx
        # the two halves of the composition, every third case each
        if case % 3 == 0:
            wantp = O.prune(g, alpha, seed, offset)
            gotp = lgn.lgn_prune(d, p, seed, offset, dtype=lgn_dtype[dtype])
            assert np.array_equal(raw(gotp, g), raw(_as_tensor(wantp), g)), ctx
        elif case % 3 == 1:
            wantq = O.fp_quantize(g, e, m, s, rounding, seed, offset, O.OUT_CODE8)
            gotq = lgn.lgn_fp_quantize(d, f, rounding, seed, offset, out_kind=O.OUT_CODE8, dtype=lgn_dtype[dtype])
            assert np.array_equal(gotq.cpu().numpy(), wantq), ctx


class _as_tensor:
    """numpy array wrapped so that raw() can treat oracle output like a device result."""

    def __init__(self, a):
        self.a = a

    def cpu(self):
        return self

    def numpy(self):
        return self.a


def test_random_sweep_of_statistics_and_parameters(lgn):
    """Random sizes, element types, zero shares, special values and masks: counts and extrema exact,
    mu and sigma to 1e-6; then threshold and format from the device's own statistics: the oracle's
    bits for alpha, its (e, m, s)."""
    import math
    rng = np.random.default_rng(4242 + SEED_SHIFT)
    lgn_dtype = {SI.F32: lgn.LGN_F32, SI.BF16: lgn.LGN_BF16, SI.F16: lgn.LGN_F16}
    odt = {SI.F32: O.F32, SI.BF16: O.BF16, SI.F16: O.F16}
    for case in range(70):
        dtype = (SI.F32, SI.BF16, SI.F16)[case % 3]
        n = int(rng.choice([rng.integers(1, 3000), rng.integers(3000, 300_000), rng.integers(300_000, 3_000_000)]))
        mu = float(rng.uniform(-14.0, -4.0)) if dtype != SI.F16 else float(rng.uniform(-9.0, -3.0))
        sigma = float(rng.uniform(0.2, 3.0))
        g = SI.lognormal_tensor(n, seed=int(rng.integers(0, 1 << 30)), mu=mu, sigma=sigma,
                                zero_frac=float(rng.uniform(0.0, 0.7)), dtype=dtype)
        if n > 50 and dtype != SI.F16 and rng.random() < 0.5:      # a few special bit patterns
            v = g.view(np.uint32 if dtype == SI.F32 else np.uint16)
            pos = rng.choice(n, 6, replace=False)
            pats = (0x7FC00000, 0xFF800000, 0x00000001, 0x807FFFFF, 0x80000000, 0x7F7FFFFF) if dtype == SI.F32 \
                else (0x7FC0, 0xFF80, 0x0001, 0x807F, 0x8000, 0x7F7F)
            v[pos] = pats
        d = to_dev(g)
        mode = case % 4
        if mode == 0:
            mask = (rng.random(n) < 0.6).astype(np.uint8)
            want = O.stats_masked(g, mask)
            st = lgn.lgn_stats_masked(d, torch.from_numpy(mask).cuda(), dtype=lgn_dtype[dtype])
        elif mode == 1:
            mask = g.copy()
            mask.view(np.uint16 if dtype != SI.F32 else np.uint32)[rng.random(n) < 0.4] = 0
            want = O.stats_masked(g, mask)
            st = lgn.lgn_stats_masked(d, to_dev(mask), dtype=lgn_dtype[dtype])
        else:
            want = O.stats(g)
            st = lgn.lgn_stats(d, dtype=lgn_dtype[dtype])
        got = lgn.read_stats(st)
        ctx = (case, dtype, n, mode)
        assert (got.n, got.nnz, got.n_nonfinite, got.status) == (want.n, want.nnz, want.n_nonfinite, want.status), ctx
        assert np.float32(got.max_abs) == np.float32(want.max_abs), ctx
        assert np.float32(got.min_abs_nz) == np.float32(want.min_abs_nz), ctx
        if want.nnz == 0:
            assert math.isnan(got.mu) and math.isnan(got.sigma), ctx
            continue
        assert abs(got.mu - want.mu) <= 1e-6 * abs(want.mu) + 1e-12, ctx
        assert abs(got.sigma - want.sigma) <= 1e-6 * want.sigma + 1e-12, ctx
        # parameters from identical inputs: the device's statistics handed to the oracle
        same = O.make_stats(got.n, got.nnz, got.mu, got.sigma, got.max_abs, got.min_abs_nz, got.n_nonfinite, got.status)
        target = float(rng.uniform(0.05, 0.99))
        nb = int(rng.integers(2, 9))
        wp, wf = O.threshold(same, target, odt[dtype]), O.fp_params(same, nb)
        gp = lgn.read_prune_params(lgn.lgn_threshold(st, target, lgn_dtype[dtype]))
        gf = lgn.read_fp_params(lgn.lgn_fp_params(st, nb))
        assert np.float32(gp.alpha).view(np.uint32) == np.float32(wp.alpha).view(np.uint32), ctx
        assert gp.status == wp.status, ctx
        assert (gf.e_bits, gf.m_bits, gf.scale_exp, gf.status) == (wf.e_bits, wf.m_bits, wf.scale_exp, wf.status), ctx


SPECIAL_PATTERNS = {SI.F32: (0x7FC00000, 0xFF800000, 0x7F800000, 0x00000001, 0x807FFFFF, 0x80000000, 0x7F7FFFFF, 0x00800000),
                    SI.BF16: (0x7FC0, 0xFF80, 0x7F80, 0x0001, 0x807F, 0x8000, 0x7F7F, 0x0080),
                    SI.F16: (0x7E00, 0xFC00, 0x7C00, 0x0001, 0x83FF, 0x8000, 0x7BFF, 0x0400)}


def test_random_sweep_over_the_whole_parameter_range(lgn):
    """As the first sweep, but nothing is kept near the tensor's own scale: magnitudes from the
    bottom to the top of the element type, scales from -150 to 125, thresholds anywhere in fp32,
    NaN / Inf / subnormal / extreme patterns planted, all three output kinds and the two halves
    of the composition for every case."""
    rng = np.random.default_rng(8 + SEED_SHIFT)
    lgn_dtype = {SI.F32: lgn.LGN_F32, SI.BF16: lgn.LGN_BF16, SI.F16: lgn.LGN_F16}
    with np.errstate(over="ignore"):
        for case in range(200):
            dtype = (SI.F32, SI.BF16, SI.F16)[int(rng.integers(0, 3))]
            n = int(rng.choice([rng.integers(1, 600), rng.integers(600, 9000), rng.integers(9000, 200_000)]))
            lim = 9.0 if dtype == SI.F16 else 80.0
            mu, sigma = float(rng.uniform(-lim, lim * 0.9)), float(rng.uniform(0.1, 6.0))
            g = SI.lognormal_tensor(n, seed=int(rng.integers(0, 1 << 30)), mu=mu, sigma=sigma,
                                    zero_frac=float(rng.uniform(0, 0.6)), dtype=dtype)
            if n > 20:
                g.view(np.uint32 if dtype == SI.F32 else np.uint16)[rng.choice(n, 8, replace=False)] = SPECIAL_PATTERNS[dtype]
            nb = int(rng.integers(2, 9))
            e = int(rng.integers(1, nb))
            m = nb - 1 - e
            s = int(rng.integers(-150, 126))
            if rng.random() < 0.5:
                s = max(-150, min(125, int(round(mu / np.log(2.0))) + int(rng.integers(-12, 13))))
            a = float(np.float32(np.exp(rng.uniform(-103.0, 88.0)))) if rng.random() < 0.5 \
                else float(np.float32(np.exp(mu + sigma * rng.uniform(-2, 3))))
            a = alpha_in_dtype(min(a, 60000.0) if dtype == SI.F16 else a, dtype)
            if not np.isfinite(a) or rng.random() < 0.08:
                a = 0.0
            rounding, seed = int(rng.integers(0, 2)), int(rng.integers(0, 1 << 63))
            offset = int(rng.choice([0, 4 * rng.integers(0, 1 << 40), rng.integers(0, 1 << 34),
                                     (1 << 34) - 4 * rng.integers(1, 2000), (1 << 34) - rng.integers(1, 300)]))
            ctx = (case, dtype, n, a, e, m, s, rounding, seed, offset)
            d = to_dev(g)
            p = lgn.upload_struct(lgn.LgnPruneParams(a, 0, 0.0, 0.0))
            f = lgn.upload_struct(lgn.LgnFpParams(nb, e, m, s, 0.0, 0, 0))
            for kind in (O.OUT_CODE8, O.OUT_PACKED, O.OUT_VALUE):
                want = O.prune_quantize(g, a, e, m, s, rounding, seed, offset, kind)
                got = lgn.lgn_prune_quantize_fused(d, p, f, rounding, seed, offset, out_kind=kind, n_bits=nb,
                                                   dtype=lgn_dtype[dtype])
                if kind == O.OUT_VALUE:
                    assert np.array_equal(raw(got, g), raw(_as_tensor(want), g)), (kind,) + ctx
                else:
                    assert np.array_equal(got.cpu().numpy(), want), (kind,) + ctx
            gotp = lgn.lgn_prune(d, p, seed, offset, dtype=lgn_dtype[dtype])
            assert np.array_equal(raw(gotp, g), raw(_as_tensor(O.prune(g, a, seed, offset)), g)), ctx
            gotq = lgn.lgn_fp_quantize(d, f, rounding, seed, offset, out_kind=O.OUT_PACKED, n_bits=nb, dtype=lgn_dtype[dtype])
            assert np.array_equal(gotq.cpu().numpy(), O.fp_quantize(g, e, m, s, rounding, seed, offset, O.OUT_PACKED)), ctx


def test_random_sweep_of_statistics_over_the_whole_range(lgn):
    """Statistics of tensors anywhere in the element type's range, spreads from 0.05 to 9, a stretch
    of a very different magnitude somewhere, special patterns, all mask kinds: counts and extrema
    exact, mu and sigma to 1e-6 of max(|mu|, sigma) and of sigma (mu may be near zero here)."""
    rng = np.random.default_rng(3 + SEED_SHIFT)
    code = {SI.F32: lgn.LGN_F32, SI.BF16: lgn.LGN_BF16, SI.F16: lgn.LGN_F16}
    with np.errstate(over="ignore"):
        for case in range(150):
            dtype = (SI.F32, SI.BF16, SI.F16)[case % 3]
            n = int(rng.choice([rng.integers(1, 3000), rng.integers(3000, 300_000), rng.integers(300_000, 2_000_000)]))
            lim = 10.0 if dtype == SI.F16 else 86.0
            mu = float(rng.uniform(-lim, lim))
            sigma = float(rng.choice([rng.uniform(0.05, 0.5), rng.uniform(0.5, 3.0), rng.uniform(3.0, 9.0)]))
            g = SI.lognormal_tensor(n, seed=int(rng.integers(0, 1 << 30)), mu=mu, sigma=sigma,
                                    zero_frac=float(rng.uniform(0.0, 0.7)), dtype=dtype)
            if rng.random() < 0.3 and n > 600:
                at = int(rng.integers(0, n - 500))
                length = int(rng.integers(1, min(n - at, 200_000)))
                g[at:at + length] = SI.lognormal_tensor(length, seed=int(rng.integers(0, 1 << 30)), mu=float(rng.uniform(-lim, lim)),
                                                        sigma=0.3, zero_frac=0.0, dtype=dtype)
            if n > 50 and rng.random() < 0.5:
                g.view(np.uint32 if dtype == SI.F32 else np.uint16)[rng.choice(n, 8, replace=False)] = SPECIAL_PATTERNS[dtype]
            d = to_dev(g)
            mode = int(rng.integers(0, 3))
            if mode == 0:
                mask = (rng.random(n) < 0.6).astype(np.uint8)
                want, st = O.stats_masked(g, mask), lgn.lgn_stats_masked(d, torch.from_numpy(mask).cuda(), dtype=code[dtype])
            elif mode == 1:
                mask = g.copy()
                mask.view(np.uint16 if dtype != SI.F32 else np.uint32)[rng.random(n) < 0.4] = 0
                want, st = O.stats_masked(g, mask), lgn.lgn_stats_masked(d, to_dev(mask), dtype=code[dtype])
            else:
                want, st = O.stats(g), lgn.lgn_stats(d, dtype=code[dtype])
            got = lgn.read_stats(st)
            ctx = (case, dtype, n, mode, mu, sigma)
            assert (got.n, got.nnz, got.n_nonfinite, got.status) == (want.n, want.nnz, want.n_nonfinite, want.status), ctx
            assert np.float32(got.max_abs) == np.float32(want.max_abs), ctx
            assert np.float32(got.min_abs_nz) == np.float32(want.min_abs_nz), ctx
            if want.nnz == 0:
                continue
            assert abs(got.mu - want.mu) <= 1e-6 * max(abs(want.mu), want.sigma) + 1e-12, ctx
            assert abs(got.sigma - want.sigma) <= 1e-6 * want.sigma + 1e-12, ctx

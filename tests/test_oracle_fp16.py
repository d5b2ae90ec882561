"""Pins of the oracle's half-precision element access: its value-domain conversions against numpy's
float16 (an independent IEEE implementation), and the element operators on fp16 tensors against
the same operators on the exactly equal fp32 tensors."""
import numpy as np
import pytest

import oracle as O
import synth_inputs as SI


def test_half_to_float_is_exact_for_every_pattern():
    h = np.arange(65536, dtype=np.uint16)
    got = np.array([O.f16_to_float(int(x)) for x in h], dtype=np.float32)
    ref = h.view(np.float16).astype(np.float32)
    nan = np.isnan(ref)
    assert np.all(np.isnan(got[nan]))
    assert np.array_equal(got.view(np.uint32)[~nan], ref.view(np.uint32)[~nan])


def test_float_to_half_rounds_to_nearest_even():
    rng = np.random.default_rng(0)
    halves = np.arange(65536, dtype=np.uint16).view(np.float16).astype(np.float32)
    halves = halves[~np.isnan(halves)]
    mids = ((halves[:-1].astype(np.float64) + halves[1:].astype(np.float64)) / 2).astype(np.float32)  # ties
    mids = mids[np.isfinite(mids)]
    x = np.concatenate([
        rng.standard_normal(100_000).astype(np.float32) * np.float32(10) ** rng.integers(-9, 6, 100_000).astype(np.float32),
        halves, mids, np.nextafter(mids, np.float32(np.inf)), np.nextafter(mids, np.float32(-np.inf)),
        np.float32([65504, 65519.99, 65520, 65536, 1e9, -1e9, 5.96e-8, 2.98e-8, 2.9802322e-8, 2.9802326e-8, 0, -0.0])])
    got = np.array([O.float_to_f16(v) for v in x], dtype=np.uint16)
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    assert np.array_equal(got, want)
    assert O.float_to_f16(np.nan) & 0x7C00 == 0x7C00 and O.float_to_f16(np.nan) & 0x3FF


def test_operators_on_fp16_equal_operators_on_the_same_values_in_fp32():
    g16 = SI.lognormal_tensor(100_000, seed=9, mu=-7.0, sigma=2.0, zero_frac=0.3, dtype=SI.F16)
    g16[:4] = np.float16([6e-8, -6.1e-5, 65504, -2e-7])           # subnormals and the largest value
    g32 = g16.astype(np.float32)
    a, b = O.stats(g16), O.stats(g32)
    assert bytes(a) == bytes(b)
    alpha = float(np.float16(3e-4))
    y16, y32 = O.prune(g16, alpha, 5, 0), O.prune(g32, alpha, 5, 0)
    assert np.array_equal(y16.astype(np.float32), y32)            # every output value is a half already
    for rounding in (O.ROUND_NEAREST_EVEN, O.ROUND_STOCHASTIC):
        c16 = O.prune_quantize(g16, alpha, 3, 2, -12, rounding, 5, 0, O.OUT_CODE8)
        c32 = O.prune_quantize(g32, alpha, 3, 2, -12, rounding, 5, 0, O.OUT_CODE8)
        assert np.array_equal(c16, c32)
    v16 = O.fp_quantize(g16, 3, 2, -12, O.ROUND_NEAREST_EVEN, 0, 0, O.OUT_VALUE)
    v32 = O.fp_quantize(g32, 3, 2, -12, O.ROUND_NEAREST_EVEN, 0, 0, O.OUT_VALUE)
    assert v16.dtype == np.float16 and np.array_equal(v16, v32.astype(np.float16))
    # alpha is rounded to half precision and saturates at the largest finite half
    st = O.make_stats(1000, 1000, -7.0, 2.0, 1.0, 1e-7)
    p = O.threshold(st, 0.8, O.F16)
    assert np.float32(p.alpha) == np.float32(np.float16(p.alpha))
    huge = O.make_stats(1000, 1000, 30.0, 1.0, 1.0, 1e-7)
    assert O.threshold(huge, 0.9, O.F16).alpha == 65504.0

"""Seeded synthetic neural-gradient tensors.

This module only draws random numbers and shapes them into tensors; it holds none of the
compression method's arithmetic.  Both the CPU oracle's tests and the HIP path's tests and
benchmark take their inputs from here, so the two sides always see the same bytes.

The tensors follow the paper's model of a neural gradient (Section "Neural gradients
distribution"): magnitudes are lognormal, signs are symmetric, and a fraction of the entries is
exactly zero (the ReLU mask described in the appendix on gradient histograms).  They stand in
for the ImageNet / CIFAR ResNet gradients the paper measures on, which are not available here.

Element recipe.  With independent draws b0, b1 ~ U[0,1) and Z ~ N(0,1):

    g = 0                                   if b0 < zero_frac
    g = (-1 if b1 < 0.5 else +1) * exp(mu + sigma * Z)   otherwise      (computed in fp64)

then rounded to the tensor dtype (fp64 -> fp32 by IEEE round-to-nearest; bf16 is that fp32 value
rounded to nearest-even on its upper 16 bits).  Optionally a fraction `outlier_frac` of the
entries is replaced by values with |g| log-uniform in `outlier_range`, and a fraction `tiny_frac`
by values with |g| log-uniform in `tiny_range` (used to reach the bf16 subnormal range).

Generation is chunked: chunk c of CHUNK elements uses numpy's counter-based Philox bit generator
keyed by (seed, c), so any slice of a tensor can be produced without producing the rest.
bf16 tensors are returned as numpy uint16 bit patterns.
"""
from __future__ import annotations

import concurrent.futures as _cf
import os as _os

import numpy as np

CHUNK = 1 << 20

F32 = "f32"
BF16 = "bf16"
F16 = "f16"


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to bf16 (nearest, ties to even); returns uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    nan = (b & 0x7FFFFFFF) > 0x7F800000
    r = ((b + (0x7FFF + ((b >> 16) & 1))) >> 16).astype(np.uint16)
    if nan.any():
        r[nan] = ((b[nan] >> 16) | 0x0040).astype(np.uint16)
    return r


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to fp32 exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def _chunk(c, lo, hi, seed, mu, sigma, zero_frac, dtype, outlier_frac, outlier_range,
           tiny_frac, tiny_range):
    """Elements [lo, hi) of chunk c (indices relative to the chunk start)."""
    rng = np.random.Generator(np.random.Philox(key=[int(seed), int(c)]))
    b0 = rng.random(CHUNK)
    b1 = rng.random(CHUNK)
    z = rng.standard_normal(CHUNK)
    mag = np.exp(mu + sigma * z)
    if outlier_frac > 0.0 or tiny_frac > 0.0:
        b2 = rng.random(CHUNK)
        b3 = rng.random(CHUNK)
        if outlier_frac > 0.0:
            sel = b2 < outlier_frac
            l0, l1 = np.log(outlier_range[0]), np.log(outlier_range[1])
            mag[sel] = np.exp(l0 + (l1 - l0) * b3[sel])
        if tiny_frac > 0.0:
            sel = (b2 >= outlier_frac) & (b2 < outlier_frac + tiny_frac)
            l0, l1 = np.log(tiny_range[0]), np.log(tiny_range[1])
            mag[sel] = np.exp(l0 + (l1 - l0) * b3[sel])
    g = np.where(b1 < 0.5, -mag, mag)
    g[b0 < zero_frac] = 0.0
    g32 = g[lo:hi].astype(np.float32)
    if dtype == BF16:
        return f32_to_bf16_bits(g32)
    if dtype == F16:
        return g32.astype(np.float16)
    return g32


def lognormal_tensor(n, *, seed, mu, sigma, zero_frac=0.0, dtype=F32, start=0,
                     outlier_frac=0.0, outlier_range=(1e2, 1e4),
                     tiny_frac=0.0, tiny_range=(2.0 ** -133, 2.0 ** -120), workers=None):
    """Elements [start, start+n) of the seeded synthetic tensor (flat, contiguous).

    Returns float32 for dtype 'f32', uint16 bit patterns for dtype 'bf16', float16 for 'f16'.
    """
    n = int(n)
    start = int(start)
    out = np.empty(n, dtype={F32: np.float32, BF16: np.uint16, F16: np.float16}[dtype])
    if n == 0:
        return out
    first, last = start // CHUNK, (start + n - 1) // CHUNK
    jobs = []
    for c in range(first, last + 1):
        lo = max(start, c * CHUNK) - c * CHUNK
        hi = min(start + n, (c + 1) * CHUNK) - c * CHUNK
        jobs.append((c, lo, hi))

    def run(job):
        c, lo, hi = job
        part = _chunk(c, lo, hi, seed, mu, sigma, zero_frac, dtype, outlier_frac, outlier_range,
                      tiny_frac, tiny_range)
        o = c * CHUNK + lo - start
        out[o:o + (hi - lo)] = part

    if workers is None:
        workers = min(8, _os.cpu_count() or 1)
    if len(jobs) == 1 or workers <= 1:
        for j in jobs:
            run(j)
    else:
        with _cf.ThreadPoolExecutor(max_workers=workers) as ex:
            list(ex.map(run, jobs))
    return out


def bimodal_pair(n, *, seed, left_frac, mu_right, sigma_right, mu_left, sigma_left, dtype=F32):
    """A pre-batch-norm style gradient and the post-batch-norm gradient that splits it in two modes.

    Returns (x, m).  m is a ReLU-masked lognormal tensor: a fraction `left_frac` of exact zeros.  x is
    dense: lognormal(mu_left, sigma_left) where m is zero (the left mode, orders of magnitude
    smaller) and lognormal(mu_right, sigma_right) elsewhere, symmetric signs.
    """
    m = lognormal_tensor(n, seed=seed, mu=mu_right, sigma=sigma_right, zero_frac=left_frac, dtype=dtype)
    right = lognormal_tensor(n, seed=seed + 101, mu=mu_right, sigma=sigma_right, dtype=dtype)
    left = lognormal_tensor(n, seed=seed + 202, mu=mu_left, sigma=sigma_left, dtype=dtype)
    x = np.where(m == 0, left, right)
    return x, m


# ---------------------------------------------------------------------------------------------
# The five benchmark configurations (sizes, distributions and work).
# `seed` is the data seed; `rng_seed` keys the random words the pruning / rounding steps draw.
# ---------------------------------------------------------------------------------------------

def config_c1():
    """2^20 fp32 elements, 30 % zeros, ln|g| ~ N(-12, 2^2); prune to 0.85, then FP6."""
    return dict(name="c1", n=1 << 20, dtype=F32, seed=0, mu=-12.0, sigma=2.0, zero_frac=0.30,
                sparsity=0.85, n_bits=6, rng_seed=1001)


def config_c2():
    """256x64x56x56 fp32, 50 % zeros, ln|g| ~ N(-14, 2.5^2); prune at four sparsities."""
    return dict(name="c2", n=256 * 64 * 56 * 56, dtype=F32, seed=1, mu=-14.0, sigma=2.5,
                zero_frac=0.50, sparsities=(0.5, 0.7, 0.85, 0.9), rng_seed=1002)


# Conv-output shapes (C, H, W) of an ImageNet ResNet-18 at batch 256, with multiplicities.
_RESNET18_SHAPES = ([(64, 112, 112)] + [(64, 56, 56)] * 4 + [(128, 28, 28)] * 5
                    + [(256, 14, 14)] * 5 + [(512, 7, 7)] * 5)


def config_c3():
    """20 tensors with ResNet-18 activation-gradient shapes at batch 256.

    Per tensor mu ~ U(-16,-8), sigma ~ U(1.5,3), target sparsity ~ U(0.6,0.95), all drawn from
    seed 2; 50 % zeros; FP6 with the closed-form split.
    """
    rng = np.random.Generator(np.random.Philox(key=[2, 0xC3]))
    tensors = []
    for i, (c, h, w) in enumerate(_RESNET18_SHAPES):
        tensors.append(dict(name=f"c3.{i}", n=256 * c * h * w, dtype=F32, seed=2000 + i,
                            mu=float(rng.uniform(-16, -8)), sigma=float(rng.uniform(1.5, 3.0)),
                            zero_frac=0.5, sparsity=float(rng.uniform(0.6, 0.95)), n_bits=6,
                            rng_seed=1003))
    return tensors


def config_c4():
    """256x256x56x56 fp32 (205.5 M), 40 % zeros, ln|g| ~ N(-13, 2^2); FP-n sweep and headline."""
    return dict(name="c4", n=256 * 256 * 56 * 56, dtype=F32, seed=3, mu=-13.0, sigma=2.0,
                zero_frac=0.40, sparsity=0.85, n_bits=6, rng_seed=1004,
                formats=[(nb, e) for nb in (4, 5, 6, 8) for e in range(1, nb)])


def config_c5(n=1_000_000_000):
    """Flat bf16 tensor, ln|g| ~ N(-20, 3.5^2), 0.01 % outliers and 0.01 % bf16-subnormal-range
    values; prune at 0.9, FP6, packed 6-bit codes."""
    return dict(name="c5", n=n, dtype=BF16, seed=4, mu=-20.0, sigma=3.5, zero_frac=0.0,
                outlier_frac=1e-4, tiny_frac=1e-4, sparsity=0.9, n_bits=6, rng_seed=1005)


def make(cfg, n=None, start=0, workers=None):
    """Materialise (a slice of) the tensor a config dict describes."""
    kw = dict(seed=cfg["seed"], mu=cfg["mu"], sigma=cfg["sigma"], zero_frac=cfg["zero_frac"],
              dtype=cfg["dtype"], start=start, workers=workers)
    for k in ("outlier_frac", "tiny_frac"):
        if k in cfg:
            kw[k] = cfg[k]
    return lognormal_tensor(cfg["n"] if n is None else n, **kw)

// Device code of lgn_threshold and lgn_fp_params: the closed-form parameter choices, evaluated on the device in
// fp64 by one wave each, so that the chain stats -> parameters -> streaming pass needs no host
// round trip.
//
//   threshold (Section 5.1-5.2 and Appendix "From sparsity to the threshold"):
//       S(alpha) = Phi(L/sigma) - exp(sigma^2/2 - L) Phi((L - sigma^2)/sigma),  L = ln(alpha) - mu,
//     which is the printed closed form with erf(a) - 1 written as -erfc(a).  S is increasing in
//     v = ln(alpha); dS/dv equals the second term B and d2S/dv2 = -B + phi(L/sigma)/sigma, so a
//     third-order (Halley) step costs one more exponential.  The iteration is safeguarded by a
//     bracket and falls back to bisection when a step leaves it.
//   format (Section 4.2-4.3): expected relative error of FP(1,e,m) for every e in [1, N-1], one
//     lane per candidate, then an arg-min across lanes (ties to the smaller e).
//   scale (Section 4.4, Alg. 1, Appendix "Neural gradients lognormal distributions are truncated").
#pragma once

#include "lgn_device.hpp"

namespace lgn {

constexpr double kSqrt2 = 1.41421356237309504880168872421;
constexpr double kLn2 = 0.693147180559945309417232121458;

__device__ __forceinline__ double normal_cdf(double z) { return 0.5 * erfc(-z / kSqrt2); }

// Standard normal quantile: a rational first guess (Abramowitz & Stegun 26.2.23, |error| < 5e-4)
// polished by Newton steps on the tail probability, which keeps full relative accuracy in both
// tails.
__device__ double normal_quantile(double q)
{
    const bool upper = q > 0.5;
    const double p = upper ? 1.0 - q : q;  // tail probability, p <= 0.5
    if (!(p > 0.0)) return upper ? 40.0 : -40.0;
    const double t = sqrt(-2.0 * log(p));
    double z = t - (2.515517 + 0.802853 * t + 0.010328 * t * t) /
                       (1.0 + 1.432788 * t + 0.189269 * t * t + 0.001308 * t * t * t);
    // z >= 0 is the distance into the tail: solve Q(z) = p with Q the upper tail probability
    for (int it = 0; it < 8; ++it) {
        const double qz = 0.5 * erfc(z / kSqrt2);
        const double pdf = exp(-0.5 * z * z) * 0.398942280401432677939946059934;
        const double step = (qz - p) / pdf;
        z += step;
        if (fabs(step) <= 1e-16 * fmax(1.0, fabs(z))) break;
    }
    return upper ? z : -z;
}

// Rational first guess of the standard normal quantile alone (|error| < 4.5e-4).
__device__ __forceinline__ double normal_quantile_guess(double q)
{
    const bool upper = q > 0.5;
    const double p = upper ? 1.0 - q : q;
    if (!(p > 0.0)) return upper ? 40.0 : -40.0;
    const double t = sqrt(-2.0 * log(p));
    const double z = t - (2.515517 + 0.802853 * t + 0.010328 * t * t) /
                             (1.0 + 1.432788 * t + 0.189269 * t * t + 0.001308 * t * t * t);
    return upper ? z : -z;
}

// S(v) and its derivative B(v) = dS/dv.
__device__ __forceinline__ void sparsity_terms(double mu, double sigma, double v, double &S, double &B)
{
    const double L = v - mu;
    const double A = 0.5 * erfc(-L / (kSqrt2 * sigma));
    const double tail = erfc((sigma * sigma - L) / (kSqrt2 * sigma));
    B = tail > 0.0 ? 0.5 * exp(0.5 * sigma * sigma - L + log(tail)) : 0.0;
    S = A - B;
}

// Second derivative of S given B: the derivative of the second term of S is -B + phi(L/sigma)/sigma
// (the exponents of its two factors add up to -L^2 / (2 sigma^2)).
__device__ __forceinline__ double sparsity_curvature(double mu, double sigma, double v, double B)
{
    const double a = (v - mu) / sigma;
    return exp(-0.5 * a * a) * (0.398942280401432677939946059934 / sigma) - B;
}

__device__ __forceinline__ float round_to_bf16(float f)
{
    uint32_t b = __float_as_uint(f);
    b += 0x7fffu + ((b >> 16) & 1u);
    b &= 0xffff0000u;
    if ((b & 0x7fffffffu) >= 0x7f800000u) b = (b & 0x80000000u) | 0x7f7f0000u;
    return __uint_as_float(b);
}

// fp32 -> fp16 -> fp32, round to nearest even, saturating at the largest finite fp16 value.
__device__ __forceinline__ float round_to_f16(float f)
{
    const float r = (float)(_Float16)f;
    if (r > 65504.0f) return 65504.0f;
    if (r < -65504.0f) return -65504.0f;
    return r;
}

// alpha rounded to the element type of the tensor it will be compared with and stored into
__device__ __forceinline__ float round_alpha(float alpha, int alpha_dtype)
{
    if (alpha_dtype == LGN_BF16) return round_to_bf16(alpha);
    if (alpha_dtype == LGN_F16) return round_to_f16(alpha);
    return alpha;
}

// Runs in one lane (the caller picks it); `st` may point to LDS or global memory.
__device__ __forceinline__ void threshold_body(const lgn_stats_t *st, double target, int alpha_dtype,
                                               lgn_prune_params_t *out)
{
    lgn_prune_params_t r;
    r.alpha = 0.0f;
    r.s_eff = 0.0;
    r.s_pred = 0.0;
    r.status = st->status & (LGN_ST_EMPTY | LGN_ST_SIGMA0 | LGN_ST_HAS_NONFINITE);
    const uint64_t nn = st->n, nz = st->nnz;
    if (nz == 0) {
        *out = r;
        return;
    }
    const double n = (double)nn, nnz = (double)nz;
    const double s_eff = (target * n - (n - nnz)) / nnz;
    r.s_eff = s_eff;
    if (!(s_eff > 0.0)) {
        r.status |= LGN_ST_NOTHING_TO_PRUNE;
        *out = r;
        return;
    }
    const double mu = st->mu, sigma = st->sigma;
    double v;
    const bool point_mass = sigma < 1e-12;
    if (point_mass) {
        v = mu - log1p(-s_eff);
        r.status |= LGN_ST_SIGMA0;
    } else {
        // Bracket: stochastic pruning zeroes less than a hard threshold at the same alpha, so the
        // lognormal quantile of s_eff is a lower bound of the root; the unpolished guess of the
        // normal quantile, lowered by more than its error, is enough for that.
        double lo = mu + sigma * (normal_quantile_guess(s_eff) - 1e-3), hi = lo, S, B;
        double step = sigma;
        bool ok = false;
        for (int i = 0; i < 64; ++i) {
            hi += step;
            step *= 2.0;
            sparsity_terms(mu, sigma, hi, S, B);
            if (S > s_eff) { ok = true; break; }
            lo = hi;
        }
        if (!ok) r.status |= LGN_ST_NOT_CONVERGED;
        v = 0.5 * (lo + hi);
        bool converged = false;
        for (int it = 0; it < 200 && ok; ++it) {
            sparsity_terms(mu, sigma, v, S, B);
            const double f = S - s_eff;
            if (f < 0.0) lo = v; else hi = v;
            double nv = 0.5 * (lo + hi);
            bool third_order = false;
            if (B > 0.0) {
                const double den = 2.0 * B * B - f * sparsity_curvature(mu, sigma, v, B);
                const double h = v - 2.0 * f * B / den;
                if (h > lo && h < hi) { nv = h; third_order = true; }
            }
            // a third-order step of size d leaves an error of order d^3: below 3e-6 that is under
            // one unit in the last place of v, so no further evaluation is needed
            const double d = fabs(nv - v), scale = fmax(1.0, fabs(nv));
            const bool done = (third_order && d <= 3e-6 * scale) || d <= 1e-15 * scale ||
                              hi - lo <= 1e-15 * scale;
            v = nv;
            if (done) { converged = true; break; }
        }
        if (ok && !converged) r.status |= LGN_ST_NOT_CONVERGED;
    }
    const double alpha = exp(v);
    float af = alpha >= 3.4028234663852886e38 ? 3.4028234663852886e38f : (float)alpha;
    af = round_alpha(af, alpha_dtype);
    r.alpha = af;
    if (af > 0.0f) {
        if (point_mass) {
            r.s_pred = fmax(0.0, 1.0 - exp(mu) / (double)af);
        } else {
            double S, B;
            sparsity_terms(mu, sigma, log((double)af), S, B);
            r.s_pred = S;
        }
    }
    *out = r;
}

// Expected relative error of FP(1,e,m) on lognormal data (Section 4.2, final expression; 2^m
// mantissa levels).  The saturation term 2^(E_max-1) e^{sigma^2 ln^2 2 / 2} (erf(z) - 1) is formed
// in the log domain so that a huge power of two times a vanishing erfc stays finite.
__device__ double expected_relative_error(double sigma, int e_bits, int m_bits)
{
    const double emax = ldexp(1.0, e_bits - 1);
    const double phi = normal_cdf(emax / sigma);
    const double mantissa = (2.0 * phi - 1.0) / (8.0 * kLn2 * ldexp(1.0, m_bits));
    const double z = sigma * kLn2 / kSqrt2 + emax / (kSqrt2 * sigma);
    const double tail = erfc(z);
    const double over =
        tail > 0.0 ? -exp((emax - 1.0) * kLn2 + 0.5 * sigma * sigma * kLn2 * kLn2 + log(tail)) : 0.0;
    return mantissa + over - 0.5 * erf(emax / (kSqrt2 * sigma)) + 1.5 - phi;
}

// Runs in all 64 lanes of one wave; `st` may point to LDS or global memory.
__device__ __forceinline__ void fp_params_body(const lgn_stats_t *st, int n_bits, int e_fixed,
                                               int scale_mode, double scale_arg, int sigma_units,
                                               lgn_fp_params_t *out)
{
    const int lane = threadIdx.x & (kWave - 1);
    const uint64_t nnz = st->nnz;
    const double mu = st->mu, sigma = st->sigma;
    const bool spread = nnz != 0 && sigma >= 1e-12;
    const double sg = sigma_units == LGN_SIGMA_BASE2 ? sigma / kLn2 : sigma;

    // one candidate exponent width per lane
    const int cand = lane + 1;
    double eta = __builtin_inf();
    if (spread && cand <= n_bits - 1 && (e_fixed < 1 || cand == e_fixed))
        eta = expected_relative_error(sg, cand, n_bits - 1 - cand);
    // lane 63 meanwhile evaluates the quantile the scale rule needs
    double zq = 0.0;
    if (lane == kWave - 1 && nnz != 0 && scale_mode == LGN_SCALE_QUANTILE) zq = normal_quantile(scale_arg);
    zq = __shfl(zq, kWave - 1);

    double best = eta;
    int best_e = cand;
#pragma unroll
    for (int off = 1; off < 8; off <<= 1) {  // candidates live in lanes 0..6
        const double o = __shfl_xor(best, off);
        const int oe = __shfl_xor(best_e, off);
        if (o < best || (o == best && oe < best_e)) { best = o; best_e = oe; }
    }
    if (lane != 0) return;

    lgn_fp_params_t r;
    r.n_bits = n_bits;
    r.status = st->status & (LGN_ST_EMPTY | LGN_ST_SIGMA0 | LGN_ST_HAS_NONFINITE);
    r.reserved = 0u;
    int e;
    if (e_fixed >= 1) {
        e = e_fixed;
        r.eta = spread ? best : 0.0;
    } else if (!spread) {
        e = 1;
        r.eta = 0.0;
    } else {
        e = best_e;
        r.eta = best;
    }
    r.e_bits = e;
    r.m_bits = n_bits - 1 - e;
    const int etop = (1 << (e - 1)) - 1;
    int s = 0;
    if (nnz != 0) {
        if (scale_mode == LGN_SCALE_MAX) {
            // floor(log2 max|g|) straight from the bit pattern (subnormals normalised)
            const uint32_t a = __float_as_uint(st->max_abs) & 0x7fffffffu;
            int ex = (int)(a >> 23) - 127;
            if ((a >> 23) == 0u) ex = -126 - (__clz(a & 0x7fffffu) - 8);
            s = ex - etop;
        } else if (scale_mode == LGN_SCALE_CENTER) {
            s = (int)floor(mu / kLn2 + 0.5);
        } else {
            s = (int)floor((mu + zq * sigma) / kLn2) - etop;
        }
    }
    r.scale_exp = s;
    *out = r;
}

}  // namespace lgn

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

// S(v), its derivative B(v) = dS/dv and its second derivative C(v).  The second derivative of the
// second term of S is -B + phi(L/sigma)/sigma (the exponents of its two factors add up to
// -L^2 / (2 sigma^2)).
//
// COOP = false: an ordinary per-lane function.  COOP = true: called by all lanes of a wave, the two
// lanes of a pair (2p, 2p+1) with the same arguments.  The chain of one evaluation is
// erfc -> log -> exp; the two erfc calls and the two exp calls are independent of each other, so
// the even and the odd lane of a pair take one each and swap the values: the same operations on
// the same operands as the per-lane form, in three transcendental latencies instead of five.
template <bool COOP>
__device__ __forceinline__ void sparsity_terms(double mu, double sigma, double v, double &S, double &B,
                                               double &C)
{
    const double L = v - mu;
    const double a = L / sigma;
    const double za = -L / (kSqrt2 * sigma), zb = (sigma * sigma - L) / (kSqrt2 * sigma);
    const double xb = -0.5 * a * a;  // exponent of the density term
    double A, tail, eb, ec;
    if (COOP) {
        const bool odd = (threadIdx.x & 1u) != 0u;
        const double e = erfc(odd ? zb : za), e_other = __shfl_xor(e, 1);
        A = 0.5 * (odd ? e_other : e);
        tail = odd ? e : e_other;
        const double x = exp(odd ? xb : 0.5 * sigma * sigma - L + (tail > 0.0 ? log(tail) : 0.0));
        const double x_other = __shfl_xor(x, 1);
        eb = odd ? x_other : x;
        ec = odd ? x : x_other;
    } else {
        A = 0.5 * erfc(za);
        tail = erfc(zb);
        eb = exp(0.5 * sigma * sigma - L + (tail > 0.0 ? log(tail) : 0.0));
        ec = exp(xb);
    }
    B = tail > 0.0 ? 0.5 * eb : 0.0;
    C = ec * (0.398942280401432677939946059934 / sigma) - B;
    S = A - B;
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

// COOP = false: runs in one lane (the caller picks it).  COOP = true: runs in all lanes of one wave,
// every lane with the same values, and lane 0 stores the result.  `st` may point to LDS or global
// memory.
template <bool COOP>
__device__ __forceinline__ void threshold_body(const lgn_stats_t *st, double target, int alpha_dtype,
                                               lgn_prune_params_t *out)
{
    lgn_prune_params_t r;
    r.alpha = 0.0f;
    r.s_eff = 0.0;
    r.s_pred = 0.0;
    r.status = st->status & (LGN_ST_EMPTY | LGN_ST_SIGMA0 | LGN_ST_HAS_NONFINITE);
    const uint64_t nn = st->n, nz = st->nnz;
    const bool writer = !COOP || (threadIdx.x & (kWave - 1)) == 0;
    if (nz == 0) {
        if (writer) *out = r;
        return;
    }
    const double n = (double)nn, nnz = (double)nz;
    const double s_eff = (target * n - (n - nnz)) / nnz;
    r.s_eff = s_eff;
    if (!(s_eff > 0.0)) {
        r.status |= LGN_ST_NOTHING_TO_PRUNE;
        if (writer) *out = r;
        return;
    }
    const double mu = st->mu, sigma = st->sigma;
    double v;
    double v_at = 0.0, S_at = 0.0, B_at = 0.0, C_at = 0.0;  // last point evaluated; S, S', S'' there
    bool evaluated = false;
    const bool point_mass = sigma < 1e-12;
    if (point_mass) {
        v = mu - log1p(-s_eff);
        r.status |= LGN_ST_SIGMA0;
    } else {
        // Bracket: stochastic pruning zeroes less than a hard threshold at the same alpha, so the
        // lognormal quantile of s_eff is a lower bound of the root; the unpolished guess of the
        // normal quantile, lowered by more than its error, is enough for that.
        double lo = mu + sigma * (normal_quantile_guess(s_eff) - 1e-3), hi = lo;
        double S = 0.0, B = 0.0, C = 0.0;
        bool ok = false;
        v = lo;
        if constexpr (COOP) {
            // One evaluation time buys 32 points, one per lane pair, at distances from the lower
            // bound that grow by sqrt(2) per pair (0.02 sigma (2^(p/2) - 1): pair 0 sits on the
            // bound, pair 31 at 927 sigma).  S is increasing, so the first pair above the target
            // and the pair before it bracket the root within a factor sqrt(2) of its distance;
            // the iteration starts from a third-order step taken at the nearer of the two.
            const int lane = (int)(threadIdx.x & (kWave - 1)), pair = lane >> 1;
            const double vp = lo + sigma * 0.02 * (ldexp((pair & 1) ? kSqrt2 : 1.0, pair >> 1) - 1.0);
            double Sp, Bp, Cp;
            sparsity_terms<true>(mu, sigma, vp, Sp, Bp, Cp);
            const uint64_t above = __ballot(Sp > s_eff);
            if (above != 0ull && (above & 1ull) == 0ull) {
                const int up = __ffsll((long long)above) - 1, down = up - 2;  // even lanes of the two pairs
                hi = __shfl(vp, up);
                lo = __shfl(vp, down);
                const double f_up = __shfl(Sp, up) - s_eff, f_down = __shfl(Sp, down) - s_eff;
                const int from = fabs(f_down) < fabs(f_up) ? down : up;
                const double v0 = __shfl(vp, from), f0 = __shfl(Sp, from) - s_eff;
                const double B0 = __shfl(Bp, from), C0 = __shfl(Cp, from);
                v = 0.5 * (lo + hi);
                if (B0 > 0.0) {
                    const double h = v0 - 2.0 * f0 * B0 / (2.0 * B0 * B0 - f0 * C0);
                    if (h > lo && h < hi) v = h;
                }
                ok = true;
            }
        }
        if (!ok) {  // one lane, or the grid did not bracket the root: widen upwards step by step
            hi = lo;
            double step = sigma;
            for (int i = 0; i < 64; ++i) {
                hi += step;
                step *= 2.0;
                sparsity_terms<COOP>(mu, sigma, hi, S, B, C);
                if (S > s_eff) { ok = true; break; }
                lo = hi;
            }
            v = 0.5 * (lo + hi);
        }
        if (!ok) r.status |= LGN_ST_NOT_CONVERGED;
        bool converged = false;
        for (int it = 0; it < 200 && ok; ++it) {
            sparsity_terms<COOP>(mu, sigma, v, S, B, C);
            v_at = v;
            evaluated = true;
            const double f = S - s_eff;
            if (f < 0.0) lo = v; else hi = v;
            double nv = 0.5 * (lo + hi);
            bool third_order = false;
            if (B > 0.0) {
                const double den = 2.0 * B * B - f * C;
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
        S_at = S; B_at = B; C_at = C;
    }
    const double alpha = exp(v);
    float af = alpha >= 3.4028234663852886e38 ? 3.4028234663852886e38f : (float)alpha;
    af = round_alpha(af, alpha_dtype);
    r.alpha = af;
    if (af > 0.0f) {
        if (point_mass) {
            r.s_pred = fmax(0.0, 1.0 - exp(mu) / (double)af);
        } else {
            // S at the rounded threshold.  Its logarithm is v plus log1p of the relative rounding
            // error; if that lies within 1e-5 sigma of the last point the iteration evaluated,
            // the second-order expansion there is exact to ~1e-16 (the next term is D^3 / 6 times
            // the third derivative, which is O(1 / sigma^3)) and saves an evaluation; otherwise
            // (16-bit thresholds, a last step that was not small) S is evaluated at the point.
            const double rel = ((double)af - alpha) / alpha;
            const double D = (v - v_at) + (rel - 0.5 * rel * rel);
            if (evaluated && alpha < 3.4028234663852886e38 && fabs(rel) < 1e-6 && fabs(D) <= 1e-5 * sigma) {
                r.s_pred = S_at + B_at * D + 0.5 * C_at * D * D;
            } else {
                double S, B, C;
                sparsity_terms<COOP>(mu, sigma, log((double)af), S, B, C);
                r.s_pred = S;
            }
        }
    }
    if (writer) *out = r;
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
// `scale_z` is the standard normal quantile of the scale rule's probability (the host evaluates
// it: it depends on the call's argument only); unused by the other scale rules.
__device__ __forceinline__ void fp_params_body(const lgn_stats_t *st, int n_bits, int e_fixed,
                                               int scale_mode, double scale_z, int sigma_units,
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
    const double zq = scale_z;

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

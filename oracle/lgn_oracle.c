/*
 * lgn_oracle.c -- TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT.
 *
 * A plain, slow, CPU-only statement of what the lognormal gradient-compression path computes,
 * written from the paper ("Neural gradients are near-lognormal: improved quantized and sparse
 * training").  It exists so that the GPU library can be checked against something that can be
 * read next to the paper by eye.  Only tests, the smoke check and the benchmark's cpu_baseline
 * leg may call it.  It shares no code, header, table or constant with the GPU library; it has
 * its own struct layouts and its own names.
 *
 * Every function states the passage it follows.  Scalar mathematics is in double precision;
 * the per-element operators work in the value domain (frexp / ldexp / comparisons of values),
 * not on bit patterns.  Loops over elements carry an OpenMP pragma because elements are
 * independent; nothing else is done for speed.
 *
 * Conventions the paper leaves open (all listed in the design document):
 *   - statistics use the population standard deviation over finite non-zero entries;
 *   - random words come from Philox4x32-10 (Salmon et al., SC'11) keyed by the 64-bit seed, with
 *     counter (lo32(j>>2), hi32(j>>2), 0, 0) and word index j&3 for global element j: one 32-bit
 *     word per element, whose upper half drives stochastic pruning and whose lower half drives
 *     stochastic rounding (independent bits of one uniform word);
 *   - the uniform variable of stochastic pruning lives on a 16-bit midpoint grid,
 *     u = (k + 1/2) / 2^16 with k the upper 16 bits of the element's word, so 0 < u < 1, and the
 *     comparison value alpha*u is one IEEE single-precision product;
 *   - stochastic rounding goes up iff (cut-off part) + (r + 1/2) / 2^16 spacings reach one
 *     spacing, r the lower 16 bits of the element's word: the up-probability is the cut-off
 *     fraction rounded to the nearest multiple of 2^-16 (exact for 16-bit element types);
 *   - an FP(1,e,m) word has exponent field c in [1, 2^e-1] meaning E = c - 2^(e-1), field 0 is
 *     zero; saturation goes to the largest finite code; underflow flushes to zero and is decided
 *     on the exponent before rounding.
 *
 *   - the prefix code of the appendix "Encoding" is laid out as a bit stream in which stream bit
 *     k is bit (k & 7) of byte k >> 3, codewords are written first symbol first, the value that
 *     follows "11" is the element's own bit pattern (32, 16 or N bits) least significant bit
 *     first, every chunk of 4096 elements starts on a 32-bit boundary listed in a table, and the
 *     bit lengths of a chunk's 16 sub-blocks of 256 elements are listed beside it.
 *
 * Pins (tests/test_oracle_*.py): Philox known-answer vectors; Table 2 of the paper for the
 * format choice; quadrature of the sparsity definition (the expectation over the uniform
 * variable of the lognormal CDF) and Monte-Carlo pruning for the threshold; exhaustive
 * enumeration of all FP-n codes for the quantizer; exact results on powers of two for the
 * statistics; the code table of the appendix, an independent string decoder and the paper's
 * bits-per-value claim for the prefix code.  Parity unpinned (pure conventions): the 0.997 default quantile of the scale rule,
 * the tie rule of nearest rounding, the 16-bit midpoint grids of the two random variables.
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- enumerations (oracle's own; values are part of the documented C interface) ---------- */
enum { ORC_F32 = 0, ORC_BF16 = 1, ORC_F16 = 2 };
enum { ORC_ROUND_NEAREST_EVEN = 0, ORC_ROUND_STOCHASTIC = 1 };
enum { ORC_OUT_VALUE = 0, ORC_OUT_CODE8 = 1, ORC_OUT_PACKED = 2 };
enum { ORC_SCALE_QUANTILE = 0, ORC_SCALE_MAX = 1, ORC_SCALE_CENTER = 2 };
enum { ORC_SIGMA_PAPER_LITERAL = 0, ORC_SIGMA_BASE2 = 1 };
enum {
    ORC_ST_EMPTY = 1u,             /* no finite non-zero element                          */
    ORC_ST_SIGMA0 = 2u,            /* all finite non-zero magnitudes equal                */
    ORC_ST_NOTHING_TO_PRUNE = 4u,  /* target sparsity already met by existing zeros       */
    ORC_ST_NOT_CONVERGED = 8u,
    ORC_ST_ALPHA_BELOW_FP_RANGE = 16u,
    ORC_ST_HAS_NONFINITE = 32u
};

typedef struct {
    uint64_t n, nnz, n_nonfinite;
    double mu, sigma;          /* of ln|g| over finite non-zero entries, population std */
    float max_abs, min_abs_nz; /* over finite non-zero entries; 0 when there is none    */
    uint32_t status;
} orc_stats_t;

typedef struct {
    float alpha;   /* threshold, already rounded to the tensor dtype             */
    double s_eff;  /* S' : sparsity asked of the non-zero part                    */
    double s_pred; /* closed-form sparsity of the non-zero part at the rounded alpha */
    uint32_t status;
} orc_prune_params_t;

typedef struct {
    int32_t n_bits, e_bits, m_bits, scale_exp;
    double eta; /* expected relative error of the chosen split */
    uint32_t status;
} orc_fp_params_t;

static int g_threads = 1;
void orc_set_threads(int t) { g_threads = t < 1 ? 1 : t; }
int orc_get_threads(void) { return g_threads; }
int orc_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_num_procs();
#else
    return 1;
#endif
}

/* ---- element access ---------------------------------------------------------------------- */
static float bf16_to_float(uint16_t h)
{
    uint32_t b = (uint32_t)h << 16;
    float f;
    memcpy(&f, &b, 4);
    return f;
}
/* fp32 -> bf16, round to nearest, ties to even; only ever applied to values that are exactly
 * representable, and to alpha. */
static uint16_t float_to_bf16(float f)
{
    uint32_t b;
    memcpy(&b, &f, 4);
    if ((b & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((b >> 16) | 0x40u);
    b += 0x7fffu + ((b >> 16) & 1u);
    return (uint16_t)(b >> 16);
}
/* IEEE half precision in the value domain: 1 sign, 5 exponent (bias 15), 10 fraction bits;
 * exponent field 0 holds the subnormals k 2^-24, field 31 infinity and NaN. */
static float f16_to_float(uint16_t h)
{
    const int sign = h >> 15, ex = (h >> 10) & 31, fr = h & 1023;
    double v;
    if (ex == 31) v = fr ? (double)NAN : (double)INFINITY;
    else if (ex == 0) v = ldexp((double)fr, -24);
    else v = ldexp(1.0 + (double)fr / 1024.0, ex - 15);
    return (float)(sign ? -v : v);
}
/* fp32 -> fp16, round to nearest, ties to even (nearbyint in the default rounding mode);
 * magnitudes that round to 2^16 or more become infinity. */
static uint16_t float_to_f16(float f)
{
    const uint16_t sign = signbit(f) ? 0x8000u : 0u;
    const double a = fabs((double)f);
    if (isnan(f)) return (uint16_t)(sign | 0x7e00u);
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e); /* a = m 2^e, m in [0.5, 1): the binade is 2^(e-1) */
    int E = e - 1;
    if (E < -14) E = -14;                              /* subnormal range: spacing 2^-24 */
    const double units = nearbyint(ldexp(a, 10 - E));  /* a in units of the spacing 2^(E-10) */
    const double r = ldexp(units, E - 10);
    if (r >= 65536.0) return (uint16_t)(sign | 0x7c00u);
    if (r < ldexp(1.0, -14)) return (uint16_t)(sign | (uint16_t)units); /* subnormal or zero */
    int e2;
    const double m = frexp(r, &e2); /* r = m 2^e2; rounding may have moved r to the next binade */
    return (uint16_t)(sign | (uint16_t)((e2 - 1 + 15) << 10) | (uint16_t)nearbyint((2.0 * m - 1.0) * 1024.0));
}
static float load_elem(const void *g, uint64_t i, int dtype)
{
    if (dtype == ORC_F32) return ((const float *)g)[i];
    if (dtype == ORC_BF16) return bf16_to_float(((const uint16_t *)g)[i]);
    return f16_to_float(((const uint16_t *)g)[i]);
}
static void store_elem(void *out, uint64_t i, int dtype, float v)
{
    if (dtype == ORC_F32) ((float *)out)[i] = v;
    else if (dtype == ORC_BF16) ((uint16_t *)out)[i] = float_to_bf16(v);
    else ((uint16_t *)out)[i] = float_to_f16(v);
}
/* alpha rounded to the element type, saturating at the largest finite value of that type */
static float round_alpha(float af, int alpha_dtype)
{
    if (alpha_dtype == ORC_BF16) {
        af = bf16_to_float(float_to_bf16(af));
        if (!isfinite(af)) af = bf16_to_float(0x7f7f);
    } else if (alpha_dtype == ORC_F16) {
        af = f16_to_float(float_to_f16(af));
        if (!isfinite(af)) af = 65504.0f;
    }
    return af;
}
float orc_f16_to_float(uint16_t h) { return f16_to_float(h); }
uint16_t orc_float_to_f16(float f) { return float_to_f16(f); }

/* ==========================================================================================
 * Step 1.  Lognormal parameters (Section "Neural gradients distribution": the fit is made on
 * the absolute values, zero-valued entries excluded; appendix "Stochastic pruning complexity":
 * mean and standard deviation, O(n)).
 * mu = mean of ln|g|, sigma = population standard deviation of ln|g|, both over the entries
 * that are finite and non-zero.  Two passes: mean first, then squared deviations.
 * ========================================================================================== */
/* Is element i part of the fit?  Without a mask every element is.  With one (appendix "Algorithm
 * for bi-Modal lognormal pruning", step 3: only the values whose corresponding entries in the
 * other gradient tensor are non-zero), element i counts iff the mask's entry i is non-zero; the
 * mask is either a tensor of the same type as g (kind 1) or one byte per element (kind 2). */
static int in_fit(const void *mask, int mask_kind, uint64_t i, int dtype)
{
    if (mask_kind == 1) return load_elem(mask, i, dtype) != 0.0f; /* NaN != 0: counts */
    if (mask_kind == 2) return ((const uint8_t *)mask)[i] != 0;
    return 1;
}

static void stats_impl(const void *g, const void *mask, int mask_kind, uint64_t n, int dtype,
                       orc_stats_t *out)
{
    uint64_t nnz = 0, nonfinite = 0;
    long double sum = 0.0L;
    float mx = 0.0f, mn = INFINITY;
    int64_t i, N = (int64_t)n;
#pragma omp parallel for num_threads(g_threads) reduction(+ : nnz, nonfinite, sum) \
    reduction(max : mx) reduction(min : mn)
    for (i = 0; i < N; ++i) {
        if (!in_fit(mask, mask_kind, (uint64_t)i, dtype)) continue;
        float x = load_elem(g, (uint64_t)i, dtype);
        if (!isfinite(x)) { ++nonfinite; continue; }
        if (x == 0.0f) continue;
        float a = fabsf(x);
        ++nnz;
        sum += (long double)log((double)a);
        if (a > mx) mx = a;
        if (a < mn) mn = a;
    }
    memset(out, 0, sizeof *out);
    out->n = n;
    out->nnz = nnz;
    out->n_nonfinite = nonfinite;
    if (nonfinite) out->status |= ORC_ST_HAS_NONFINITE;
    if (nnz == 0) {
        out->mu = NAN;
        out->sigma = NAN;
        out->max_abs = 0.0f;
        out->min_abs_nz = 0.0f;
        out->status |= ORC_ST_EMPTY;
        return;
    }
    double mu = (double)(sum / (long double)nnz);
    long double ss = 0.0L;
#pragma omp parallel for num_threads(g_threads) reduction(+ : ss)
    for (i = 0; i < N; ++i) {
        if (!in_fit(mask, mask_kind, (uint64_t)i, dtype)) continue;
        float x = load_elem(g, (uint64_t)i, dtype);
        if (!isfinite(x) || x == 0.0f) continue;
        long double d = (long double)log((double)fabsf(x)) - (long double)mu;
        ss += d * d;
    }
    out->mu = mu;
    out->sigma = sqrt((double)(ss / (long double)nnz));
    out->max_abs = mx;
    out->min_abs_nz = mn;
    if (mx == mn) out->status |= ORC_ST_SIGMA0;
}

void orc_stats(const void *g, uint64_t n, int dtype, orc_stats_t *out)
{
    stats_impl(g, NULL, 0, n, dtype, out);
}

/* Statistics of the right mode of a bi-modal gradient (appendix "Algorithm for bi-Modal lognormal
 * pruning", steps 1 and 3).  n stays the size of the whole tensor and nnz counts the entries of
 * the fit, so the zero credit of orc_threshold, S' = (S n - (n - nnz)) / nnz, is step 2's
 * S' = (S - l) / (1 - l) with l the fraction left out of the fit. */
void orc_stats_masked(const void *g, const void *mask, uint64_t n, int dtype, int mask_kind,
                      orc_stats_t *out)
{
    stats_impl(g, mask, mask_kind, n, dtype, out);
}

/* ==========================================================================================
 * Step 2a.  Sparsity as a function of the threshold (Section "Analytical derivation of
 * Sparsity", the closed form that follows the integral over the uniform variable; derivation
 * in the appendix "From sparsity to the threshold").  With L = ln(alpha / e^mu):
 *
 *   S = 1/2 + (e^mu / 2 alpha) [ e^{sigma^2/2} erf(sigma/sqrt2 - L/(sqrt2 sigma))
 *                                + (alpha/e^mu) erf(L/(sqrt2 sigma)) - e^{sigma^2/2} ]
 *
 * The two terms that carry e^{sigma^2/2} are combined as erf(a) - 1 = -erfc(a) so that nothing
 * cancels, and the product e^{sigma^2/2 - L} erfc(a) is formed as exp of a sum of logarithms so
 * that it neither overflows nor turns into inf * 0.
 * ========================================================================================== */
double orc_sparsity_of_log_alpha(double mu, double sigma, double v)
{
    double L = v - mu;
    double a = sigma / M_SQRT2 - L / (M_SQRT2 * sigma);
    double tail = erfc(a);
    double second = tail > 0.0 ? exp(0.5 * sigma * sigma - L + log(tail)) : 0.0;
    return 0.5 + 0.5 * erf(L / (M_SQRT2 * sigma)) - 0.5 * second;
}
double orc_sparsity_of_alpha(double mu, double sigma, double alpha)
{
    return orc_sparsity_of_log_alpha(mu, sigma, log(alpha));
}

/* Standard normal quantile by bisection on the CDF (used by the scale rule only). */
static double normal_cdf(double z) { return 0.5 * erfc(-z / M_SQRT2); }
double orc_normal_quantile(double q)
{
    double lo = -40.0, hi = 40.0;
    for (int it = 0; it < 200; ++it) {
        double mid = 0.5 * (lo + hi);
        if (normal_cdf(mid) < q) lo = mid; else hi = mid;
        if (hi - lo <= 1e-16 * fmax(1.0, fabs(mid))) break;
    }
    return 0.5 * (lo + hi);
}

/* ==========================================================================================
 * Step 2b.  Threshold for a target sparsity (Section "Stochastic pruning", problem
 * formulation: find alpha that induces sparsity S; the closed form "can easily be solved
 * numerically").  The target S is the zero fraction of the whole output tensor, so the
 * non-zero part must be pruned to S' = (S - l)/(1 - l) with l the fraction already zero
 * (appendix "Algorithm for bi-Modal lognormal pruning", step 2).
 * Solved by bisection on v = ln(alpha); S is increasing in v.
 * ========================================================================================== */
void orc_threshold(const orc_stats_t *st, double target_sparsity, int alpha_dtype,
                   orc_prune_params_t *out)
{
    memset(out, 0, sizeof *out);
    out->status = st->status & (ORC_ST_EMPTY | ORC_ST_SIGMA0 | ORC_ST_HAS_NONFINITE);
    if (st->nnz == 0) {
        out->alpha = 0.0f;
        out->s_eff = 0.0;
        out->s_pred = 0.0;
        return;
    }
    double n = (double)st->n, nnz = (double)st->nnz;
    double s_eff = (target_sparsity * n - (n - nnz)) / nnz;
    out->s_eff = s_eff;
    if (!(s_eff > 0.0)) {
        out->alpha = 0.0f;
        out->s_pred = 0.0;
        out->status |= ORC_ST_NOTHING_TO_PRUNE;
        return;
    }
    double mu = st->mu, sigma = st->sigma, v;
    if (sigma < 1e-12) {
        /* point mass at c = e^mu: the fraction zeroed is P(c < alpha u) = 1 - c/alpha */
        v = mu - log1p(-s_eff);
        out->status |= ORC_ST_SIGMA0;
    } else {
        double lo = mu - 40.0 * sigma, hi = mu + 40.0 * sigma + sigma * sigma + 50.0;
        if (!(orc_sparsity_of_log_alpha(mu, sigma, lo) < s_eff &&
              orc_sparsity_of_log_alpha(mu, sigma, hi) > s_eff))
            out->status |= ORC_ST_NOT_CONVERGED;
        for (int it = 0; it < 400; ++it) {
            double mid = 0.5 * (lo + hi);
            if (orc_sparsity_of_log_alpha(mu, sigma, mid) < s_eff) lo = mid; else hi = mid;
            if (hi - lo <= 1e-15 * fmax(1.0, fabs(mid))) break;
        }
        v = 0.5 * (lo + hi);
    }
    double alpha = exp(v);
    float af = alpha >= (double)FLT_MAX ? FLT_MAX : (float)alpha;
    af = round_alpha(af, alpha_dtype);
    out->alpha = af;
    if (af > 0.0f)
        out->s_pred = sigma < 1e-12 ? fmax(0.0, 1.0 - exp(mu) / (double)af)
                                    : orc_sparsity_of_alpha(mu, sigma, (double)af);
}

/* ==========================================================================================
 * Step 3a.  Expected relative error of an FP(1, e, m) quantizer on lognormal data (Section
 * "Analytical derivation of the relative error", the closed form, and its appendix).  Three
 * contributions: mantissa noise when the exponent is in range, saturation above, flush below.
 * E_max = 2^(e-1).  The mantissa term uses 2^m levels (spacing 1/2^m as the problem
 * formulation states); the printed denominator 2^m - 1 would make every m = 0 split infinitely
 * bad, against the paper's own table of optimal formats.
 * ========================================================================================== */
double orc_expected_relative_error(double sigma, int e_bits, int m_bits)
{
    double emax = ldexp(1.0, e_bits - 1);
    double phi = normal_cdf(emax / sigma);
    double mantissa = (2.0 * phi - 1.0) / (8.0 * M_LN2 * ldexp(1.0, m_bits));
    double z = sigma * M_LN2 / M_SQRT2 + emax / (M_SQRT2 * sigma);
    double tail = erfc(z);
    /* 2^(E_max-1) e^{sigma^2 ln^2 2 / 2} (erf(z) - 1), formed in the log domain */
    double over = tail > 0.0
                      ? -exp((emax - 1.0) * M_LN2 + 0.5 * sigma * sigma * M_LN2 * M_LN2 + log(tail))
                      : 0.0;
    return mantissa + over - 0.5 * erf(emax / (M_SQRT2 * sigma)) + 1.5 - phi;
}

/* ==========================================================================================
 * Step 3b.  Exponent/mantissa split and power-of-two scale.
 * Split (Section "The optimal mantissa-exponent representation"): the e in [1, N-1] that
 * minimises the expected relative error with m = N-1-e; ties go to the smaller e.
 * Scale (Section "Per-Layer Gradient scaling" and the appendix algorithm "Gradient scaling"):
 * an integer exponent s such that the tensor is quantized as 2^s Q(x / 2^s), chosen so that the
 * largest gradients land in the top binade 2^(E_max-1):
 *   MAX       s = floor(log2 max|x|)                      - (E_max - 1)
 *   QUANTILE  s = floor(log2 of the q-quantile of the fitted lognormal) - (E_max - 1)
 *             (the appendix on truncated lognormals takes a high quantile, e.g. 0.997,
 *              because the sample maximum is a noisy estimator)
 *   CENTER    s = round(mu / ln 2)
 * ========================================================================================== */
void orc_fp_params(const orc_stats_t *st, int n_bits, int e_bits, int scale_mode, double scale_arg,
                   int sigma_units, orc_fp_params_t *out)
{
    memset(out, 0, sizeof *out);
    out->n_bits = n_bits;
    out->status = st->status & (ORC_ST_EMPTY | ORC_ST_SIGMA0 | ORC_ST_HAS_NONFINITE);
    int e;
    if (e_bits >= 1) {
        e = e_bits;
        out->eta = (st->nnz && st->sigma >= 1e-12)
                       ? orc_expected_relative_error(
                             sigma_units == ORC_SIGMA_BASE2 ? st->sigma / M_LN2 : st->sigma, e,
                             n_bits - 1 - e)
                       : 0.0;
    } else if (st->nnz == 0 || st->sigma < 1e-12) {
        e = 1; /* no spread: every bit to the mantissa */
        out->eta = 0.0;
    } else {
        double sg = sigma_units == ORC_SIGMA_BASE2 ? st->sigma / M_LN2 : st->sigma;
        double best = INFINITY;
        e = 1;
        for (int c = 1; c <= n_bits - 1; ++c) {
            double eta = orc_expected_relative_error(sg, c, n_bits - 1 - c);
            if (eta < best) { best = eta; e = c; }
        }
        out->eta = best;
    }
    out->e_bits = e;
    out->m_bits = n_bits - 1 - e;
    int etop = (1 << (e - 1)) - 1;
    if (st->nnz == 0) { out->scale_exp = 0; return; }
    double top_log2;
    if (scale_mode == ORC_SCALE_MAX) {
        int ex;
        frexp((double)st->max_abs, &ex); /* max = f 2^ex, f in [1/2,1)  =>  floor(log2 max) = ex-1 */
        out->scale_exp = (ex - 1) - etop;
        return;
    } else if (scale_mode == ORC_SCALE_CENTER) {
        out->scale_exp = (int)floor(st->mu / M_LN2 + 0.5);
        return;
    }
    top_log2 = (st->mu + orc_normal_quantile(scale_arg) * st->sigma) / M_LN2;
    out->scale_exp = (int)floor(top_log2) - etop;
}

/* ==========================================================================================
 * Random words: Philox4x32-10 as published (Salmon, Moraes, Dror, Shaw, "Parallel random
 * numbers: as easy as 1, 2, 3", SC'11): ten rounds; per round the two products
 * 0xD2511F53 * c0 and 0xCD9E8D57 * c2 are split in high and low halves and recombined with the
 * other two counter words and the key; the key advances by the Weyl constants between rounds.
 * ========================================================================================== */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The word of global element j: upper half for the pruning variable, lower half for rounding. */
uint32_t orc_random_word(uint64_t seed, uint64_t j)
{
    uint64_t q = j >> 2;
    uint32_t ctr[4] = { (uint32_t)q, (uint32_t)(q >> 32), 0u, 0u };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t w[4];
    orc_philox4x32_10(ctr, key, w);
    return w[j & 3u];
}

/* ==========================================================================================
 * Step 4.  Stochastic pruning T_{alpha,eps} (Section "Stochastic pruning", the three-case
 * definition):  |x| > alpha -> x;  alpha eps <= |x| <= alpha -> sign(x) alpha;
 * |x| < alpha eps -> 0.   eps = u = ((w >> 16) + 1/2) / 2^16 and alpha*u is one single-precision product.
 * Exact zeros stay zero whatever u is, NaN passes through.
 * ========================================================================================== */
static float prune_one(float x, float alpha, uint32_t w)
{
    if (isnan(x)) return x;
    float a = fabsf(x);
    if (a == 0.0f) return 0.0f;
    if (a > alpha) return x;
    double u = ((double)(w >> 16) + 0.5) / 65536.0; /* 16-bit midpoint grid, 0 < u < 1 */
    float t = (float)((double)alpha * u);             /* exact product, one rounding to single */
    if (a < t) return 0.0f;
    return copysignf(alpha, x);
}

void orc_prune(const void *g, uint64_t n, int dtype, float alpha, uint64_t seed,
               uint64_t elem_offset, void *out)
{
    int64_t i, N = (int64_t)n;
#pragma omp parallel for num_threads(g_threads)
    for (i = 0; i < N; ++i) {
        float x = load_elem(g, (uint64_t)i, dtype);
        uint32_t w = orc_random_word(seed, elem_offset + (uint64_t)i);
        float y = prune_one(x, alpha, w);
        if (dtype == ORC_F32) ((float *)out)[i] = y; /* keeps NaN payloads */
        else if (isnan(y)) ((uint16_t *)out)[i] = ((const uint16_t *)g)[i];
        else store_elem(out, (uint64_t)i, dtype, y);
    }
}

/* ==========================================================================================
 * Step 5.  FP(1,e,m) quantizer with scale 2^s (Section "Problem formulation" of the
 * quantization application: decomposition x = M 2^E with M in [1,2); saturate above, flush
 * below, mantissa on 2^m levels; appendix algorithm "Gradient scaling": X_Q = 2^s Q(X / 2^s)).
 * Returns the N-bit code:  sign << (e+m) | (E + E_max) << m | k.
 * ========================================================================================== */
static uint32_t quantize_one(float x, int e, int m, int s, int rounding, uint32_t w)
{
    int emax = 1 << (e - 1), etop = emax - 1, emin = 1 - emax;
    uint32_t sign = signbit(x) ? 1u << (e + m) : 0u;
    uint32_t maxmag = (1u << (e + m)) - 1u;
    if (x == 0.0f) return 0u;
    if (isnan(x) || isinf(x)) return sign | maxmag; /* not finite: saturates (NaN stays NaN in VALUE output) */
    int ex;
    double M = 2.0 * frexp(fabs((double)x), &ex); /* |x| = M 2^(ex-1), M in [1,2) */
    int E = (ex - 1) - s;
    if (E < emin) return 0u;
    if (E > etop) return sign | maxmag;
    double levels = ldexp(1.0, m);
    double k = floor((M - 1.0) * levels);
    /* what is cut off, in units of the input's own last mantissa place (2^-23) */
    double f = (M - 1.0) * 8388608.0 - k * ldexp(1.0, 23 - m);
    double unit = ldexp(1.0, 23 - m);
    int up;
    if (rounding == ORC_ROUND_STOCHASTIC) {
        /* (r + 1/2) / 2^16 of a spacing, r the lower half of the element's word */
        double r = ((double)(w & 0xffffu) + 0.5) / 65536.0 * unit;
        up = f + r >= unit;
    } else {
        uint32_t code_below = ((uint32_t)(E + emax) << m) | (uint32_t)k;
        up = f > 0.5 * unit || (f == 0.5 * unit && (code_below & 1u));
    }
    if (up) {
        k += 1.0;
        if (k == levels) { k = 0.0; E += 1; }
        if (E > etop) return sign | maxmag;
    }
    return sign | ((uint32_t)(E + emax) << m) | (uint32_t)k;
}

/* Value of a code: exponent field 0 is zero whatever the other bits say. */
double orc_decode(uint32_t code, int e, int m, int s)
{
    int emax = 1 << (e - 1);
    uint32_t c = (code >> m) & ((1u << e) - 1u);
    uint32_t k = code & ((1u << m) - 1u);
    if (c == 0) return 0.0;
    double v = ldexp(1.0 + (double)k / ldexp(1.0, m), (int)c - emax + s);
    return ((code >> (e + m)) & 1u) ? -v : v;
}

uint64_t orc_packed_bytes(uint64_t n, int n_bits) { return (n * (uint64_t)n_bits + 7u) / 8u; }

/* Little-endian bit stream: bit b of code i is bit i*N + b of the stream. */
void orc_pack(const uint8_t *codes, uint64_t n, int n_bits, uint8_t *out)
{
    memset(out, 0, orc_packed_bytes(n, n_bits));
    for (uint64_t i = 0; i < n; ++i)
        for (int b = 0; b < n_bits; ++b)
            if ((codes[i] >> b) & 1u) {
                uint64_t pos = i * (uint64_t)n_bits + (uint64_t)b;
                out[pos >> 3] |= (uint8_t)(1u << (pos & 7u));
            }
}
void orc_unpack(const uint8_t *packed, uint64_t n, int n_bits, uint8_t *codes)
{
    for (uint64_t i = 0; i < n; ++i) {
        uint8_t c = 0;
        for (int b = 0; b < n_bits; ++b) {
            uint64_t pos = i * (uint64_t)n_bits + (uint64_t)b;
            if ((packed[pos >> 3] >> (pos & 7u)) & 1u) c |= (uint8_t)(1u << b);
        }
        codes[i] = c;
    }
}

static void emit(void *out, uint64_t i, int dtype, int out_kind, const void *g, float x,
                 uint32_t code, int e, int m, int s, uint8_t *codes)
{
    if (out_kind == ORC_OUT_VALUE) {
        if (isnan(x)) {
            if (dtype == ORC_F32) ((float *)out)[i] = x;
            else ((uint16_t *)out)[i] = g ? ((const uint16_t *)g)[i] : 0x7fc0;
        } else {
            store_elem(out, i, dtype, (float)orc_decode(code, e, m, s));
        }
    } else {
        codes[i] = (uint8_t)code;
    }
}

/* Quantize (and optionally prune first).  For PACKED output `scratch_codes` must hold n bytes. */
static void quantize_impl(const void *g, uint64_t n, int dtype, int do_prune, float alpha, int e,
                          int m, int s, int rounding, uint64_t seed, uint64_t elem_offset,
                          void *out, int out_kind, uint8_t *scratch_codes)
{
    uint8_t *codes = out_kind == ORC_OUT_CODE8 ? (uint8_t *)out : scratch_codes;
    int64_t i, N = (int64_t)n;
#pragma omp parallel for num_threads(g_threads)
    for (i = 0; i < N; ++i) {
        uint64_t j = elem_offset + (uint64_t)i;
        float x = load_elem(g, (uint64_t)i, dtype);
        uint32_t w = orc_random_word(seed, j); /* upper half prunes, lower half rounds */
        if (do_prune) x = prune_one(x, alpha, w);
        uint32_t code = quantize_one(x, e, m, s, rounding, w);
        emit(out, (uint64_t)i, dtype, out_kind, g, x, code, e, m, s, codes);
    }
    if (out_kind == ORC_OUT_PACKED) orc_pack(codes, n, 1 + e + m, (uint8_t *)out);
}

void orc_fp_quantize(const void *g, uint64_t n, int dtype, int e, int m, int s, int rounding,
                     uint64_t seed, uint64_t elem_offset, void *out, int out_kind,
                     uint8_t *scratch_codes)
{
    quantize_impl(g, n, dtype, 0, 0.0f, e, m, s, rounding, seed, elem_offset, out, out_kind,
                  scratch_codes);
}

/* Step 6 (composition): prune, then quantize what pruning returned; the two decisions of an
 * element use disjoint halves of its word. */
void orc_prune_quantize(const void *g, uint64_t n, int dtype, float alpha, int e, int m, int s,
                        int rounding, uint64_t seed, uint64_t elem_offset, void *out, int out_kind,
                        uint8_t *scratch_codes)
{
    quantize_impl(g, n, dtype, 1, alpha, e, m, s, rounding, seed, elem_offset, out, out_kind,
                  scratch_codes);
}

void orc_dequantize(const uint8_t *codes, uint64_t n, int e, int m, int s, int dtype, void *out)
{
    for (uint64_t i = 0; i < n; ++i) store_elem(out, i, dtype, (float)orc_decode(codes[i], e, m, s));
}

/* single-element entry points for exhaustive tests */
uint32_t orc_quantize_one(float x, int e, int m, int s, int rounding, uint32_t w)
{
    return quantize_one(x, e, m, s, rounding, w);
}
float orc_prune_one(float x, float alpha, uint32_t w) { return prune_one(x, alpha, w); }

/* ------------------------------------------------------------------------------------------
 * Prefix code of the pruned tensor (appendix "Encoding", table "Simple proposed encoding for the
 * values after stochastic pruning"):
 *     0 -> "0",   +alpha -> "100",   -alpha -> "101",   any other value -> "11" then the value.
 * An element is given as its raw pattern of `width` bits (fp32: 32, bf16: 16, FP-n code: N);
 * the top bit of the pattern is the sign, `special` is the magnitude pattern of alpha.  Only the
 * all-zero pattern takes the one-bit codeword, so the code is lossless for any input.
 * Container (this build's choice, the paper gives the codewords only): chunks of 4096 elements,
 * each starting on a 32-bit boundary; table[c] = index of the first 32-bit word of chunk c,
 * table[nchunks] = total number of words, table[nchunks + 1] = 0 (status, no overflow here).
 * A chunk is further divided into 16 sub-blocks of 256 elements whose lengths in bits are listed
 * (sub[16 c + j], 16-bit numbers; 0 for a sub-block past the end of the tensor), so that decoding
 * can start at any multiple of 256 elements: sub-block j of chunk c begins at stream bit
 * 32 table[c] + sub[16 c] + ... + sub[16 c + j - 1].
 * ------------------------------------------------------------------------------------------ */
#define ORC_PREFIX_CHUNK 4096u
#define ORC_PREFIX_SUB 256u

static uint32_t raw_pattern(const void *in, uint64_t i, int width)
{
    if (width == 32) return ((const uint32_t *)in)[i];
    if (width == 16) return ((const uint16_t *)in)[i];
    return ((const uint8_t *)in)[i];
}

static unsigned symbol_bits(uint32_t v, int width, uint32_t special)
{
    const uint32_t mag = v & ((1u << (width - 1)) - 1u);
    if (v == 0u) return 1u;
    if (special != 0u && mag == special) return 3u;
    return 2u + (unsigned)width;
}

static void put_bit(uint8_t *out, uint64_t k, unsigned bit)
{
    if (bit) out[k >> 3] |= (uint8_t)(1u << (k & 7u));
}

uint64_t orc_prefix_chunks(uint64_t n) { return (n + ORC_PREFIX_CHUNK - 1u) / ORC_PREFIX_CHUNK; }

/* Worst case: every element takes the long codeword. */
uint64_t orc_prefix_bound_bytes(uint64_t n, int width)
{
    const uint64_t words_per_chunk = ((uint64_t)ORC_PREFIX_CHUNK * (2u + (unsigned)width) + 31u) / 32u;
    return orc_prefix_chunks(n) * words_per_chunk * 4u;
}

/* Fills table (nchunks + 2 entries), sub (16 nchunks entries, if not NULL) and, if out is not
 * NULL, the zero-initialised stream.  Returns the number of bytes of the stream. */
uint64_t orc_prefix_encode(const void *in, uint64_t n, int width, uint32_t special, uint8_t *out,
                           uint64_t *table, uint16_t *sub)
{
    const uint64_t nchunks = orc_prefix_chunks(n);
    int64_t c;
#pragma omp parallel for num_threads(g_threads)
    for (c = 0; c < (int64_t)nchunks; ++c) {
        uint64_t bits = 0, i = (uint64_t)c * ORC_PREFIX_CHUNK;
        const uint64_t end = i + ORC_PREFIX_CHUNK < n ? i + ORC_PREFIX_CHUNK : n;
        unsigned j;
        if (sub) for (j = 0; j < 16u; ++j) sub[16 * c + j] = 0;
        for (; i < end; ++i) {
            const unsigned len = symbol_bits(raw_pattern(in, i, width), width, special);
            bits += len;
            if (sub) sub[16 * c + (i - (uint64_t)c * ORC_PREFIX_CHUNK) / ORC_PREFIX_SUB] += (uint16_t)len;
        }
        table[c + 1] = (bits + 31u) / 32u; /* words of this chunk, turned into offsets below */
    }
    table[0] = 0;
    for (c = 0; c < (int64_t)nchunks; ++c) table[c + 1] += table[c];
    table[nchunks + 1] = 0;
    if (!out) return table[nchunks] * 4u;
#pragma omp parallel for num_threads(g_threads)
    for (c = 0; c < (int64_t)nchunks; ++c) {
        uint64_t k = table[c] * 32u, i = (uint64_t)c * ORC_PREFIX_CHUNK;
        const uint64_t end = i + ORC_PREFIX_CHUNK < n ? i + ORC_PREFIX_CHUNK : n;
        for (; i < end; ++i) {
            const uint32_t v = raw_pattern(in, i, width);
            const unsigned len = symbol_bits(v, width, special);
            if (len == 1u) {
                put_bit(out, k++, 0u);
            } else if (len == 3u) {
                put_bit(out, k++, 1u);
                put_bit(out, k++, 0u);
                put_bit(out, k++, (v >> (width - 1)) & 1u);
            } else {
                int b;
                put_bit(out, k++, 1u);
                put_bit(out, k++, 1u);
                for (b = 0; b < width; ++b) put_bit(out, k++, (v >> b) & 1u);
            }
        }
    }
    return table[nchunks] * 4u;
}

static unsigned get_bit(const uint8_t *in, uint64_t k) { return (in[k >> 3] >> (k & 7u)) & 1u; }

void orc_prefix_decode(const uint8_t *stream, const uint64_t *table, uint64_t n, int width,
                       uint32_t special, void *out)
{
    const uint64_t nchunks = orc_prefix_chunks(n);
    int64_t c;
#pragma omp parallel for num_threads(g_threads)
    for (c = 0; c < (int64_t)nchunks; ++c) {
        uint64_t k = table[c] * 32u, i = (uint64_t)c * ORC_PREFIX_CHUNK;
        const uint64_t end = i + ORC_PREFIX_CHUNK < n ? i + ORC_PREFIX_CHUNK : n;
        for (; i < end; ++i) {
            uint32_t v = 0;
            if (get_bit(stream, k++)) {
                if (get_bit(stream, k++)) {
                    int b;
                    for (b = 0; b < width; ++b) v |= (uint32_t)get_bit(stream, k++) << b;
                } else {
                    v = special | ((uint32_t)get_bit(stream, k++) << (width - 1));
                }
            }
            if (width == 32) ((uint32_t *)out)[i] = v;
            else if (width == 16) ((uint16_t *)out)[i] = (uint16_t)v;
            else ((uint8_t *)out)[i] = (uint8_t)v;
        }
    }
}

/* Decodes every sub-block of 256 elements on its own, from the bit position the container gives
 * for it: what the list of sub-block lengths is for. */
void orc_prefix_decode_sub(const uint8_t *stream, const uint64_t *table, const uint16_t *sub,
                           uint64_t n, int width, uint32_t special, void *out)
{
    const uint64_t nsub = (n + ORC_PREFIX_SUB - 1u) / ORC_PREFIX_SUB;
    int64_t b;
#pragma omp parallel for num_threads(g_threads)
    for (b = 0; b < (int64_t)nsub; ++b) {
        const uint64_t c = (uint64_t)b / 16u, j = (uint64_t)b % 16u;
        uint64_t k = table[c] * 32u, i = (uint64_t)b * ORC_PREFIX_SUB, t;
        const uint64_t end = i + ORC_PREFIX_SUB < n ? i + ORC_PREFIX_SUB : n;
        for (t = 0; t < j; ++t) k += sub[16 * c + t];
        for (; i < end; ++i) {
            uint32_t v = 0;
            if (get_bit(stream, k++)) {
                if (get_bit(stream, k++)) {
                    int q;
                    for (q = 0; q < width; ++q) v |= (uint32_t)get_bit(stream, k++) << q;
                } else {
                    v = special | ((uint32_t)get_bit(stream, k++) << (width - 1));
                }
            }
            if (width == 32) ((uint32_t *)out)[i] = v;
            else if (width == 16) ((uint16_t *)out)[i] = (uint16_t)v;
            else ((uint8_t *)out)[i] = (uint8_t)v;
        }
    }
}

/* ------------------------------------------------------------------------------------------
 * Cosine similarity of stochastic pruning and heterogeneous sparsity allocation (appendix
 * "Cosine similarity and heterogeneous stochastic pruning").
 *
 * Model: ln|x| - mu ~ N(0, sigma^2) truncated at c = k sigma above mu ("maximum value of
 * k sigma"; the section on truncated lognormals measures the cut in standard deviations of the
 * logarithm, 3 to 5, so the cut-off is taken in the log domain -- the derivation's ln(k sigma)
 * is the same formula with another name for the cut-off).  With L = ln(alpha) - mu and
 * Phi the standard normal CDF, per element and up to the common factor e^{2 mu}:
 *     E[x T(x)] = E[x^2] = e^{2 sigma^2} Phi((c - 2 sigma^2)/sigma)
 *     E[T(x)^2] = e^{L + sigma^2/2} Phi((min(L, c) - sigma^2)/sigma)
 *                 + e^{2 sigma^2} [Phi((c - 2 sigma^2)/sigma) - Phi((L - 2 sigma^2)/sigma)]_+
 * (the printed equations with (1 +- erf)/2 written as Phi), and
 *     cos = E[x T(x)] / sqrt(E[x^2] E[T(x)^2]) = sqrt(E[x^2] / E[T(x)^2]).
 * Everything is divided by e^{2 sigma^2} before it is evaluated, so large sigma cannot overflow.
 * ------------------------------------------------------------------------------------------ */
double orc_cosine_similarity(double sigma, double L, double c)
{
    const double s2 = sigma * sigma;
    const double q = normal_cdf((c - 2.0 * s2) / sigma);
    const double below = exp(L + 0.5 * s2 - 2.0 * s2) * normal_cdf((fmin(L, c) - s2) / sigma);
    double above = q - normal_cdf((L - 2.0 * s2) / sigma);
    if (above < 0.0) above = 0.0;
    return sqrt(q / (below + above));
}

/* Largest L (threshold in the log domain, relative to mu) whose cosine similarity is still at
 * least min_cosine; the similarity falls from 1 as L grows.  Plain bisection. */
double orc_log_alpha_for_cosine(double sigma, double c, double min_cosine)
{
    double lo = -40.0 * sigma - 2.0 * sigma * sigma - 50.0, hi = c;
    if (orc_cosine_similarity(sigma, hi, c) >= min_cosine) return hi;
    for (int it = 0; it < 400; ++it) {
        const double mid = 0.5 * (lo + hi);
        if (orc_cosine_similarity(sigma, mid, c) >= min_cosine) lo = mid; else hi = mid;
        if (hi - lo <= 1e-15 * fmax(1.0, fabs(mid))) break;
    }
    return 0.5 * (lo + hi);
}

/* Histogram of the magnitudes of the finite non-zero entries on a logarithmic grid with eight
 * bins per binade: a value M 2^E with M in [1, 2) and E >= -126 falls in bin
 * (E + 127) * 8 + floor((M - 1) * 8); smaller (subnormal) values in bin floor(|x| 2^129) < 8.
 * 2048 bins.  Used to read off a high quantile of ln|g| (section "Neural gradients lognormal
 * distributions are truncated": the sample maximum is too noisy, a quantile such as 0.997 is
 * taken instead). */
#define ORC_HIST_BINS 2048
static int hist_bin(float x)
{
    const double a = fabs((double)x);
    int e;
    if (a < ldexp(1.0, -126)) return (int)floor(a * ldexp(1.0, 129));
    const double m = 2.0 * frexp(a, &e); /* a = m 2^(e-1), m in [1, 2) */
    return (e - 1 + 127) * 8 + (int)floor((m - 1.0) * 8.0);
}

void orc_log_histogram(const void *g, uint64_t n, int dtype, uint64_t *hist)
{
    memset(hist, 0, ORC_HIST_BINS * sizeof *hist);
    for (uint64_t i = 0; i < n; ++i) {
        const float x = load_elem(g, i, dtype);
        if (!isfinite(x) || x == 0.0f) continue;
        ++hist[hist_bin(x)];
    }
}

/* ln of the lower edge of bin b (b >= 8); the upper edge of b is the lower edge of b + 1. */
static double bin_log_edge(int b)
{
    return log(1.0 + (double)(b % 8) / 8.0) + (double)(b / 8 - 127) * M_LN2;
}

/* Truncation point in units of sigma: k = (y_q - mu) / sigma with y_q the q-quantile of ln|g|
 * read off the histogram -- the bin that holds the entry of rank ceil(q N), interpolated
 * linearly in the logarithm inside the bin.  Without a histogram (hist == NULL) the quantile of
 * the fitted normal is used. */
double orc_truncation_k(const uint64_t *hist, double mu, double sigma, double q)
{
    if (!hist) return orc_normal_quantile(q);
    uint64_t total = 0;
    for (int b = 0; b < ORC_HIST_BINS; ++b) total += hist[b];
    if (total == 0 || !(sigma > 0.0)) return orc_normal_quantile(q);
    uint64_t rank = (uint64_t)ceil(q * (double)total);
    if (rank < 1) rank = 1;
    if (rank > total) rank = total;
    uint64_t before = 0;
    int b = 0;
    for (; b < ORC_HIST_BINS; ++b) {
        if (before + hist[b] >= rank) break;
        before += hist[b];
    }
    if (b < 8) b = 8; /* subnormal magnitudes: the edge of the first normal bin */
    const double lo = bin_log_edge(b), hi = bin_log_edge(b + 1);
    const double frac = hist[b] ? (double)(rank - before) / (double)hist[b] : 1.0;
    return (lo + (hi - lo) * frac - mu) / sigma;
}

typedef struct {
    double sparsity; /* zero fraction of the whole tensor predicted at the layer's threshold */
    double cosine;   /* predicted cosine similarity at that threshold (1 if not defined)      */
    double k;        /* truncation point used, in units of sigma                               */
    uint32_t status; /* bit 0: the threshold was lowered to keep the minimum cosine similarity;
                        bit 1: the compensating sparsity hit the cap                           */
    uint32_t reserved;
} orc_alloc_t;

static double whole_tensor_sparsity(const orc_stats_t *st, const orc_prune_params_t *p)
{
    const double zero_frac = st->n ? 1.0 - (double)st->nnz / (double)st->n : 0.0;
    return zero_frac + (1.0 - zero_frac) * (p->alpha > 0.0f ? p->s_pred : 0.0);
}

/* Heterogeneous allocation (appendix "Heterogeneous algorithm").  Layers are given in the order
 * of the backward pass, deepest first.  For each of the first n_deep layers the threshold for the
 * overall sparsity is computed; if the predicted cosine similarity falls short of the layer's
 * minimum, the threshold is lowered until it is met.  The sparsity those layers lose is made up by
 * the remaining layers, weighted by element counts, so that the element-weighted mean stays at
 * the overall sparsity -- but never above max_sparsity.  hists: n_layers x 2048 counts, or NULL. */
void orc_sparsity_allocate(const orc_stats_t *stats, const uint64_t *hists, int n_layers,
                           double overall_sparsity, int n_deep, const double *min_cosine,
                           double max_sparsity, double quantile, int alpha_dtype,
                           orc_prune_params_t *p_out, orc_alloc_t *a_out)
{
    double total = 0.0, deep_elems = 0.0, deep_zeros = 0.0;
    for (int i = 0; i < n_layers; ++i) total += (double)stats[i].n;
    if (n_deep > n_layers) n_deep = n_layers;
    for (int i = 0; i < n_layers; ++i) {
        const orc_stats_t *st = &stats[i];
        memset(&a_out[i], 0, sizeof a_out[i]);
        double target = overall_sparsity;
        if (i >= n_deep) {
            const double rest = total - deep_elems;
            target = rest > 0.0 ? (overall_sparsity * total - deep_zeros) / rest : overall_sparsity;
            if (target > max_sparsity) {
                target = max_sparsity;
                a_out[i].status |= 2u;
            }
            if (target < 0.0) target = 0.0;
        }
        orc_threshold(st, target, alpha_dtype, &p_out[i]);
        const int fitted = st->nnz != 0 && st->sigma >= 1e-12;
        const double k = fitted ? orc_truncation_k(hists ? hists + (size_t)i * ORC_HIST_BINS : NULL,
                                                   st->mu, st->sigma, quantile)
                                : 0.0;
        a_out[i].k = k;
        a_out[i].cosine = 1.0;
        if (fitted && p_out[i].alpha > 0.0f) {
            const double c = k * st->sigma;
            double L = log((double)p_out[i].alpha) - st->mu;
            if (i < n_deep && orc_cosine_similarity(st->sigma, L, c) < min_cosine[i]) {
                /* lower the threshold to the one that just keeps the minimum similarity */
                L = orc_log_alpha_for_cosine(st->sigma, c, min_cosine[i]);
                double alpha = exp(st->mu + L);
                float af = alpha >= (double)FLT_MAX ? FLT_MAX : (float)alpha;
                af = round_alpha(af, alpha_dtype);
                p_out[i].alpha = af;
                p_out[i].s_pred = af > 0.0f ? orc_sparsity_of_alpha(st->mu, st->sigma, (double)af) : 0.0;
                p_out[i].s_eff = p_out[i].s_pred;
                a_out[i].status |= 1u;
                L = af > 0.0f ? log((double)af) - st->mu : L;
            }
            if (p_out[i].alpha > 0.0f) a_out[i].cosine = orc_cosine_similarity(st->sigma, L, c);
        }
        a_out[i].sparsity = whole_tensor_sparsity(st, &p_out[i]);
        if (i < n_deep) {
            deep_elems += (double)st->n;
            deep_zeros += (double)st->n * a_out[i].sparsity;
        }
    }
}

/* ------------------------------------------------------------------------------------------
 * Stochastic underflow.  Section 4.1 sends every magnitude below the smallest representable one,
 * 2^(E_min + s) with E_min = 1 - 2^(e-1), to zero; the stochastic pruning operator of Section 5
 * with alpha equal to that smallest magnitude sends it to 0 or +-alpha with the probabilities
 * that keep the mean instead.  The threshold to use is therefore the larger of the pruning
 * threshold (0 if there is none) and 2^(E_min + s); status bit 16 reports that the given
 * threshold was below the format's range.  A floor below the normal range of the element type
 * cannot be expressed and is dropped.
 * ------------------------------------------------------------------------------------------ */
/* Composition of the two operators (pruning first, then the quantizer of Section 4.1): every
 * survivor of pruning with magnitude at most alpha comes out as +-alpha, and the quantizer sends a
 * magnitude below 2^(E_min + s), E_min = 1 - 2^(e-1), to zero.  So when 0 < alpha < 2^(E_min + s)
 * everything pruning touched is lost; that condition is reported as status bit 16 of the pruning
 * parameters.  Returns 1 if it holds. */
int orc_alpha_below_fp_range(float alpha, int e_bits, int scale_exp)
{
    const int emin = 1 - (1 << (e_bits - 1));
    return alpha > 0.0f && (double)alpha < ldexp(1.0, emin + scale_exp);
}

void orc_threshold_floor(int e_bits, int scale_exp, const orc_prune_params_t *in, int alpha_dtype,
                         orc_prune_params_t *out)
{
    (void)alpha_dtype; /* a power of two in the normal range is exact in both element types */
    if (in) *out = *in; else memset(out, 0, sizeof *out);
    const int k = 1 - (1 << (e_bits - 1)) + scale_exp;
    if (k < -126 || k > 127) return;
    const float floor_alpha = (float)ldexp(1.0, k);
    if (out->alpha < floor_alpha) {
        out->alpha = floor_alpha;
        out->status |= 16u;
    }
}

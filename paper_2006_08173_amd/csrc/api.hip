// C interface of the library (see include/lgn.h): argument checks and kernel launches only.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>

#include <atomic>

#include "launch.hpp"

namespace lgn {

// ---- tuning knobs: process-wide, lock-free ---------------------------------------------------
namespace {
constexpr int kKnobs = 5;
constexpr long kKnobDefault[kKnobs] = {224, 0, 0, 1024, 0};
constexpr long kKnobMin[kKnobs] = {0, 0, 0, 1, 0};
constexpr long kKnobMax[kKnobs] = {4096, 8, 4096, 1024, 1};
std::atomic<long> g_knob[kKnobs] = {{224}, {0}, {0}, {1024}, {0}};
std::atomic<int> g_cus[64];  // zero = not yet asked
}  // namespace

long tuning(int knob) { return knob >= 0 && knob < kKnobs ? g_knob[knob].load(std::memory_order_relaxed) : -1; }

int set_tuning(int knob, long value)
{
    if (knob < 0 || knob >= kKnobs) return -1;
    if (value < 0) value = kKnobDefault[knob];
    if (value < kKnobMin[knob] || value > kKnobMax[knob]) return -1;
    g_knob[knob].store(value, std::memory_order_relaxed);
    return 0;
}

int device_cus()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    int v = g_cus[dev].load(std::memory_order_relaxed);
    if (v) return v;
    int q = 0;
    v = hipDeviceGetAttribute(&q, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && q > 0 ? q : 256;
    g_cus[dev].store(v, std::memory_order_relaxed);  // every thread would store the same value
    return v;
}

}  // namespace lgn

namespace {

thread_local char g_err[256] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

int device_fail(const char *what, hipError_t e)
{
    return fail(LGN_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
}

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

bool dtype_ok(int d) { return d == LGN_F32 || d == LGN_BF16 || d == LGN_F16; }

int check_stats_args(const void *g, uint64_t n, int dtype, const lgn_stats_t *out, const void *ws,
                     size_t ws_bytes)
{
    if (!dtype_ok(dtype)) return fail(LGN_ERR_UNSUPPORTED, "unknown dtype %d", dtype);
    if (!out) return fail(LGN_ERR_INVALID_ARG, "null stats pointer");
    if (!aligned(out, 8)) return fail(LGN_ERR_INVALID_ARG, "stats struct not 8-byte aligned");
    if (n && !g) return fail(LGN_ERR_INVALID_ARG, "null tensor pointer");
    if (!aligned(g, 16)) return fail(LGN_ERR_INVALID_ARG, "input tensor not 16-byte aligned");
    if (n > (1ull << 60)) return fail(LGN_ERR_INVALID_ARG, "n too large");
    if (!ws || ws_bytes < lgn::stats_workspace_bytes())
        return fail(LGN_ERR_WORKSPACE, "workspace missing or smaller than %zu bytes",
                    lgn::stats_workspace_bytes());
    if (!aligned(ws, 8)) return fail(LGN_ERR_WORKSPACE, "workspace not 8-byte aligned");
    return LGN_OK;
}

int check_mask_args(const void *mask, int mask_kind, uint64_t n)
{
    if (mask_kind != LGN_MASK_NONE && mask_kind != LGN_MASK_SAME_DTYPE && mask_kind != LGN_MASK_U8)
        return fail(LGN_ERR_UNSUPPORTED, "unknown mask kind %d", mask_kind);
    if (mask_kind != LGN_MASK_NONE && n && (!mask || !aligned(mask, 16)))
        return fail(LGN_ERR_INVALID_ARG, "mask null or not 16-byte aligned");
    return LGN_OK;
}

int check_threshold_args(double target_sparsity, int alpha_dtype)
{
    if (!dtype_ok(alpha_dtype)) return fail(LGN_ERR_UNSUPPORTED, "unknown alpha dtype %d", alpha_dtype);
    if (!(target_sparsity >= 0.0 && target_sparsity < 1.0))
        return fail(LGN_ERR_INVALID_ARG, "target sparsity %g outside [0, 1)", target_sparsity);
    return LGN_OK;
}

// Standard normal quantile of the scale rule's probability.  It depends on an argument of the
// call only, not on the tensor, so it is evaluated here instead of in the last workgroup of the
// statistics pass, where every microsecond is on the critical path of the next launch.  A
// rational first guess (Abramowitz & Stegun 26.2.23) polished by Newton steps on the tail
// probability, which keeps full relative accuracy in both tails.
double scale_rule_z(int scale_mode, double q)
{
    if (scale_mode != LGN_SCALE_QUANTILE) return 0.0;
    const bool upper = q > 0.5;
    const double p = upper ? 1.0 - q : q;  // tail probability, 0 < p <= 0.5 (checked by the caller)
    const double t = sqrt(-2.0 * log(p));
    double z = t - (2.515517 + 0.802853 * t + 0.010328 * t * t) /
                       (1.0 + 1.432788 * t + 0.189269 * t * t + 0.001308 * t * t * t);
    for (int it = 0; it < 8; ++it) {
        const double qz = 0.5 * erfc(z / 1.41421356237309504880168872421);
        const double pdf = exp(-0.5 * z * z) * 0.398942280401432677939946059934;
        const double step = (qz - p) / pdf;
        z += step;
        if (fabs(step) <= 1e-16 * fmax(1.0, fabs(z))) break;
    }
    return upper ? z : -z;
}

int check_fp_args(int n_bits, int e_bits, int scale_mode, double scale_arg, int sigma_units)
{
    if (n_bits < 2 || n_bits > 8) return fail(LGN_ERR_INVALID_ARG, "n_bits %d outside [2, 8]", n_bits);
    if (e_bits != -1 && (e_bits < 1 || e_bits > n_bits - 1))
        return fail(LGN_ERR_INVALID_ARG, "e_bits %d outside [1, %d]", e_bits, n_bits - 1);
    if (scale_mode != LGN_SCALE_QUANTILE && scale_mode != LGN_SCALE_MAX && scale_mode != LGN_SCALE_CENTER)
        return fail(LGN_ERR_UNSUPPORTED, "unknown scale mode %d", scale_mode);
    if (scale_mode == LGN_SCALE_QUANTILE && !(scale_arg > 0.0 && scale_arg < 1.0))
        return fail(LGN_ERR_INVALID_ARG, "quantile %g outside (0, 1)", scale_arg);
    if (sigma_units != LGN_SIGMA_PAPER_LITERAL && sigma_units != LGN_SIGMA_BASE2)
        return fail(LGN_ERR_UNSUPPORTED, "unknown sigma units %d", sigma_units);
    return LGN_OK;
}

// Arguments of the one-launch statistics + solvers form beyond those of lgn_stats.
int check_solve_args(const void *mask, int mask_kind, uint64_t n, double target_sparsity, int alpha_dtype,
                     int n_bits, int e_bits, int scale_mode, double scale_arg, int sigma_units,
                     const lgn_prune_params_t *p_out, const lgn_fp_params_t *f_out, bool *want_p)
{
    if (int rc = check_mask_args(mask, mask_kind, n)) return rc;
    *want_p = target_sparsity >= 0.0 || target_sparsity != target_sparsity;
    if (*want_p) {
        if (int rc = check_threshold_args(target_sparsity, alpha_dtype)) return rc;
        if (!p_out || !aligned(p_out, 8))
            return fail(LGN_ERR_INVALID_ARG, "prune params struct null or not 8-byte aligned");
    }
    if (n_bits != 0) {
        if (int rc = check_fp_args(n_bits, e_bits, scale_mode, scale_arg, sigma_units)) return rc;
        if (!f_out || !aligned(f_out, 8))
            return fail(LGN_ERR_INVALID_ARG, "fp params struct null or not 8-byte aligned");
    }
    return LGN_OK;
}

int check_stream_common(const void *g, uint64_t n, int dtype, const void *out, int out_kind)
{
    if (!dtype_ok(dtype)) return fail(LGN_ERR_UNSUPPORTED, "unknown dtype %d", dtype);
    if (out_kind != LGN_OUT_VALUE && out_kind != LGN_OUT_CODE8 && out_kind != LGN_OUT_PACKED)
        return fail(LGN_ERR_UNSUPPORTED, "unknown out_kind %d", out_kind);
    if (n == 0) return LGN_OK;
    if (!g || !out) return fail(LGN_ERR_INVALID_ARG, "null tensor pointer");
    if (!aligned(g, 16)) return fail(LGN_ERR_INVALID_ARG, "input tensor not 16-byte aligned");
    if (!aligned(out, out_kind == LGN_OUT_VALUE ? 16 : 4))
        return fail(LGN_ERR_INVALID_ARG, "output not %d-byte aligned", out_kind == LGN_OUT_VALUE ? 16 : 4);
    if (n > (1ull << 60)) return fail(LGN_ERR_INVALID_ARG, "n too large");
    return LGN_OK;
}

}  // namespace

extern "C" {

size_t lgn_workspace_bytes(uint64_t, int) { return lgn::stats_workspace_bytes(); }

size_t lgn_packed_bytes(uint64_t n, int n_bits) { return (size_t)((n * (uint64_t)n_bits + 7) / 8); }

const char *lgn_last_error(void) { return g_err; }

int lgn_version(void) { return LGN_VERSION; }

int lgn_set_tuning(int knob, long value)
{
    if (lgn::set_tuning(knob, value) != 0)
        return fail(LGN_ERR_INVALID_ARG, "tuning knob %d cannot take the value %ld", knob, value);
    return LGN_OK;
}

long lgn_get_tuning(int knob) { return lgn::tuning(knob); }

int lgn_workspace_init(void *ws, size_t ws_bytes, void *stream)
{
    if (!ws || ws_bytes < lgn::stats_workspace_bytes())
        return fail(LGN_ERR_WORKSPACE, "workspace missing or smaller than %zu bytes",
                    lgn::stats_workspace_bytes());
    if (!aligned(ws, 8)) return fail(LGN_ERR_WORKSPACE, "workspace not 8-byte aligned");
    const hipError_t e = lgn::launch_workspace_init(ws, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LGN_OK : device_fail("lgn_workspace_init", e);
}

int lgn_stats(const void *g, uint64_t n, int dtype, lgn_stats_t *out, void *ws, size_t ws_bytes,
              void *stream)
{
    if (int rc = check_stats_args(g, n, dtype, out, ws, ws_bytes)) return rc;
    const hipError_t e = lgn::launch_stats(g, nullptr, LGN_MASK_NONE, n, dtype, out, ws,
                                           static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LGN_OK : device_fail("lgn_stats", e);
}

int lgn_stats_masked(const void *g, const void *mask, int mask_kind, uint64_t n, int dtype,
                     lgn_stats_t *out, void *ws, size_t ws_bytes, void *stream)
{
    if (int rc = check_stats_args(g, n, dtype, out, ws, ws_bytes)) return rc;
    if (int rc = check_mask_args(mask, mask_kind, n)) return rc;
    const hipError_t e = lgn::launch_stats(g, mask, mask_kind, n, dtype, out, ws,
                                           static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LGN_OK : device_fail("lgn_stats_masked", e);
}

int lgn_stats_solve(const void *g, const void *mask, int mask_kind, uint64_t n, int dtype,
                    double target_sparsity, int alpha_dtype, int n_bits, int e_bits, int scale_mode,
                    double scale_arg, int sigma_units, lgn_stats_t *st_out,
                    lgn_prune_params_t *p_out, lgn_fp_params_t *f_out, void *ws, size_t ws_bytes,
                    void *stream)
{
    if (int rc = check_stats_args(g, n, dtype, st_out, ws, ws_bytes)) return rc;
    bool want_p = false;
    if (int rc = check_solve_args(mask, mask_kind, n, target_sparsity, alpha_dtype, n_bits, e_bits, scale_mode,
                                  scale_arg, sigma_units, p_out, f_out, &want_p))
        return rc;
    const hipError_t e = lgn::launch_stats_solve(
        g, mask, mask_kind, n, dtype, want_p ? target_sparsity : -1.0, alpha_dtype, n_bits, e_bits, scale_mode,
        n_bits ? scale_rule_z(scale_mode, scale_arg) : 0.0, sigma_units, st_out, want_p ? p_out : nullptr,
        n_bits ? f_out : nullptr, ws, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LGN_OK : device_fail("lgn_stats_solve", e);
}

int lgn_stats_solve_static(const void *g, const void *mask, int mask_kind, uint64_t n, int dtype,
                           double target_sparsity, int alpha_dtype, int n_bits, int e_bits,
                           int scale_mode, double scale_arg, int sigma_units, lgn_stats_t *st_out,
                           lgn_prune_params_t *p_out, lgn_fp_params_t *f_out, void *stream)
{
    if (n > LGN_STATIC_MAX_ELEMENTS)
        return fail(LGN_ERR_INVALID_ARG, "n = %llu exceeds LGN_STATIC_MAX_ELEMENTS = %llu of the built-in scratch array",
                    (unsigned long long)n, (unsigned long long)LGN_STATIC_MAX_ELEMENTS);
    // the workspace checks do not apply: any non-null aligned pointer passes them
    alignas(16) static const char none[16] = {};
    if (int rc = check_stats_args(g, n, dtype, st_out, none, lgn::stats_workspace_bytes())) return rc;
    bool want_p = false;
    if (int rc = check_solve_args(mask, mask_kind, n, target_sparsity, alpha_dtype, n_bits, e_bits, scale_mode,
                                  scale_arg, sigma_units, p_out, f_out, &want_p))
        return rc;
    const hipError_t e = lgn::launch_stats_solve_static(
        g, mask, mask_kind, n, dtype, want_p ? target_sparsity : -1.0, alpha_dtype, n_bits, e_bits, scale_mode,
        n_bits ? scale_rule_z(scale_mode, scale_arg) : 0.0, sigma_units, st_out, want_p ? p_out : nullptr,
        n_bits ? f_out : nullptr, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LGN_OK : device_fail("lgn_stats_solve_static", e);
}

size_t lgn_static_scratch_bytes(void) { return lgn::stats_scratch_bytes(); }

int lgn_threshold(const lgn_stats_t *st, double target_sparsity, int alpha_dtype,
                  lgn_prune_params_t *out, void *stream)
{
    if (!st || !out) return fail(LGN_ERR_INVALID_ARG, "null struct pointer");
    if (!aligned(st, 8) || !aligned(out, 8)) return fail(LGN_ERR_INVALID_ARG, "struct not 8-byte aligned");
    if (int rc = check_threshold_args(target_sparsity, alpha_dtype)) return rc;
    const hipError_t e = lgn::launch_threshold(st, target_sparsity, alpha_dtype, out,
                                               static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LGN_OK : device_fail("lgn_threshold", e);
}

int lgn_threshold_floor(const lgn_fp_params_t *f, const lgn_prune_params_t *in, lgn_prune_params_t *out,
                        void *stream)
{
    if (!f || !out) return fail(LGN_ERR_INVALID_ARG, "null struct pointer");
    if (!aligned(f, 8) || !aligned(in, 8) || !aligned(out, 8))
        return fail(LGN_ERR_INVALID_ARG, "struct not 8-byte aligned");
    const hipError_t e = lgn::launch_threshold_floor(f, in, out, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LGN_OK : device_fail("lgn_threshold_floor", e);
}

int lgn_fp_params(const lgn_stats_t *st, int n_bits, int e_bits, int scale_mode, double scale_arg,
                  int sigma_units, lgn_fp_params_t *out, void *stream)
{
    if (!st || !out) return fail(LGN_ERR_INVALID_ARG, "null struct pointer");
    if (!aligned(st, 8) || !aligned(out, 8)) return fail(LGN_ERR_INVALID_ARG, "struct not 8-byte aligned");
    if (int rc = check_fp_args(n_bits, e_bits, scale_mode, scale_arg, sigma_units)) return rc;
    const hipError_t e = lgn::launch_fp_params(st, n_bits, e_bits, scale_mode,
                                               scale_rule_z(scale_mode, scale_arg), sigma_units, out,
                                               static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LGN_OK : device_fail("lgn_fp_params", e);
}

int lgn_prune(const void *g, uint64_t n, int dtype, const lgn_prune_params_t *p, uint64_t seed,
              uint64_t elem_offset, void *out, void *stream)
{
    if (int rc = check_stream_common(g, n, dtype, out, LGN_OUT_VALUE)) return rc;
    if (!p) return fail(LGN_ERR_INVALID_ARG, "null prune params");
    lgn::StreamArgs a = {g, out, n, elem_offset, p, nullptr, (uint32_t)seed, (uint32_t)(seed >> 32)};
    const hipError_t e = lgn::launch_stream(dtype, true, false, 0, LGN_OUT_VALUE, a,
                                            static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LGN_OK : device_fail("lgn_prune", e);
}

int lgn_fp_quantize(const void *g, uint64_t n, int dtype, const lgn_fp_params_t *f, int rounding,
                    uint64_t seed, uint64_t elem_offset, void *out, int out_kind, void *stream)
{
    if (int rc = check_stream_common(g, n, dtype, out, out_kind)) return rc;
    if (!f) return fail(LGN_ERR_INVALID_ARG, "null fp params");
    if (rounding != LGN_ROUND_NEAREST_EVEN && rounding != LGN_ROUND_STOCHASTIC)
        return fail(LGN_ERR_UNSUPPORTED, "unknown rounding %d", rounding);
    lgn::StreamArgs a = {g, out, n, elem_offset, nullptr, f, (uint32_t)seed, (uint32_t)(seed >> 32)};
    const hipError_t e = lgn::launch_stream(dtype, false, true, rounding, out_kind, a,
                                            static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LGN_OK : device_fail("lgn_fp_quantize", e);
}

int lgn_prune_quantize_fused(const void *g, uint64_t n, int dtype, const lgn_prune_params_t *p,
                             const lgn_fp_params_t *f, int rounding, uint64_t seed,
                             uint64_t elem_offset, void *out, int out_kind, void *stream)
{
    if (int rc = check_stream_common(g, n, dtype, out, out_kind)) return rc;
    if (!p || !f) return fail(LGN_ERR_INVALID_ARG, "null params");
    if (rounding != LGN_ROUND_NEAREST_EVEN && rounding != LGN_ROUND_STOCHASTIC)
        return fail(LGN_ERR_UNSUPPORTED, "unknown rounding %d", rounding);
    lgn::StreamArgs a = {g, out, n, elem_offset, p, f, (uint32_t)seed, (uint32_t)(seed >> 32)};
    const hipError_t e = lgn::launch_stream(dtype, true, true, rounding, out_kind, a,
                                            static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LGN_OK : device_fail("lgn_prune_quantize_fused", e);
}

int lgn_batch_stats_solve(const lgn_batch_item_t *items, int count, int dtype, int alpha_dtype,
                          int scale_mode, double scale_arg, int sigma_units, void *ws, size_t ws_bytes,
                          void *stream)
{
    if (count < 0) return fail(LGN_ERR_INVALID_ARG, "negative count");
    if (count == 0) return LGN_OK;
    if (!items) return fail(LGN_ERR_INVALID_ARG, "null item array");
    bool any_format = false;
    for (int i = 0; i < count; ++i) {
        const lgn_batch_item_t &it = items[i];
        int rc = check_stats_args(it.g, it.n, dtype, it.st, ws, ws_bytes);
        bool want_p = false;
        if (!rc)
            rc = check_solve_args(nullptr, LGN_MASK_NONE, it.n, it.target_sparsity, alpha_dtype, it.n_bits, it.e_bits,
                                  scale_mode, scale_arg, sigma_units, it.p, it.f, &want_p);
        if (rc) {
            char first[200];
            snprintf(first, sizeof first, "%s", g_err);
            return fail(rc, "item %d: %s", i, first);
        }
        any_format = any_format || it.n_bits != 0;
    }
    const hipError_t e = lgn::launch_batch_stats_solve(items, count, dtype, alpha_dtype, scale_mode,
                                                       any_format ? scale_rule_z(scale_mode, scale_arg) : 0.0,
                                                       sigma_units, ws, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LGN_OK : device_fail("lgn_batch_stats_solve", e);
}

int lgn_batch_prune_quantize_fused(const lgn_batch_item_t *items, int count, int dtype, int rounding,
                                   int out_kind, void *stream)
{
    if (count < 0) return fail(LGN_ERR_INVALID_ARG, "negative count");
    if (count == 0) return LGN_OK;
    if (!items) return fail(LGN_ERR_INVALID_ARG, "null item array");
    if (rounding != LGN_ROUND_NEAREST_EVEN && rounding != LGN_ROUND_STOCHASTIC)
        return fail(LGN_ERR_UNSUPPORTED, "unknown rounding %d", rounding);
    for (int i = 0; i < count; ++i) {
        const lgn_batch_item_t &it = items[i];
        int rc = check_stream_common(it.g, it.n, dtype, it.out, out_kind);
        if (!rc && (!it.p || !it.f)) rc = fail(LGN_ERR_INVALID_ARG, "null params");
        if (rc) {
            char first[200];
            snprintf(first, sizeof first, "%s", g_err);
            return fail(rc, "item %d: %s", i, first);
        }
    }
    const hipError_t e = lgn::launch_batch_stream(items, count, dtype, rounding, out_kind,
                                                  static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LGN_OK : device_fail("lgn_batch_prune_quantize_fused", e);
}

int lgn_dequantize(const void *codes, uint64_t n, int in_kind, const lgn_fp_params_t *f, int dtype,
                   void *out, void *stream)
{
    if (!dtype_ok(dtype)) return fail(LGN_ERR_UNSUPPORTED, "unknown dtype %d", dtype);
    if (in_kind != LGN_OUT_CODE8 && in_kind != LGN_OUT_PACKED)
        return fail(LGN_ERR_UNSUPPORTED, "codes must be CODE8 or PACKED");
    if (n == 0) return LGN_OK;
    if (!codes || !out || !f) return fail(LGN_ERR_INVALID_ARG, "null pointer");
    const hipError_t e = lgn::launch_dequant(codes, n, in_kind, f, dtype, out,
                                             static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LGN_OK : device_fail("lgn_dequantize", e);
}

size_t lgn_prefix_table_bytes(uint64_t n)
{
    const uint64_t nchunks = (n + LGN_PREFIX_CHUNK - 1) / LGN_PREFIX_CHUNK;
    // chunk table, the encoder's scratch entries, sixteen 16-bit sub-block lengths per chunk
    return (size_t)((nchunks + 2 + LGN_PREFIX_MAX_BLOCKS) * 8 + nchunks * 32);
}

size_t lgn_prefix_bound_bytes(uint64_t n, int width)
{
    if (width < 2 || width > 32) return 0;
    const uint64_t words_per_chunk = ((uint64_t)LGN_PREFIX_CHUNK * (2 + (uint64_t)width) + 31) / 32;
    return (size_t)((n + LGN_PREFIX_CHUNK - 1) / LGN_PREFIX_CHUNK * words_per_chunk * 4);
}

static int prefix_width_class(int in_kind, int dtype, const lgn_fp_params_t *f)
{
    if (in_kind == LGN_OUT_CODE8) {
        if (!f) return fail(LGN_ERR_INVALID_ARG, "codes need the fp params they were made with") - 100;
        return 0;
    }
    if (in_kind != LGN_OUT_VALUE) return fail(LGN_ERR_UNSUPPORTED, "prefix code takes VALUE or CODE8 input") - 100;
    if (!dtype_ok(dtype)) return fail(LGN_ERR_UNSUPPORTED, "unknown dtype %d", dtype) - 100;
    return dtype == LGN_F32 ? 2 : 1;
}

int lgn_prefix_encode(const void *in, uint64_t n, int in_kind, int dtype, const lgn_prune_params_t *p,
                      const lgn_fp_params_t *f, void *out, size_t out_capacity, uint64_t *table,
                      void *stream)
{
    const int wc = prefix_width_class(in_kind, dtype, f);
    if (wc < 0) return wc + 100;
    if (!table || !aligned(table, 8)) return fail(LGN_ERR_INVALID_ARG, "table null or not 8-byte aligned");
    if (n > (1ull << 60)) return fail(LGN_ERR_INVALID_ARG, "n too large");
    if (n && (!in || !aligned(in, 16))) return fail(LGN_ERR_INVALID_ARG, "input null or not 16-byte aligned");
    if (out_capacity && (!out || !aligned(out, 4))) return fail(LGN_ERR_INVALID_ARG, "stream buffer null or not 4-byte aligned");
    const hipError_t e = lgn::launch_prefix_encode(wc, dtype, in, n, p, f, out, out_capacity / 4, table,
                                                   static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LGN_OK : device_fail("lgn_prefix_encode", e);
}

int lgn_prefix_decode(const void *in, const uint64_t *table, uint64_t n, int in_kind, int dtype,
                      const lgn_prune_params_t *p, const lgn_fp_params_t *f, void *out, void *stream)
{
    const int wc = prefix_width_class(in_kind, dtype, f);
    if (wc < 0) return wc + 100;
    if (!table || !aligned(table, 8)) return fail(LGN_ERR_INVALID_ARG, "table null or not 8-byte aligned");
    if (n > (1ull << 60)) return fail(LGN_ERR_INVALID_ARG, "n too large");
    if (n && (!in || !out || !aligned(in, 4) || !aligned(out, 16)))
        return fail(LGN_ERR_INVALID_ARG, "null or misaligned buffer (stream 4, output 16 bytes)");
    const hipError_t e = lgn::launch_prefix_decode(wc, dtype, in, table, n, p, f, out,
                                                   static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LGN_OK : device_fail("lgn_prefix_decode", e);
}

int lgn_log_histogram(const void *g, uint64_t n, int dtype, uint64_t *hist, void *stream)
{
    if (!dtype_ok(dtype)) return fail(LGN_ERR_UNSUPPORTED, "unknown dtype %d", dtype);
    if (!hist || !aligned(hist, 8)) return fail(LGN_ERR_INVALID_ARG, "histogram null or not 8-byte aligned");
    if (n && (!g || !aligned(g, 16))) return fail(LGN_ERR_INVALID_ARG, "input null or not 16-byte aligned");
    if (n > (1ull << 60)) return fail(LGN_ERR_INVALID_ARG, "n too large");
    const hipError_t e = lgn::launch_log_histogram(g, n, dtype, hist,
                                                   static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LGN_OK : device_fail("lgn_log_histogram", e);
}

int lgn_sparsity_allocate(const lgn_stats_t *stats, const uint64_t *hists, int n_layers,
                          double overall_sparsity, int n_deep, const double *min_cosine,
                          double max_sparsity, double quantile, int alpha_dtype,
                          lgn_prune_params_t *p_out, lgn_alloc_t *a_out, void *stream)
{
    if (n_layers < 0 || n_layers > (1 << 20)) return fail(LGN_ERR_INVALID_ARG, "n_layers %d out of range", n_layers);
    if (n_layers == 0) return LGN_OK;
    if (!stats || !p_out || !a_out) return fail(LGN_ERR_INVALID_ARG, "null struct pointer");
    if (!aligned(stats, 8) || !aligned(p_out, 8) || !aligned(a_out, 8) || !aligned(hists, 8) || !aligned(min_cosine, 8))
        return fail(LGN_ERR_INVALID_ARG, "pointer not 8-byte aligned");
    if (n_deep < 0) return fail(LGN_ERR_INVALID_ARG, "negative n_deep");
    if (n_deep > 0 && !min_cosine) return fail(LGN_ERR_INVALID_ARG, "deep layers need their minimum cosine similarities");
    if (int rc = check_threshold_args(overall_sparsity, alpha_dtype)) return rc;
    if (!(max_sparsity >= 0.0 && max_sparsity < 1.0))
        return fail(LGN_ERR_INVALID_ARG, "max_sparsity %g outside [0, 1)", max_sparsity);
    if (!(quantile > 0.0 && quantile < 1.0)) return fail(LGN_ERR_INVALID_ARG, "quantile %g outside (0, 1)", quantile);
    const hipError_t e = lgn::launch_sparsity_allocate(stats, hists, n_layers, overall_sparsity, n_deep,
                                                       min_cosine, max_sparsity, quantile, alpha_dtype,
                                                       p_out, a_out, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LGN_OK : device_fail("lgn_sparsity_allocate", e);
}

}  // extern "C"

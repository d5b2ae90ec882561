// Kernels of lgn_threshold and lgn_fp_params: one wave each (see solver_device.hpp).
#include "launch.hpp"
#include "solver_device.hpp"

namespace lgn {

__global__ __launch_bounds__(kWave) void threshold_kernel(const lgn_stats_t *__restrict__ st,
                                                          double target, int alpha_dtype,
                                                          lgn_prune_params_t *__restrict__ out)
{
    threshold_body<true>(st, target, alpha_dtype, out);
}

__global__ __launch_bounds__(kWave) void fp_params_kernel(const lgn_stats_t *__restrict__ st,
                                                          int n_bits, int e_fixed, int scale_mode,
                                                          double scale_z, int sigma_units,
                                                          lgn_fp_params_t *__restrict__ out)
{
    fp_params_body(st, n_bits, e_fixed, scale_mode, scale_z, sigma_units, out);
}

// Stochastic underflow: the pruning threshold raised to the smallest magnitude the format can
// represent, 2^(E_min + s) with E_min = 1 - 2^(e-1) (Section 4.1), so that the pruning operator of
// Section 5 sends smaller values to 0 or +-alpha with their mean kept instead of flushing them.
__global__ __launch_bounds__(kWave) void threshold_floor_kernel(const lgn_fp_params_t *__restrict__ f,
                                                                const lgn_prune_params_t *in,
                                                                lgn_prune_params_t *out)
{
    if (threadIdx.x != 0) return;
    lgn_prune_params_t r;
    if (in) {
        r = *in;
    } else {
        r.alpha = 0.0f;
        r.status = 0u;
        r.s_eff = 0.0;
        r.s_pred = 0.0;
    }
    const int e = min(max(f->e_bits, 1), 7);
    const int k = 1 - (1 << (e - 1)) + f->scale_exp;
    if (k >= -126 && k <= 127) {  // otherwise the floor is not a normal number of the element type
        const float floor_alpha = __uint_as_float((uint32_t)(k + 127) << 23);
        if (r.alpha < floor_alpha) {
            r.alpha = floor_alpha;
            r.status |= LGN_ST_ALPHA_BELOW_FP_RANGE;
        }
    }
    *out = r;
}

hipError_t launch_threshold_floor(const lgn_fp_params_t *f, const lgn_prune_params_t *in,
                                  lgn_prune_params_t *out, hipStream_t stream)
{
    threshold_floor_kernel<<<1, kWave, 0, stream>>>(f, in, out);
    return hipGetLastError();
}

hipError_t launch_threshold(const lgn_stats_t *st, double target, int alpha_dtype,
                            lgn_prune_params_t *out, hipStream_t stream)
{
    threshold_kernel<<<1, kWave, 0, stream>>>(st, target, alpha_dtype, out);
    return hipGetLastError();
}

hipError_t launch_fp_params(const lgn_stats_t *st, int n_bits, int e_bits, int scale_mode,
                            double scale_z, int sigma_units, lgn_fp_params_t *out,
                            hipStream_t stream)
{
    fp_params_kernel<<<1, kWave, 0, stream>>>(st, n_bits, e_bits, scale_mode, scale_z,
                                              sigma_units, out);
    return hipGetLastError();
}

}  // namespace lgn

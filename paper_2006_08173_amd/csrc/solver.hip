// Kernels of lgn_threshold and lgn_fp_params: one wave each (see solver_device.hpp).
#include "solver_device.hpp"

namespace lgn {

__global__ __launch_bounds__(kWave) void threshold_kernel(const lgn_stats_t *__restrict__ st,
                                                          double target, int alpha_dtype,
                                                          lgn_prune_params_t *__restrict__ out)
{
    if (threadIdx.x == 0) threshold_body(st, target, alpha_dtype, out);
}

__global__ __launch_bounds__(kWave) void fp_params_kernel(const lgn_stats_t *__restrict__ st,
                                                          int n_bits, int e_fixed, int scale_mode,
                                                          double scale_arg, int sigma_units,
                                                          lgn_fp_params_t *__restrict__ out)
{
    fp_params_body(st, n_bits, e_fixed, scale_mode, scale_arg, sigma_units, out);
}

hipError_t launch_threshold(const lgn_stats_t *st, double target, int alpha_dtype,
                            lgn_prune_params_t *out, hipStream_t stream)
{
    threshold_kernel<<<1, kWave, 0, stream>>>(st, target, alpha_dtype, out);
    return hipGetLastError();
}

hipError_t launch_fp_params(const lgn_stats_t *st, int n_bits, int e_bits, int scale_mode,
                            double scale_arg, int sigma_units, lgn_fp_params_t *out,
                            hipStream_t stream)
{
    fp_params_kernel<<<1, kWave, 0, stream>>>(st, n_bits, e_bits, scale_mode, scale_arg,
                                              sigma_units, out);
    return hipGetLastError();
}

}  // namespace lgn

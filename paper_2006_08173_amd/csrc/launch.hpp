// Host-side declarations shared by the translation units of the library: the argument block of the
// streaming kernels, the launch functions api.hip calls, the tuning knobs and the per-device
// compute-unit count.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/lgn.h"

namespace lgn {

// By-value argument of every streaming kernel (stream_kernels.hpp).
struct StreamArgs {
    const void *g;
    void *out;
    uint64_t n;
    uint64_t elem_offset;
    const lgn_prune_params_t *p;
    const lgn_fp_params_t *f;
    uint32_t k0, k1;  // the two halves of the seed: the Philox key
};

// Tuning knobs (lgn_set_tuning); process-wide, read at every launch.
long tuning(int knob);
int set_tuning(int knob, long value);

// Compute units of the current device (cached per device; 256 if the query fails).
int device_cus();

hipError_t launch_stats(const void *g, const void *mask, int mask_kind, uint64_t n, int dtype,
                        lgn_stats_t *out, void *ws, hipStream_t stream);
size_t stats_workspace_bytes();
hipError_t launch_workspace_init(void *ws, hipStream_t stream);
hipError_t launch_stats_solve(const void *g, const void *mask, int mask_kind, uint64_t n, int dtype,
                              double target_sparsity, int alpha_dtype, int n_bits, int e_bits,
                              int scale_mode, double scale_z, int sigma_units, lgn_stats_t *st,
                              lgn_prune_params_t *p, lgn_fp_params_t *f, void *ws,
                              hipStream_t stream);
// The same launch on the library's own per-device scratch array (no workspace argument).
hipError_t launch_stats_solve_static(const void *g, const void *mask, int mask_kind, uint64_t n,
                                     int dtype, double target_sparsity, int alpha_dtype, int n_bits,
                                     int e_bits, int scale_mode, double scale_z, int sigma_units,
                                     lgn_stats_t *st, lgn_prune_params_t *p, lgn_fp_params_t *f,
                                     hipStream_t stream);
size_t stats_scratch_bytes();
hipError_t launch_batch_stats_solve(const lgn_batch_item_t *items, int count, int dtype, int alpha_dtype,
                                    int scale_mode, double scale_z, int sigma_units, void *ws,
                                    hipStream_t stream);
hipError_t launch_batch_stream(const lgn_batch_item_t *items, int count, int dtype, int rounding,
                               int out_kind, hipStream_t stream);
hipError_t launch_threshold(const lgn_stats_t *st, double target, int alpha_dtype,
                            lgn_prune_params_t *out, hipStream_t stream);
hipError_t launch_threshold_floor(const lgn_fp_params_t *f, const lgn_prune_params_t *in,
                                  lgn_prune_params_t *out, hipStream_t stream);
hipError_t launch_fp_params(const lgn_stats_t *st, int n_bits, int e_bits, int scale_mode,
                            double scale_z, int sigma_units, lgn_fp_params_t *out,
                            hipStream_t stream);
hipError_t launch_stream(int dtype, bool prune, bool quant, int rounding, int out_kind,
                         const StreamArgs &args, hipStream_t stream);
hipError_t launch_dequant(const void *codes, uint64_t n, int in_kind, const lgn_fp_params_t *f,
                          int dtype, void *out, hipStream_t stream);
hipError_t launch_prefix_encode(int width_class, int dtype, const void *in, uint64_t n,
                                const lgn_prune_params_t *p, const lgn_fp_params_t *f, void *out,
                                uint64_t capacity_words, uint64_t *table, hipStream_t stream);
hipError_t launch_prefix_decode(int width_class, int dtype, const void *in, const uint64_t *table,
                                uint64_t n, const lgn_prune_params_t *p, const lgn_fp_params_t *f,
                                void *out, hipStream_t stream);
hipError_t launch_log_histogram(const void *g, uint64_t n, int dtype, uint64_t *hist,
                                hipStream_t stream);
hipError_t launch_sparsity_allocate(const lgn_stats_t *stats, const uint64_t *hists, int n_layers,
                                    double overall, int n_deep, const double *min_cosine,
                                    double max_sparsity, double quantile, int alpha_dtype,
                                    lgn_prune_params_t *p_out, lgn_alloc_t *a_out, hipStream_t stream);

}  // namespace lgn

// Heterogeneous sparsity allocation (appendix "Cosine similarity and heterogeneous stochastic
// pruning") and the histogram pass that feeds it.
//
//   lgn_log_histogram      counts of the finite non-zero magnitudes on a logarithmic grid, eight bins
//                          per binade: the bin is the top eleven bits of the fp32 magnitude pattern
//                          (exponent and three mantissa bits).  A high quantile of ln|g| read off
//                          it is the truncation point k sigma of the section "Neural gradients
//                          lognormal distributions are truncated" (the sample maximum is too noisy).
//   lgn_sparsity_allocate  one small workgroup: per layer the threshold for the overall sparsity,
//                          the closed-form cosine similarity at that threshold, a lower threshold
//                          where a deep layer's minimum similarity asks for it, and the
//                          compensating sparsity of the remaining layers (capped).
//
// Cosine similarity, per element and divided by e^{2 mu + 2 sigma^2}, with L = ln(alpha) - mu, the
// cut-off c = k sigma in the log domain and Phi the standard normal CDF:
//     xx = Phi((c - 2 s^2)/s)                                       E[x^2] = E[x T(x)]
//     tt = e^{L - 3 s^2 / 2} Phi((min(L,c) - s^2)/s) + [xx - Phi((L - 2 s^2)/s)]_+      E[T(x)^2]
//     cos = sqrt(xx / tt)
#include "launch.hpp"
#include "solver_device.hpp"

namespace lgn {

constexpr int kHistBins = LGN_HIST_BINS;

// ---- histogram ------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void hist_clear_kernel(unsigned long long *hist)
{
    for (int b = threadIdx.x; b < kHistBins; b += kBlock) hist[b] = 0ull;
}

__device__ __forceinline__ void hist_count(uint32_t *lds, uint32_t bits)
{
    const uint32_t a = bits & 0x7fffffffu;
    if (a != 0u && a < 0x7f800000u) atomicAdd(lds + (a >> 20), 1u);
}

template <int DTYPE>
__global__ __launch_bounds__(kBlock) void hist_kernel(const void *__restrict__ g, uint64_t n,
                                                      unsigned long long *hist)
{
    constexpr int EPV = DTYPE == LGN_F32 ? 4 : 8;
    constexpr uint64_t kFlushEvery = 1ull << 18;  // vectors per thread between flushes: counts stay < 2^32
    __shared__ uint32_t lds[kHistBins];
    for (int b = threadIdx.x; b < kHistBins; b += kBlock) lds[b] = 0u;
    __syncthreads();
    const uint64_t nvec = n / EPV;
    const uint64_t stride = (uint64_t)gridDim.x * kBlock;
    const uint4 *gv = reinterpret_cast<const uint4 *>(g);
    // every thread of the block runs the same number of rounds, so the barriers of a flush match
    const uint64_t rounds = (nvec + stride - 1) / stride;
    uint64_t since_flush = 0;
    for (uint64_t r = 0; r < rounds; ++r) {
        const uint64_t v = r * stride + (uint64_t)blockIdx.x * kBlock + threadIdx.x;
        if (v < nvec) {
            const uint4 x = load_stream16(gv + v);
            const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (DTYPE == LGN_F32) {
                    hist_count(lds, w[j]);
                } else {
                    uint32_t lo, hi;
                    widen_pair<DTYPE>(w[j], lo, hi);
                    hist_count(lds, lo);
                    hist_count(lds, hi);
                }
            }
        }
        if (++since_flush == kFlushEvery || r + 1 == rounds) {
            since_flush = 0;
            __syncthreads();
            for (int b = threadIdx.x; b < kHistBins; b += kBlock) {
                const uint32_t c = lds[b];
                if (c) atomicAdd(hist + b, (unsigned long long)c);
                lds[b] = 0u;
            }
            __syncthreads();
        }
    }
    // fewer than EPV elements at the end of the tensor
    if (blockIdx.x == 0 && threadIdx.x < (unsigned)EPV) {
        const uint64_t i = nvec * EPV + threadIdx.x;
        if (i < n) {
            const uint32_t a = load_elem<DTYPE>(g, i) & 0x7fffffffu;
            if (a != 0u && a < 0x7f800000u) atomicAdd(hist + (a >> 20), 1ull);
        }
    }
}

hipError_t launch_log_histogram(const void *g, uint64_t n, int dtype, uint64_t *hist,
                                hipStream_t stream)
{
    unsigned long long *h = reinterpret_cast<unsigned long long *>(hist);
    hist_clear_kernel<<<1, kBlock, 0, stream>>>(h);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || n == 0) return e;
    const uint64_t epv = dtype == LGN_F32 ? 4 : 8;
    uint64_t blocks = (n / epv + kBlock - 1) / kBlock;
    if (blocks < 1) blocks = 1;
    const uint64_t max_blocks = (uint64_t)device_cus() * 8;  // resident grid: eight workgroups per CU
    if (blocks > max_blocks) blocks = max_blocks;
    if (dtype == LGN_F32) hist_kernel<LGN_F32><<<(int)blocks, kBlock, 0, stream>>>(g, n, h);
    else if (dtype == LGN_BF16) hist_kernel<LGN_BF16><<<(int)blocks, kBlock, 0, stream>>>(g, n, h);
    else hist_kernel<LGN_F16><<<(int)blocks, kBlock, 0, stream>>>(g, n, h);
    return hipGetLastError();
}

// ---- scalar pieces of the allocation --------------------------------------------------------
__device__ double cosine_of_pruning(double sigma, double L, double c)
{
    const double s2 = sigma * sigma;
    const double xx = normal_cdf((c - 2.0 * s2) / sigma);
    const double small = exp(L - 1.5 * s2) * normal_cdf((fmin(L, c) - s2) / sigma);
    const double kept = fmax(xx - normal_cdf((L - 2.0 * s2) / sigma), 0.0);
    return sqrt(xx / (small + kept));
}

// Largest L whose similarity is still >= min_cosine (the similarity falls as L grows); bisection.
__device__ double log_alpha_for_cosine(double sigma, double c, double min_cosine)
{
    double lo = -40.0 * sigma - 2.0 * sigma * sigma - 50.0, hi = c;
    if (cosine_of_pruning(sigma, hi, c) >= min_cosine) return hi;
    for (int it = 0; it < 400; ++it) {
        const double mid = 0.5 * (lo + hi);
        if (cosine_of_pruning(sigma, mid, c) >= min_cosine) lo = mid; else hi = mid;
        if (hi - lo <= 1e-15 * fmax(1.0, fabs(mid))) break;
    }
    return 0.5 * (lo + hi);
}

// ln of the lower edge of histogram bin b >= 8
__device__ __forceinline__ double bin_log_edge(int b)
{
    return log(1.0 + (double)(b & 7) * 0.125) + (double)((b >> 3) - 127) * kLn2;
}

// k = (q-quantile of ln|g| - mu) / sigma from the histogram (linear in the logarithm inside the
// bin of the entry of rank ceil(q N)); the quantile of the fitted normal without a histogram.
__device__ double truncation_k(const uint64_t *hist, double mu, double sigma, double q)
{
    if (!hist) return normal_quantile(q);
    uint64_t total = 0;
    for (int b = 0; b < kHistBins; ++b) total += hist[b];
    if (total == 0 || !(sigma > 0.0)) return normal_quantile(q);
    uint64_t rank = (uint64_t)ceil(q * (double)total);
    rank = rank < 1 ? 1 : (rank > total ? total : rank);
    uint64_t before = 0;
    int b = 0;
    for (; b < kHistBins; ++b) {
        if (before + hist[b] >= rank) break;
        before += hist[b];
    }
    if (b < 8) b = 8;
    const double lo = bin_log_edge(b), hi = bin_log_edge(b + 1);
    const uint64_t in_bin = hist[b];
    const double frac = in_bin ? (double)(rank - before) / (double)in_bin : 1.0;
    return (lo + (hi - lo) * frac - mu) / sigma;
}

struct AllocArgs {
    const lgn_stats_t *stats;
    const uint64_t *hists;
    int n_layers, n_deep;
    double overall, max_sparsity, quantile;
    const double *min_cosine;
    int alpha_dtype;
    lgn_prune_params_t *p_out;
    lgn_alloc_t *a_out;
};

// One layer: threshold for `target`, lowered if the layer has a minimum similarity that it misses.
__device__ void allocate_layer(const AllocArgs &a, int i, double target, uint32_t status, bool deep)
{
    const lgn_stats_t *st = a.stats + i;
    lgn_prune_params_t *p = a.p_out + i;
    threshold_body<false>(st, target, a.alpha_dtype, p);
    lgn_alloc_t r;
    r.status = status;
    r.reserved = 0u;
    r.cosine = 1.0;
    const double mu = st->mu, sigma = st->sigma;
    const bool fitted = st->nnz != 0 && sigma >= 1e-12;
    r.k = fitted ? truncation_k(a.hists ? a.hists + (size_t)i * kHistBins : nullptr, mu, sigma, a.quantile) : 0.0;
    float alpha = p->alpha;
    double s_pred = p->s_pred;
    if (fitted && alpha > 0.0f) {
        const double c = r.k * sigma;
        double L = log((double)alpha) - mu;
        if (deep && cosine_of_pruning(sigma, L, c) < a.min_cosine[i]) {
            L = log_alpha_for_cosine(sigma, c, a.min_cosine[i]);
            const double av = exp(mu + L);
            alpha = av >= 3.4028234663852886e38 ? 3.4028234663852886e38f : (float)av;
            alpha = round_alpha(alpha, a.alpha_dtype);
            double B, C;
            s_pred = 0.0;
            if (alpha > 0.0f) {
                L = log((double)alpha) - mu;
                sparsity_terms<false>(mu, sigma, mu + L, s_pred, B, C);
            }
            p->alpha = alpha;
            p->s_pred = s_pred;
            p->s_eff = s_pred;
            r.status |= LGN_ALLOC_LOWERED;
        }
        if (alpha > 0.0f) r.cosine = cosine_of_pruning(sigma, L, c);
    }
    const double zero_frac = st->n ? 1.0 - (double)st->nnz / (double)st->n : 0.0;
    r.sparsity = zero_frac + (1.0 - zero_frac) * (alpha > 0.0f ? s_pred : 0.0);
    a.a_out[i] = r;
}

__global__ __launch_bounds__(kBlock) void allocate_kernel(AllocArgs a)
{
    __shared__ double rest_target;
    __shared__ uint32_t rest_status;
    // the deep layers, one lane each
    for (int i = threadIdx.x; i < a.n_deep; i += kBlock) allocate_layer(a, i, a.overall, 0u, true);
    __syncthreads();  // orders the global writes above for the workgroup (one workgroup only)
    if (threadIdx.x == 0) {
        double total = 0.0, deep_elems = 0.0, deep_zeros = 0.0;  // summed in layer order
        for (int i = 0; i < a.n_layers; ++i) total += (double)a.stats[i].n;
        for (int i = 0; i < a.n_deep; ++i) {
            const double n = (double)a.stats[i].n;
            deep_elems += n;
            deep_zeros += n * a.a_out[i].sparsity;
        }
        const double rest = total - deep_elems;
        double t = rest > 0.0 ? (a.overall * total - deep_zeros) / rest : a.overall;
        uint32_t s = 0u;
        if (t > a.max_sparsity) {
            t = a.max_sparsity;
            s = LGN_ALLOC_CAPPED;
        }
        rest_target = t < 0.0 ? 0.0 : t;
        rest_status = s;
    }
    __syncthreads();
    for (int i = a.n_deep + threadIdx.x; i < a.n_layers; i += kBlock)
        allocate_layer(a, i, rest_target, rest_status, false);
}

hipError_t launch_sparsity_allocate(const lgn_stats_t *stats, const uint64_t *hists, int n_layers,
                                    double overall, int n_deep, const double *min_cosine,
                                    double max_sparsity, double quantile, int alpha_dtype,
                                    lgn_prune_params_t *p_out, lgn_alloc_t *a_out, hipStream_t stream)
{
    const AllocArgs a = {stats, hists, n_layers, n_deep < n_layers ? n_deep : n_layers, overall,
                         max_sparsity, quantile, min_cosine, alpha_dtype, p_out, a_out};
    allocate_kernel<<<1, kBlock, 0, stream>>>(a);
    return hipGetLastError();
}

}  // namespace lgn

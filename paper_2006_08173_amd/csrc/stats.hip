// lgn_stats: lognormal parameters of a gradient tensor (Section 3: fit on |g| without the zero
// entries; Appendix "Stochastic pruning complexity": mean and standard deviation, O(n)).
//
// Two-stage grid reduction.  Stage 1 streams the tensor once with 16-byte loads; every thread
// keeps (count, sum, sum of squares) of the deviations of log2|g| from a pivot -- the first
// value that thread meets -- in fp64, so that no large common offset is squared.  Threads,
// waves and workgroups are then merged pairwise as (count, mean, M2) with the exact parallel
// update  M2 = M2a + M2b + d^2 na nb / n,  d = mean_b - mean_a.  Stage 2 merges the per-block
// records in a fixed order, so results are reproducible for a given launch shape.
//
// log2|g| = (biased exponent field) + log2(mantissa in [1,2)); the first term is an integer, the
// second one hardware v_log_f32 on a value in [1,2), i.e. an absolute error of about 1e-7 per
// element instead of the 2e-6 that a single-precision log of the full value would have.
// Subnormal inputs are normalised with integer operations.
#include "lgn_device.hpp"

namespace lgn {

struct Moments {
    double n, mean, m2;
};

struct Partial {  // one per stage-1 workgroup, 40 bytes
    double n, mean, m2;
    uint64_t nonfinite;
    uint32_t mx, mn;
};

__device__ __forceinline__ Moments merge(Moments a, Moments b)
{
    Moments r;
    r.n = a.n + b.n;
    if (r.n == 0.0) {
        r.mean = 0.0;
        r.m2 = 0.0;
        return r;
    }
    const double d = b.mean - a.mean;
    const double fb = b.n / r.n;
    r.mean = a.mean + d * fb;
    r.m2 = a.m2 + b.m2 + d * d * (a.n * fb);
    return r;
}

struct ThreadAcc {
    double pivot, s1, s2;
    uint32_t cnt, nonfinite, mx, mn;
};

__device__ __forceinline__ void accumulate(uint32_t bits, ThreadAcc &t)
{
    const uint32_t a = bits & 0x7fffffffu;
    if (a >= 0x7f800000u) {
        ++t.nonfinite;
        return;
    }
    if (a == 0u) return;
    uint32_t frac = a & 0x7fffffu;
    int ex = (int)(a >> 23);
    if (ex == 0) {  // subnormal: value = frac * 2^-149; bring the leading one to bit 23
        const int sh = __clz(frac) - 8;
        frac = (frac << sh) & 0x7fffffu;
        ex = 1 - sh;
    }
    const float lm = __log2f(__uint_as_float(0x3f800000u | frac));  // in [0, 1)
    const double l = (double)ex + (double)lm;                        // log2|g| + 127
    if (t.cnt == 0u) t.pivot = l;
    const double d = l - t.pivot;
    t.s1 += d;
    t.s2 = fma(d, d, t.s2);
    ++t.cnt;
    t.mx = max(t.mx, a);
    t.mn = min(t.mn, a);
}

// 16 bytes = 4 fp32 or 8 bf16 elements
template <int DTYPE>
__device__ __forceinline__ void accumulate_vec(uint4 v, ThreadAcc &t)
{
    if (DTYPE == LGN_F32) {
        accumulate(v.x, t); accumulate(v.y, t); accumulate(v.z, t); accumulate(v.w, t);
    } else {
        accumulate(v.x << 16, t); accumulate(v.x & 0xffff0000u, t);
        accumulate(v.y << 16, t); accumulate(v.y & 0xffff0000u, t);
        accumulate(v.z << 16, t); accumulate(v.z & 0xffff0000u, t);
        accumulate(v.w << 16, t); accumulate(v.w & 0xffff0000u, t);
    }
}

struct BlockAcc {
    Moments m;
    double nonfinite;
    uint32_t mx, mn;
};

__device__ __forceinline__ BlockAcc wave_reduce(BlockAcc v)
{
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        Moments o;
        o.n = __shfl_xor(v.m.n, off);
        o.mean = __shfl_xor(v.m.mean, off);
        o.m2 = __shfl_xor(v.m.m2, off);
        // both partners must combine in the same order to stay bit-identical
        const bool low = (threadIdx.x & off) == 0;
        v.m = low ? merge(v.m, o) : merge(o, v.m);
        v.nonfinite += __shfl_xor(v.nonfinite, off);
        v.mx = max(v.mx, (uint32_t)__shfl_xor((int)v.mx, off));
        v.mn = min(v.mn, (uint32_t)__shfl_xor((int)v.mn, off));
    }
    return v;
}

__device__ __forceinline__ BlockAcc block_reduce(BlockAcc v)
{
    __shared__ BlockAcc lds[kBlock / kWave];
    v = wave_reduce(v);
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    if (lane == 0) lds[wave] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kBlock / kWave; ++w) {
            v.m = merge(v.m, lds[w].m);
            v.nonfinite += lds[w].nonfinite;
            v.mx = max(v.mx, lds[w].mx);
            v.mn = min(v.mn, lds[w].mn);
        }
    }
    return v;  // valid in thread 0
}

template <int DTYPE>
__global__ __launch_bounds__(kBlock) void stats_stage1(const void *__restrict__ g, uint64_t n,
                                                       Partial *__restrict__ partials)
{
    constexpr int EPV = DTYPE == LGN_F32 ? 4 : 8;  // elements per 16-byte vector
    const uint64_t nvec = n / EPV;
    const uint64_t gsize = (uint64_t)gridDim.x * kBlock;
    const uint64_t gtid = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    const uint4 *__restrict__ gv = reinterpret_cast<const uint4 *>(g);

    ThreadAcc t;
    t.pivot = 0.0; t.s1 = 0.0; t.s2 = 0.0;
    t.cnt = 0u; t.nonfinite = 0u; t.mx = 0u; t.mn = 0xffffffffu;

    uint64_t v = gtid;
    for (; v + 3 * gsize < nvec; v += 4 * gsize) {  // four independent loads in flight
        const uint4 a = gv[v], b = gv[v + gsize], c = gv[v + 2 * gsize], d = gv[v + 3 * gsize];
        accumulate_vec<DTYPE>(a, t);
        accumulate_vec<DTYPE>(b, t);
        accumulate_vec<DTYPE>(c, t);
        accumulate_vec<DTYPE>(d, t);
    }
    for (; v < nvec; v += gsize) accumulate_vec<DTYPE>(gv[v], t);
    // ragged tail: fewer than EPV elements
    const uint64_t tail = nvec * EPV + gtid;
    if (gtid < (uint64_t)EPV && tail < n) accumulate(load_elem<DTYPE>(g, tail), t);

    BlockAcc b;
    b.m.n = (double)t.cnt;
    if (t.cnt) {
        const double inv = 1.0 / (double)t.cnt;
        b.m.mean = t.pivot + t.s1 * inv;
        b.m.m2 = fmax(t.s2 - t.s1 * t.s1 * inv, 0.0);
    } else {
        b.m.mean = 0.0;
        b.m.m2 = 0.0;
    }
    b.nonfinite = (double)t.nonfinite;
    b.mx = t.mx;
    b.mn = t.mn;
    b = block_reduce(b);
    if (threadIdx.x == 0) {
        Partial p;
        p.n = b.m.n; p.mean = b.m.mean; p.m2 = b.m.m2;
        p.nonfinite = (uint64_t)b.nonfinite;
        p.mx = b.mx; p.mn = b.mn;
        partials[blockIdx.x] = p;
    }
}

__global__ __launch_bounds__(kBlock) void stats_stage2(const Partial *__restrict__ partials,
                                                       int count, uint64_t n,
                                                       lgn_stats_t *__restrict__ out)
{
    BlockAcc b;
    b.m.n = 0.0; b.m.mean = 0.0; b.m.m2 = 0.0;
    b.nonfinite = 0.0; b.mx = 0u; b.mn = 0xffffffffu;
    for (int i = threadIdx.x; i < count; i += kBlock) {
        const Partial p = partials[i];
        Moments m;
        m.n = p.n; m.mean = p.mean; m.m2 = p.m2;
        b.m = merge(b.m, m);
        b.nonfinite += (double)p.nonfinite;
        b.mx = max(b.mx, p.mx);
        b.mn = min(b.mn, p.mn);
    }
    b = block_reduce(b);
    if (threadIdx.x != 0) return;
    lgn_stats_t s;
    s.n = n;
    s.nnz = (uint64_t)b.m.n;
    s.n_nonfinite = (uint64_t)b.nonfinite;
    s.status = 0u;
    s.reserved = 0u;
    if (s.n_nonfinite) s.status |= LGN_ST_HAS_NONFINITE;
    if (s.nnz == 0) {
        s.mean_log2 = __builtin_nan("");
        s.m2_log2 = 0.0;
        s.mu = __builtin_nan("");
        s.sigma = __builtin_nan("");
        s.max_abs = 0.0f;
        s.min_abs_nz = 0.0f;
        s.status |= LGN_ST_EMPTY;
    } else {
        const double ln2 = 0.693147180559945309417232121458;
        s.mean_log2 = b.m.mean - 127.0;  // remove the exponent bias
        s.m2_log2 = b.m.m2;
        s.mu = s.mean_log2 * ln2;
        s.sigma = sqrt(b.m.m2 / b.m.n) * ln2;
        s.max_abs = __uint_as_float(b.mx);
        s.min_abs_nz = __uint_as_float(b.mn);
        if (b.mx == b.mn) s.status |= LGN_ST_SIGMA0;
    }
    *out = s;
}

int stats_blocks(uint64_t n, int dtype)
{
    const uint64_t epv = dtype == LGN_F32 ? 4 : 8;
    uint64_t blocks = (n / epv + kBlock - 1) / kBlock;
    if (blocks < 1) blocks = 1;
    if (blocks > (uint64_t)kMaxStatsBlocks) blocks = kMaxStatsBlocks;
    return (int)blocks;
}

size_t stats_workspace_bytes() { return sizeof(Partial) * (size_t)kMaxStatsBlocks; }

hipError_t launch_stats(const void *g, uint64_t n, int dtype, lgn_stats_t *out, void *ws,
                        hipStream_t stream)
{
    const int blocks = stats_blocks(n, dtype);
    Partial *partials = static_cast<Partial *>(ws);
    if (dtype == LGN_F32)
        stats_stage1<LGN_F32><<<blocks, kBlock, 0, stream>>>(g, n, partials);
    else
        stats_stage1<LGN_BF16><<<blocks, kBlock, 0, stream>>>(g, n, partials);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    stats_stage2<<<1, kBlock, 0, stream>>>(partials, blocks, n, out);
    return hipGetLastError();
}

}  // namespace lgn

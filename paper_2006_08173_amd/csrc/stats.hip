// lgn_stats: lognormal parameters of a gradient tensor (Section 3: fit on |g| without the zero
// entries; Appendix "Stochastic pruning complexity": mean and standard deviation, O(n)).
//
// Two-stage grid reduction.  Stage 1 streams the tensor once with 16-byte loads, a batch of four
// consecutive 1 KiB rows per wave, the next batch requested before the current one is reduced.
// Per element: d = v_log_f32(2^-k |g|) (one hardware instruction, at most 1 ulp of its result),
// where 2^k is a wave-uniform reference point (k = the rounded mean log2 of the wave's first
// row): the deviation from the reference point directly, widened to fp64 and accumulated as sum
// and sum of squares in fp64.  Deviations are small, so the squares are, and nothing cancels
// when the moments are formed.  Waves and workgroups are merged pairwise as
// (count, mean, M2) with the exact parallel update  M2 = M2a + M2b + d^2 na nb / n,
// d = mean_b - mean_a.  Stage 2 merges the per-block records in a fixed order, so results are
// reproducible for a given launch shape.
//
// The hot loop assumes finite, normal or zero inputs; a quad-row of the wave that contains an
// Inf, NaN or subnormal is re-done by a careful path (wave-uniform branch) that normalises
// subnormals with integer operations.  Zeros contribute a zero deviation and are counted out
// with a ballot / popcount on the scalar unit.
#include <mutex>
#include <type_traits>

#include "launch.hpp"
#include "lgn_device.hpp"
#include "solver_device.hpp"

namespace lgn {

struct Moments {
    double n, mean, m2;
};

struct Partial {  // one per stage-1 workgroup, 40 bytes
    double n, mean, m2;
    uint64_t nonfinite;
    uint32_t mx, nmn;
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

// Per-lane accumulators; the pivot and the fast-path count are wave-uniform.
struct LaneAcc {
    double s1, s2;       // sum and sum of squares of (log2|g| - pivot)
    uint32_t mx;         // largest finite magnitude pattern
    uint32_t nmn;        // max over (0 - a) of non-zero magnitudes, i.e. minus the smallest one
    uint32_t slow_cnt;   // valid elements counted by the careful path (per lane)
    uint32_t nonfinite;  // per lane
};

// log2 of a finite, normal, non-zero magnitude pattern as exponent + log2(mantissa) in fp64
// (careful path only).
__device__ __forceinline__ double careful_log2(uint32_t a)
{
    const float m = __uint_as_float((a & 0x007fffffu) | 0x3f800000u);
    return (double)((int)(a >> 23) - 127) + (double)__log2f(m);
}

// Careful per-element path: Inf/NaN counted and skipped, subnormals normalised.
__device__ __forceinline__ void accumulate_careful(uint32_t bits, float pivot, LaneAcc &t)
{
    const uint32_t a = bits & 0x7fffffffu;
    if (a >= 0x7f800000u) {
        ++t.nonfinite;
        return;
    }
    if (a == 0u) return;
    double l;
    if (a < 0x00800000u) {  // subnormal: value = a * 2^-149; bring the leading one to bit 23
        const int sh = __clz(a) - 8;
        l = careful_log2(((a << sh) & 0x007fffffu) | 0x00800000u) - (double)sh;
    } else {
        l = careful_log2(a);
    }
    const double d = l - (double)pivot;
    t.s1 += d;
    t.s2 = fma(d, d, t.s2);
    ++t.slow_cnt;
    t.mx = max(t.mx, a);
    t.nmn = max(t.nmn, 0u - a);
}

// The wave's reference point: a power of two near the bulk of its values (wave-uniform).
struct Pivot {
    uint32_t bits;        // 2^k as an fp32 pattern
    float scale;          // 2^-k
    float log2;           // k
    uint32_t hi_lim;      // magnitudes at or above this pattern leave the fast path (Inf, NaN, or 2^-k |g| overflows)
    uint32_t neg_lo_lim;  // minus the smallest pattern the fast path takes (below: subnormal, or 2^-k |g| is)
};

// Four elements per lane.  Returns the number of valid elements the fast path counted for the
// whole wave (wave-uniform), 0 if the careful path was taken.
// The logarithm is taken of 2^-k |g| (an exact product): its result is the deviation itself, a
// small number, so the instruction's error (it truncates: -0.5 ulp of the RESULT on average, up
// to 1 ulp) is small too and is spread evenly around the reference point.  Taken of |g| itself
// the result sits near -20 for typical gradients, the error is 1e-6 absolute, and its mean
// jumps where |log2| crosses a power of two -- at 2^-16, in the middle of typical gradients --
// which a narrow distribution (sigma below 0.2) sees as an error of 1e-6 and more in sigma.
// SUM4_F32: the four deviations and their squares are first summed in fp32 and enter the fp64
// accumulators as two numbers instead of eight.  Used for the 16-bit element types, where the
// pass is bound by arithmetic (twice the elements per byte): the three extra fp32 roundings per
// sum are unbiased and of the size of the logarithm's own error (~1e-7 relative on a partial
// sum of four), far inside the 1e-6 budget on mu and sigma.
template <bool SUM4_F32 = false>
__device__ __forceinline__ uint32_t accumulate_quad(uint32_t b0, uint32_t b1, uint32_t b2,
                                                    uint32_t b3, const Pivot &pv, LaneAcc &t)
{
    const uint32_t a0 = b0 & 0x7fffffffu, a1 = b1 & 0x7fffffffu;
    const uint32_t a2 = b2 & 0x7fffffffu, a3 = b3 & 0x7fffffffu;
    const bool v0 = a0 != 0u, v1 = a1 != 0u, v2 = a2 != 0u, v3 = a3 != 0u;
    // Zeros are replaced by the reference magnitude BEFORE the logarithm, so they come out as an
    // exact zero deviation (one integer select instead of masking a double afterwards).
    const float f0 = __builtin_amdgcn_logf(__uint_as_float(v0 ? a0 : pv.bits) * pv.scale);
    const float f1 = __builtin_amdgcn_logf(__uint_as_float(v1 ? a1 : pv.bits) * pv.scale);
    const float f2 = __builtin_amdgcn_logf(__uint_as_float(v2 ? a2 : pv.bits) * pv.scale);
    const float f3 = __builtin_amdgcn_logf(__uint_as_float(v3 ? a3 : pv.bits) * pv.scale);
    const uint32_t qmx = max(max(a0, a1), max(a2, a3));
    // -a is large for small a and 0 for a = 0 (unsigned): its maximum tracks the smallest non-zero
    const uint32_t qnmn = max(max(0u - a0, 0u - a1), max(0u - a2, 0u - a3));
    // Inf / NaN have a >= 0x7f800000; a subnormal has 0 < a < 0x00800000; the limits are tighter
    // by |k| binades on one side, where the scaled value would leave the normal range
    const bool odd = qmx >= pv.hi_lim || qnmn > pv.neg_lo_lim;
    if (__builtin_amdgcn_ballot_w64(odd) != 0ull) {
        accumulate_careful(b0, pv.log2, t);
        accumulate_careful(b1, pv.log2, t);
        accumulate_careful(b2, pv.log2, t);
        accumulate_careful(b3, pv.log2, t);
        return 0u;
    }
    const uint32_t cnt = (uint32_t)__popcll(__builtin_amdgcn_ballot_w64(v0)) +
                         (uint32_t)__popcll(__builtin_amdgcn_ballot_w64(v1)) +
                         (uint32_t)__popcll(__builtin_amdgcn_ballot_w64(v2)) +
                         (uint32_t)__popcll(__builtin_amdgcn_ballot_w64(v3));
    t.mx = max(t.mx, qmx);
    t.nmn = max(t.nmn, qnmn);
    if (SUM4_F32) {
        t.s1 += (double)((f0 + f1) + (f2 + f3));
        t.s2 += (double)__builtin_fmaf(f0, f0, __builtin_fmaf(f1, f1, __builtin_fmaf(f2, f2, f3 * f3)));
        return cnt;
    }
    const double d0 = (double)f0, d1 = (double)f1, d2 = (double)f2, d3 = (double)f3;
    t.s1 += d0; t.s2 = fma(d0, d0, t.s2);
    t.s1 += d1; t.s2 = fma(d1, d1, t.s2);
    t.s1 += d2; t.s2 = fma(d2, d2, t.s2);
    t.s1 += d3; t.s2 = fma(d3, d3, t.s2);
    return cnt;
}

// 16 bytes = 4 fp32 or 8 bf16 elements
template <int DTYPE>
__device__ __forceinline__ uint32_t accumulate_vec(uint4 v, const Pivot &pv, LaneAcc &t)
{
    if (DTYPE == LGN_F32) return accumulate_quad(v.x, v.y, v.z, v.w, pv, t);
    uint32_t e[8];
    widen_pair<DTYPE>(v.x, e[0], e[1]);
    widen_pair<DTYPE>(v.y, e[2], e[3]);
    widen_pair<DTYPE>(v.z, e[4], e[5]);
    widen_pair<DTYPE>(v.w, e[6], e[7]);
    return accumulate_quad<true>(e[0], e[1], e[2], e[3], pv, t) +
           accumulate_quad<true>(e[4], e[5], e[6], e[7], pv, t);
}

template <typename T>
__device__ __forceinline__ T wave_max(T v)
{
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) v = max(v, (T)__shfl_xor(v, off));
    return v;
}

struct BlockAcc {
    Moments m;
    double nonfinite;
    uint32_t mx;
    uint32_t nmn;  // max over (0 - a) of the non-zero magnitudes: 0 when there is none
};

__device__ __forceinline__ BlockAcc block_merge(BlockAcc v)  // one record per wave, in lane 0
{
    __shared__ BlockAcc lds[kBlock / kWave];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    if (lane == 0) lds[wave] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kBlock / kWave; ++w) {
            v.m = merge(v.m, lds[w].m);
            v.nonfinite += lds[w].nonfinite;
            v.mx = max(v.mx, lds[w].mx);
            v.nmn = max(v.nmn, lds[w].nmn);
        }
    }
    return v;  // valid in thread 0
}

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) v += __shfl_xor(v, off);
    return v;  // the xor butterfly adds the same pairs in every lane: all lanes agree
}

// Stores of a per-block record.  The plain form is for a consumer in a LATER launch.  The
// write-through form is for a consumer in the SAME launch on another XCD: each word goes out as a
// device-scope atomic store (written through this XCD's L2), so waiting for the stores to complete
// makes the record visible device-wide without writing back the whole L2, which a device-scope
// release fence would do (measured: +40 us on a 140 us pass when every workgroup issues one).
__device__ __forceinline__ void store_partial(Partial *dst, const Partial &p, bool write_through)
{
    if (!write_through) {
        *dst = p;
        return;
    }
    static_assert(sizeof(Partial) == 40, "five 8-byte words");
    unsigned long long w[5];
    __builtin_memcpy(w, &p, sizeof p);
    unsigned long long *d = reinterpret_cast<unsigned long long *>(dst);
#pragma unroll
    for (int i = 0; i < 5; ++i) __hip_atomic_store(d + i, w[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ---- optional mask: statistics of the right mode of a bi-modal gradient ---------------------
// (appendix "Algorithm for bi-Modal lognormal pruning", step 3: only the values whose
// corresponding entries in the other gradient tensor are non-zero).  MASK = 0: none; 1: a tensor
// of the same type as g (entry counts iff its pattern is not +-0); 2: one byte per element.
// A masked-out element is turned into a zero pattern, which the accumulation leaves out anyway.
template <int DTYPE, int MASK>
struct MaskVec {  // the mask entries that go with one 16-byte vector of g
};
template <int DTYPE>
struct MaskVec<DTYPE, 1> {
    uint4 v;
};
template <>
struct MaskVec<LGN_F32, 2> {
    uint32_t v;  // four bytes
};
template <>
struct MaskVec<LGN_BF16, 2> {
    uint2 v;  // eight bytes
};
template <>
struct MaskVec<LGN_F16, 2> {
    uint2 v;  // eight bytes
};

template <int DTYPE, int MASK>
__device__ __forceinline__ MaskVec<DTYPE, MASK> load_mask_vec(const void *mask, uint64_t vec)
{
    MaskVec<DTYPE, MASK> m;
    if constexpr (MASK == 1) {
        m.v = load_stream16(reinterpret_cast<const uint4 *>(mask) + vec);
    } else if constexpr (MASK == 2 && DTYPE == LGN_F32) {
        m.v = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(mask) + vec);
    } else if constexpr (MASK == 2) {
        const u32x2_t x = __builtin_nontemporal_load(reinterpret_cast<const u32x2_t *>(mask) + vec);
        m.v = make_uint2(x.x, x.y);
    }
    return m;
}

// keeps the 16-bit halves of w whose mask halves (sign bit aside) / mask bytes are non-zero
__device__ __forceinline__ uint32_t keep_halves(uint32_t w, bool lo, bool hi)
{
    return w & ((lo ? 0x0000ffffu : 0u) | (hi ? 0xffff0000u : 0u));
}

template <int DTYPE, int MASK>
__device__ __forceinline__ uint4 apply_mask(uint4 g, const MaskVec<DTYPE, MASK> &m)
{
    if constexpr (MASK == 1 && DTYPE == LGN_F32) {
        g.x = (m.v.x & 0x7fffffffu) ? g.x : 0u;
        g.y = (m.v.y & 0x7fffffffu) ? g.y : 0u;
        g.z = (m.v.z & 0x7fffffffu) ? g.z : 0u;
        g.w = (m.v.w & 0x7fffffffu) ? g.w : 0u;
    } else if constexpr (MASK == 1) {
        g.x = keep_halves(g.x, m.v.x & 0x7fffu, m.v.x & 0x7fff0000u);
        g.y = keep_halves(g.y, m.v.y & 0x7fffu, m.v.y & 0x7fff0000u);
        g.z = keep_halves(g.z, m.v.z & 0x7fffu, m.v.z & 0x7fff0000u);
        g.w = keep_halves(g.w, m.v.w & 0x7fffu, m.v.w & 0x7fff0000u);
    } else if constexpr (MASK == 2 && DTYPE == LGN_F32) {
        g.x = (m.v & 0x000000ffu) ? g.x : 0u;
        g.y = (m.v & 0x0000ff00u) ? g.y : 0u;
        g.z = (m.v & 0x00ff0000u) ? g.z : 0u;
        g.w = (m.v & 0xff000000u) ? g.w : 0u;
    } else if constexpr (MASK == 2) {
        g.x = keep_halves(g.x, m.v.x & 0x000000ffu, m.v.x & 0x0000ff00u);
        g.y = keep_halves(g.y, m.v.x & 0x00ff0000u, m.v.x & 0xff000000u);
        g.z = keep_halves(g.z, m.v.y & 0x000000ffu, m.v.y & 0x0000ff00u);
        g.w = keep_halves(g.w, m.v.y & 0x00ff0000u, m.v.y & 0xff000000u);
    }
    return g;
}

// mask entry of one element (tail of the tensor)
template <int DTYPE, int MASK>
__device__ __forceinline__ bool mask_elem(const void *mask, uint64_t i)
{
    if constexpr (MASK == 1) return (load_elem<DTYPE>(mask, i) & 0x7fffffffu) != 0u;
    else if constexpr (MASK == 2) return reinterpret_cast<const uint8_t *>(mask)[i] != 0;
    else return true;
}

// One 16-byte vector of g with its mask entries, as loaded (the mask is applied when the row is
// reduced, so that both loads can stay in flight).
template <int DTYPE, int MASK>
struct Row {
    uint4 g;
    MaskVec<DTYPE, MASK> m;
};

// KEEP: the vector of g is loaded without the streaming hint, so that it stays in the memory-side
// cache for the pass that reads the tensor next.
template <int DTYPE, int MASK, bool KEEP = false>
__device__ __forceinline__ Row<DTYPE, MASK> load_row(const uint4 *gv, const void *mask, uint64_t vec)
{
    Row<DTYPE, MASK> r;
    if (KEEP) r.g = gv[vec];
    else r.g = load_stream16(gv + vec);
    r.m = load_mask_vec<DTYPE, MASK>(mask, vec);
    return r;
}

// `block` of `nblocks`: the workgroup's place among the workgroups that share the tensor (the whole
// grid for a one-tensor launch, a slice of it for a batched one); partials[block] is written.
template <int DTYPE, bool WRITE_THROUGH, int MASK>
__device__ __forceinline__ void stage1_body(const void *__restrict__ g, const void *__restrict__ mask,
                                            uint64_t n, uint64_t keep_vecs, Partial *partials,
                                            uint32_t block, uint32_t nblocks)
{
    constexpr int EPV = DTYPE == LGN_F32 ? 4 : 8;  // elements per 16-byte vector
    constexpr int kWavesPerBlock = kBlock / kWave;
    using R = Row<DTYPE, MASK>;
    const uint64_t nvec = n / EPV;
    const uint64_t nrows = nvec / kWave;  // full rows of 64 vectors (1 KiB)
    const uint64_t nwaves = (uint64_t)nblocks * kWavesPerBlock;
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint64_t wave = (uint64_t)block * kWavesPerBlock +
                          (uint64_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
    const uint4 *__restrict__ gv = reinterpret_cast<const uint4 *>(g);

    LaneAcc t;
    t.s1 = 0.0; t.s2 = 0.0;
    t.mx = 0u; t.nmn = 0u; t.slow_cnt = 0u; t.nonfinite = 0u;
    uint32_t cnt = 0;  // wave-uniform; one wave sees far fewer than 2^32 elements

    // Reference point: 2^k, k = the mean log2 of the normal magnitudes in the wave's first row,
    // rounded (0 if there is none).  The mean, not an extreme: one huge or tiny value in that row
    // must not move it away from the bulk, or the squares of the deviations grow and their low
    // bits (summed in fp32 for the 16-bit types) start to matter.
    int k = 0;
    if (wave < nrows) {
        const R r = load_row<DTYPE, MASK>(gv, mask, wave * kWave + lane);
        const uint4 v = apply_mask<DTYPE, MASK>(r.g, r.m);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
        float sum = 0.0f;
        uint32_t count = 0u;
        auto take = [&](uint32_t a) {
            const bool normal = a >= 0x00800000u && a < 0x7f800000u;
            sum += normal ? __builtin_amdgcn_logf(__uint_as_float(a)) : 0.0f;
            count += normal ? 1u : 0u;
        };
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint32_t lo = w[i], hi = 0u;
            if (DTYPE != LGN_F32) widen_pair<DTYPE>(w[i], lo, hi);
            take(lo & 0x7fffffffu);
            if (DTYPE != LGN_F32) take(hi & 0x7fffffffu);
        }
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
            sum += __shfl_xor(sum, off);
            count += __shfl_xor(count, off);
        }
        if (count != 0u) k = (int)rintf(fminf(fmaxf(sum / (float)count, -126.0f), 126.0f));  // 2^k and 2^-k are normal
        k = __builtin_amdgcn_readfirstlane(k);
    }
    Pivot pv;
    pv.bits = (uint32_t)(127 + k) << 23;
    pv.scale = __uint_as_float((uint32_t)(127 - k) << 23);
    pv.log2 = (float)k;
    pv.hi_lim = k < 0 ? (uint32_t)(255 + k) << 23 : 0x7f800000u;
    pv.neg_lo_lim = 0u - (k > 0 ? (uint32_t)(1 + k) << 23 : 0x00800000u);
    const float pivot = pv.log2;
    auto reduce = [&](const R &r) {
        cnt += accumulate_vec<DTYPE>(apply_mask<DTYPE, MASK>(r.g, r.m), pv, t);
    };

    // Full rows, wave-uniform control flow.  A batch is four CONSECUTIVE rows (4 KiB contiguous
    // per wave): strides of a power-of-two number of rows between the loads of one wave alias in
    // the memory channels and cost ~20 % of the read bandwidth.  The next batch is requested
    // before the current one is reduced, so the arithmetic overlaps the memory latency.
    //
    // The last `keep_vecs` vectors of the tensor are loaded as ordinary (cache-allocating) reads and
    // everything before them as streaming reads: what was read last is then still in the
    // memory-side cache when the next pass over the same tensor arrives, and the streaming part
    // does not push it out.  A wave meets its batches in increasing order, so it runs the loop
    // once per flavour.
    const uint64_t nbatches = nrows / 4;
    const uint64_t first_kept = keep_vecs >= nvec ? 0 : (nvec - keep_vecs + 4 * kWave - 1) / (4 * kWave);
    auto walk = [&](auto keep_tag, uint64_t cur, const uint64_t limit) -> uint64_t {
        constexpr bool KEEP = decltype(keep_tag)::value;
        if (!(cur < limit)) return cur;
        // Two register sets used alternately.  Inside the loop every load is unconditional, so
        // the compiler waits for exactly the older loads while the younger ones stay in
        // flight; the last batch of the wave is reduced after the loop.
        R a0, a1, a2, a3, b0, b1, b2, b3;
        {
            const uint64_t v = cur * (4 * kWave) + lane;  // batch held in the a-set
            a0 = load_row<DTYPE, MASK, KEEP>(gv, mask, v); a1 = load_row<DTYPE, MASK, KEEP>(gv, mask, v + kWave);
            a2 = load_row<DTYPE, MASK, KEEP>(gv, mask, v + 2 * kWave); a3 = load_row<DTYPE, MASK, KEEP>(gv, mask, v + 3 * kWave);
        }
        bool in_a = true;  // which set holds the batch that is still to be reduced
        while (cur + nwaves < limit) {
            {
                const uint64_t v = (cur + nwaves) * (4 * kWave) + lane;
                b0 = load_row<DTYPE, MASK, KEEP>(gv, mask, v); b1 = load_row<DTYPE, MASK, KEEP>(gv, mask, v + kWave);
                b2 = load_row<DTYPE, MASK, KEEP>(gv, mask, v + 2 * kWave); b3 = load_row<DTYPE, MASK, KEEP>(gv, mask, v + 3 * kWave);
            }
            reduce(a0); reduce(a1); reduce(a2); reduce(a3);
            cur += nwaves;
            if (!(cur + nwaves < limit)) {
                in_a = false;
                break;
            }
            {
                const uint64_t v = (cur + nwaves) * (4 * kWave) + lane;
                a0 = load_row<DTYPE, MASK, KEEP>(gv, mask, v); a1 = load_row<DTYPE, MASK, KEEP>(gv, mask, v + kWave);
                a2 = load_row<DTYPE, MASK, KEEP>(gv, mask, v + 2 * kWave); a3 = load_row<DTYPE, MASK, KEEP>(gv, mask, v + 3 * kWave);
            }
            reduce(b0); reduce(b1); reduce(b2); reduce(b3);
            cur += nwaves;
        }
        if (in_a) {
            reduce(a0); reduce(a1); reduce(a2); reduce(a3);
        } else {
            reduce(b0); reduce(b1); reduce(b2); reduce(b3);
        }
        return cur + nwaves;
    };
    {
        uint64_t cur = walk(std::false_type{}, wave, first_kept < nbatches ? first_kept : nbatches);
        walk(std::true_type{}, cur, nbatches);
    }
    // up to three full rows after the last batch
    for (uint64_t row = nbatches * 4 + wave; row < nrows; row += nwaves)
        reduce(load_row<DTYPE, MASK>(gv, mask, row * kWave + lane));

    // what is left: fewer than 64 vectors, then fewer than EPV elements; one wave, careful path
    if (wave == nwaves - 1) {
        const uint64_t v = nrows * kWave + lane;
        if (v < nvec) {
            const R r = load_row<DTYPE, MASK>(gv, mask, v);
            const uint4 x = apply_mask<DTYPE, MASK>(r.g, r.m);
            const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (DTYPE == LGN_F32) {
                    accumulate_careful(w[i], pivot, t);
                } else {
                    uint32_t lo, hi;
                    widen_pair<DTYPE>(w[i], lo, hi);
                    accumulate_careful(lo, pivot, t);
                    accumulate_careful(hi, pivot, t);
                }
            }
        }
        const uint64_t tail = nvec * EPV + lane;
        if (lane < (uint32_t)EPV && tail < n && mask_elem<DTYPE, MASK>(mask, tail))
            accumulate_careful(load_elem<DTYPE>(g, tail), pivot, t);
    }

    // wave totals relative to the wave's pivot, then (count, mean, M2)
    const double s1 = wave_sum(t.s1), s2 = wave_sum(t.s2);
    const double nn = (double)cnt + wave_sum((double)t.slow_cnt);
    BlockAcc b;
    b.m.n = nn;
    if (nn > 0.0) {
        b.m.mean = (double)pivot + s1 / nn;
        b.m.m2 = fmax(s2 - s1 * (s1 / nn), 0.0);
    } else {
        b.m.mean = 0.0;
        b.m.m2 = 0.0;
    }
    b.nonfinite = wave_sum((double)t.nonfinite);
    b.mx = wave_max(t.mx);
    b.nmn = wave_max(t.nmn);
    b = block_merge(b);
    if (threadIdx.x == 0) {
        Partial p;
        p.n = b.m.n; p.mean = b.m.mean; p.m2 = b.m.m2;
        p.nonfinite = (uint64_t)b.nonfinite;
        p.mx = b.mx; p.nmn = b.nmn;
        store_partial(partials + block, p, WRITE_THROUGH);
    }
}

template <int DTYPE, int MASK>
__global__ __launch_bounds__(kBlock) void stats_stage1(const void *__restrict__ g,
                                                       const void *__restrict__ mask, uint64_t n,
                                                       uint64_t keep_vecs,
                                                       Partial *__restrict__ partials)
{
    stage1_body<DTYPE, false, MASK>(g, mask, n, keep_vecs, partials, blockIdx.x, gridDim.x);
}

// Merges `count` per-block records; thread 0 writes the result to *out and, if given, to *lds_out.
__device__ __forceinline__ void stage2_body(const Partial *partials, int count, uint64_t n,
                                            lgn_stats_t *out, lgn_stats_t *lds_out)
{
    // lane-serial merge of the records in index order, then a fixed butterfly: reproducible
    BlockAcc b;
    b.m.n = 0.0; b.m.mean = 0.0; b.m.m2 = 0.0;
    b.nonfinite = 0.0; b.mx = 0u; b.nmn = 0u;
    for (int i = threadIdx.x; i < count; i += kBlock) {
        const Partial p = partials[i];
        Moments m;
        m.n = p.n; m.mean = p.mean; m.m2 = p.m2;
        b.m = merge(b.m, m);
        b.nonfinite += (double)p.nonfinite;
        b.mx = max(b.mx, p.mx);
        b.nmn = max(b.nmn, p.nmn);
    }
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        Moments o;
        o.n = __shfl_xor(b.m.n, off);
        o.mean = __shfl_xor(b.m.mean, off);
        o.m2 = __shfl_xor(b.m.m2, off);
        const bool low = (threadIdx.x & off) == 0;  // both partners combine in the same order
        b.m = low ? merge(b.m, o) : merge(o, b.m);
        b.nonfinite += __shfl_xor(b.nonfinite, off);
        b.mx = max(b.mx, (uint32_t)__shfl_xor((int)b.mx, off));
        b.nmn = max(b.nmn, (uint32_t)__shfl_xor((int)b.nmn, off));
    }
    b = block_merge(b);
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
        const uint32_t mn = 0u - b.nmn;
        s.mean_log2 = b.m.mean;
        s.m2_log2 = b.mx == mn ? 0.0 : b.m.m2;
        s.mu = s.mean_log2 * ln2;
        s.sigma = sqrt(s.m2_log2 / b.m.n) * ln2;
        s.max_abs = __uint_as_float(b.mx);
        s.min_abs_nz = __uint_as_float(mn);
        if (b.mx == mn) s.status |= LGN_ST_SIGMA0;
    }
    *out = s;
    if (lds_out) *lds_out = s;
}

__global__ __launch_bounds__(kBlock) void stats_stage2(const Partial *__restrict__ partials,
                                                       int count, uint64_t n,
                                                       lgn_stats_t *__restrict__ out)
{
    stage2_body(partials, count, n, out, nullptr);
}

// ---- one launch for statistics + both parameter solves -------------------------------------
// Every workgroup publishes its record, then takes a ticket; the workgroup that draws the last
// ticket merges all records (stage 2) and runs the two solvers in two of its waves.  The ticket
// lives at the end of the workspace, must be zero on entry and is reset to zero on exit.
struct SolveRequest {
    double target_sparsity;  // < 0: no threshold asked for
    int alpha_dtype;         // bit 8: publish the per-block record with a release fence
    int n_bits;              // 0: no format asked for
    int e_bits, scale_mode, sigma_units;
    double scale_z;  // standard normal quantile of the scale rule (evaluated by the host)
};

// What follows a workgroup's stage 1 in the one-launch form: publish, take a ticket, and if it was
// the last one of the tensor's `nblocks` workgroups, combine their records and solve.
__device__ __forceinline__ void finish_and_solve(const Partial *partials, uint32_t nblocks, uint64_t n,
                                                 unsigned int *ticket, const SolveRequest &rq,
                                                 lgn_stats_t *st_out, lgn_prune_params_t *p_out,
                                                 lgn_fp_params_t *f_out)
{
    __shared__ bool is_last;
    __shared__ lgn_stats_t st_lds;
    if (threadIdx.x == 0) {
        // Thread 0 wrote the record with write-through stores; once they have completed
        // (s_waitcnt 0 = every counter at zero) the record is in memory, and only then is the
        // ticket taken.  The signal fences keep the compiler from moving memory operations
        // across the wait.
        __atomic_signal_fence(__ATOMIC_SEQ_CST);
        __builtin_amdgcn_s_waitcnt(0);
        __atomic_signal_fence(__ATOMIC_SEQ_CST);
        // That completed write-through stores are visible device-wide is how this hardware
        // behaves, not a promise of the memory model.  With the knob LGN_TUNE_STATS_STRICT_PUBLISH
        // the release fence the model asks for is added; it writes back this XCD's whole L2,
        // the dirty lines of the pass before included (+11 us on an 822 MB tensor behind a fused
        // pass, +55 us on 10^9 bf16 elements), so it is off by default and there to rule out a
        // suspected stale read.
        if (rq.alpha_dtype & 0x100) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        is_last = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) ==
                  nblocks - 1;
    }
    __syncthreads();
    if (!is_last) return;
    // one workgroup only: drop what this XCD's caches hold, then read every record
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    stage2_body(partials, (int)nblocks, n, st_out, &st_lds);
    __syncthreads();
    const int wave = threadIdx.x / kWave;
    if (wave == 0 && p_out && rq.target_sparsity >= 0.0) {
        threshold_body<true>(&st_lds, rq.target_sparsity, rq.alpha_dtype & 0xff, p_out);
    } else if (wave == 1 && f_out && rq.n_bits != 0) {
        fp_params_body(&st_lds, rq.n_bits, rq.e_bits, rq.scale_mode, rq.scale_z, rq.sigma_units, f_out);
    }
    __syncthreads();  // both parameter structs are written
    if (threadIdx.x == 0) {
        // Pruning followed by this format (Section 5's operator, then Section 4.1's underflow
        // rule): every survivor at or below alpha comes out as +-alpha, and a magnitude below
        // 2^(E_min + s), E_min = 1 - 2^(e-1), is flushed.  A threshold below that loses everything
        // pruning touched; only this kernel holds both results, so it reports the condition.
        if (p_out && f_out && rq.target_sparsity >= 0.0 && rq.n_bits != 0) {
            const float alpha = p_out->alpha;
            const int k = 1 - (1 << (f_out->e_bits - 1)) + f_out->scale_exp;
            if (alpha > 0.0f && (double)alpha < ldexp(1.0, k)) p_out->status |= LGN_ST_ALPHA_BELOW_FP_RANGE;
        }
        *ticket = 0u;  // ready for the next call on this workspace
    }
}

template <int DTYPE, int MASK>
__global__ __launch_bounds__(kBlock) void stats_solve_kernel(const void *__restrict__ g,
                                                             const void *__restrict__ mask, uint64_t n,
                                                             uint64_t keep_vecs,
                                                             Partial *partials, unsigned int *ticket,
                                                             SolveRequest rq, lgn_stats_t *st_out,
                                                             lgn_prune_params_t *p_out,
                                                             lgn_fp_params_t *f_out)
{
    stage1_body<DTYPE, true, MASK>(g, mask, n, keep_vecs, partials, blockIdx.x, gridDim.x);
    finish_and_solve(partials, gridDim.x, n, ticket, rq, st_out, p_out, f_out);
}

// ---- many tensors, one launch ----------------------------------------------------------------
// The grid is cut into one slice of workgroups per tensor (slice sizes proportional to the element
// counts, so that all slices finish together); a workgroup finds its tensor in a table of first
// workgroup indices, runs stage 1 on its share of that tensor, and the last workgroup of each
// slice combines and solves for its tensor, with a ticket of its own.  The tables travel in the
// kernel argument, so nothing has to be uploaded or allocated.
struct BatchStatsTensor {
    const void *g;
    uint64_t n;
    uint64_t keep_vecs;
    double target_sparsity;
    lgn_stats_t *st;
    lgn_prune_params_t *p;
    lgn_fp_params_t *f;
    uint32_t blocks;
    int16_t n_bits, e_bits;
};

struct BatchStatsArgs {
    Partial *partials;
    unsigned int *tickets;
    double scale_z;
    int32_t alpha_dtype, scale_mode, sigma_units, count;
    uint32_t first_block[kBatchMax];  // of tensor i; 0xffffffff past the last tensor
    BatchStatsTensor t[kBatchMax];
};
static_assert(sizeof(BatchStatsArgs) <= 4096, "must fit the kernel argument segment");

template <int DTYPE>
__global__ __launch_bounds__(kBlock) void stats_solve_batch_kernel(BatchStatsArgs a)
{
    const uint32_t b = blockIdx.x;
    int t = 0;
#pragma unroll
    for (int i = 1; i < kBatchMax; ++i) t += a.first_block[i] <= b ? 1 : 0;  // uniform: scalar unit
    t = __builtin_amdgcn_readfirstlane(t);
    const BatchStatsTensor &T = a.t[t];
    const uint32_t first = a.first_block[t];
    stage1_body<DTYPE, true, 0>(T.g, nullptr, T.n, T.keep_vecs, a.partials + first, b - first, T.blocks);
    const SolveRequest rq = {T.target_sparsity, a.alpha_dtype, T.n_bits, T.e_bits, a.scale_mode, a.sigma_units,
                             a.scale_z};
    finish_and_solve(a.partials + first, T.blocks, T.n, a.tickets + t, rq, T.st, T.p, T.f);
}

int stats_blocks(uint64_t n, int dtype)
{
    const uint64_t epv = dtype == LGN_F32 ? 4 : 8;
    uint64_t blocks = (n / epv + 4 * kBlock - 1) / (4 * kBlock);  // four rows per wave and pass
    if (blocks < 1) blocks = 1;
    if (blocks > (uint64_t)kMaxStatsBlocks) blocks = kMaxStatsBlocks;
    return (int)blocks;
}

constexpr size_t kTicketOffset = sizeof(Partial) * (size_t)kMaxStatsBlocks;  // 8-byte aligned
constexpr size_t kTicketBytes = 256;  // 64 tickets: one per tensor of a batched launch
static_assert(kBatchMax * sizeof(unsigned int) <= kTicketBytes, "a ticket per tensor");

size_t stats_workspace_bytes() { return kTicketOffset + kTicketBytes; }

__global__ void ticket_clear_kernel(unsigned int *ticket)
{
    if (threadIdx.x < kTicketBytes / sizeof(unsigned int)) ticket[threadIdx.x] = 0u;
}

hipError_t launch_workspace_init(void *ws, hipStream_t stream)
{
    ticket_clear_kernel<<<1, kWave, 0, stream>>>(
        reinterpret_cast<unsigned int *>(static_cast<char *>(ws) + kTicketOffset));
    return hipGetLastError();
}

// How much of the tensor's tail the statistics pass leaves in the memory-side cache (256 MB on
// this chip), in 16-byte vectors (knob LGN_TUNE_STATS_KEEP_MB; 0 switches it off).  The result of
// the pass does not depend on it: every wave still reduces its batches in the same order.
static uint64_t kept_vectors() { return (uint64_t)tuning(LGN_TUNE_STATS_KEEP_MB) * ((1u << 20) / 16); }

// Workgroups of the statistics pass.  Read-only streaming likes few, long-lived waves: for fp32
// two workgroups per CU (each wave keeps 8 KiB in flight) measured best, 6.3 TB/s against 5.9 at
// four; the 16-bit types have twice the arithmetic per byte and want six (10^9 bf16 elements:
// 0.398 / 0.365 / 0.348 / 0.341 / 0.335 ms at 2 / 3 / 4 / 6 / 8).  Fewer workgroups also mean fewer
// per-block records for the combine step.
static int stats_blocks_cap(int dtype)
{
    const long knob = tuning(LGN_TUNE_STATS_BLOCKS_PER_CU);
    const int per_cu = knob > 0 ? (int)knob : (dtype == LGN_F32 ? 2 : 6);
    const int blocks = device_cus() * per_cu;
    return blocks > kMaxStatsBlocks ? kMaxStatsBlocks : blocks;
}

// Calls f.template operator()<DTYPE, MASK>() for the run-time pair (dtype, mask_kind).
template <typename F>
static void dispatch_dtype_mask(int dtype, int mask_kind, F &&f)
{
    if (dtype == LGN_F32) {
        if (mask_kind == LGN_MASK_SAME_DTYPE) f.template operator()<LGN_F32, 1>();
        else if (mask_kind == LGN_MASK_U8) f.template operator()<LGN_F32, 2>();
        else f.template operator()<LGN_F32, 0>();
    } else if (dtype == LGN_BF16) {
        if (mask_kind == LGN_MASK_SAME_DTYPE) f.template operator()<LGN_BF16, 1>();
        else if (mask_kind == LGN_MASK_U8) f.template operator()<LGN_BF16, 2>();
        else f.template operator()<LGN_BF16, 0>();
    } else {
        if (mask_kind == LGN_MASK_SAME_DTYPE) f.template operator()<LGN_F16, 1>();
        else if (mask_kind == LGN_MASK_U8) f.template operator()<LGN_F16, 2>();
        else f.template operator()<LGN_F16, 0>();
    }
}

struct Stage1Launch {
    const void *g, *mask;
    uint64_t n;
    Partial *partials;
    int blocks;
    hipStream_t stream;
    template <int DTYPE, int MASK>
    void operator()() const
    {
        stats_stage1<DTYPE, MASK><<<blocks, kBlock, 0, stream>>>(g, mask, n, kept_vectors(), partials);
    }
};

struct SolveLaunch {
    const void *g, *mask;
    uint64_t n;
    Partial *partials;
    unsigned int *ticket;
    SolveRequest rq;
    lgn_stats_t *st;
    lgn_prune_params_t *p;
    lgn_fp_params_t *f;
    int blocks;
    hipStream_t stream;
    template <int DTYPE, int MASK>
    void operator()() const
    {
        stats_solve_kernel<DTYPE, MASK><<<blocks, kBlock, 0, stream>>>(g, mask, n, kept_vectors(), partials, ticket, rq,
                                                                   st, p, f);
    }
};

hipError_t launch_stats(const void *g, const void *mask, int mask_kind, uint64_t n, int dtype,
                        lgn_stats_t *out, void *ws, hipStream_t stream)
{
    int blocks = stats_blocks(n, dtype);
    if (blocks > stats_blocks_cap(dtype)) blocks = stats_blocks_cap(dtype);
    Partial *partials = static_cast<Partial *>(ws);
    dispatch_dtype_mask(dtype, mask_kind, Stage1Launch{g, mask, n, partials, blocks, stream});
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    stats_stage2<<<1, kBlock, 0, stream>>>(partials, blocks, n, out);
    return hipGetLastError();
}

hipError_t launch_stats_solve(const void *g, const void *mask, int mask_kind, uint64_t n, int dtype,
                              double target_sparsity, int alpha_dtype, int n_bits, int e_bits,
                              int scale_mode, double scale_z, int sigma_units, lgn_stats_t *st,
                              lgn_prune_params_t *p, lgn_fp_params_t *f, void *ws,
                              hipStream_t stream)
{
    int blocks = stats_blocks(n, dtype);
    if (blocks > stats_blocks_cap(dtype)) blocks = stats_blocks_cap(dtype);
    Partial *partials = static_cast<Partial *>(ws);
    unsigned int *ticket = reinterpret_cast<unsigned int *>(static_cast<char *>(ws) + kTicketOffset);
    const int strict = tuning(LGN_TUNE_STATS_STRICT_PUBLISH) ? 0x100 : 0;
    const SolveRequest rq = {target_sparsity, alpha_dtype | strict, n_bits, e_bits, scale_mode, sigma_units, scale_z};
    dispatch_dtype_mask(dtype, mask_kind,
                        SolveLaunch{g, mask, n, partials, ticket, rq, st, p, f, blocks, stream});
    return hipGetLastError();
}

// Statistics + solvers for `count` tensors in as few launches as the argument tables allow
// (kBatchMax tensors each).  Tensor t gets a share of the grid proportional to its size.
hipError_t launch_batch_stats_solve(const lgn_batch_item_t *items, int count, int dtype, int alpha_dtype,
                                    int scale_mode, double scale_z, int sigma_units, void *ws,
                                    hipStream_t stream)
{
    const int cap = stats_blocks_cap(dtype);
    const uint64_t keep_total = kept_vectors();
    for (int c0 = 0; c0 < count; c0 += kBatchMax) {
        const int m = count - c0 < kBatchMax ? count - c0 : kBatchMax;
        BatchStatsArgs a;
        a.partials = static_cast<Partial *>(ws);
        a.tickets = reinterpret_cast<unsigned int *>(static_cast<char *>(ws) + kTicketOffset);
        a.scale_z = scale_z;
        a.alpha_dtype = alpha_dtype | (tuning(LGN_TUNE_STATS_STRICT_PUBLISH) ? 0x100 : 0); a.scale_mode = scale_mode; a.sigma_units = sigma_units; a.count = m;
        long double total = 0.0L;
        for (int i = 0; i < m; ++i) total += (long double)items[c0 + i].n;
        // leave room for the one workgroup every tensor gets at least and for the rounding, so that
        // the slices together never exceed the records the workspace holds
        const int room = cap < kMaxStatsBlocks - 2 * kBatchMax ? cap : kMaxStatsBlocks - 2 * kBatchMax;
        const int budget = room > m ? room - m : 1;
        uint32_t next = 0;
        for (int i = 0; i < kBatchMax; ++i) {
            a.first_block[i] = 0xffffffffu;
            if (i >= m) { a.t[i] = BatchStatsTensor{}; continue; }
            const lgn_batch_item_t &it = items[c0 + i];
            int blocks = total > 0.0L ? (int)((long double)budget * (long double)it.n / total + 0.5L) : 0;
            if (blocks > stats_blocks(it.n, dtype)) blocks = stats_blocks(it.n, dtype);
            if (blocks < 1) blocks = 1;
            BatchStatsTensor &T = a.t[i];
            T.g = it.g; T.n = it.n;
            T.keep_vecs = total > 0.0L ? (uint64_t)((long double)keep_total * (long double)it.n / total) : 0;
            T.target_sparsity = it.target_sparsity >= 0.0 ? it.target_sparsity : -1.0;
            T.st = it.st; T.p = it.target_sparsity >= 0.0 ? it.p : nullptr; T.f = it.n_bits ? it.f : nullptr;
            T.blocks = (uint32_t)blocks;
            T.n_bits = (int16_t)it.n_bits; T.e_bits = (int16_t)it.e_bits;
            a.first_block[i] = next;
            next += (uint32_t)blocks;
        }
        if (next > (uint32_t)kMaxStatsBlocks) return hipErrorInvalidValue;  // cannot happen, see `room`
        if (dtype == LGN_F32) stats_solve_batch_kernel<LGN_F32><<<next, kBlock, 0, stream>>>(a);
        else if (dtype == LGN_BF16) stats_solve_batch_kernel<LGN_BF16><<<next, kBlock, 0, stream>>>(a);
        else stats_solve_batch_kernel<LGN_F16><<<next, kBlock, 0, stream>>>(a);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// ---- the same launch on a scratch array the library owns ------------------------------------
// For callers that cannot provide a workspace because they cannot allocate one: the per-block
// records and the ticket live in a file-scope device array (one copy per GPU the library runs
// on, held until the process ends).  Host code never uses the array's name as an address: the
// device address is asked for once per device and kept.
constexpr size_t kScratchBytes = kTicketOffset + kTicketBytes;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

static hipError_t scratch_address(void **out)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void *ptr[kMaxDevices] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));  // this device's copy of the array
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return hipSuccess;
}

hipError_t launch_stats_solve_static(const void *g, const void *mask, int mask_kind, uint64_t n,
                                     int dtype, double target_sparsity, int alpha_dtype, int n_bits,
                                     int e_bits, int scale_mode, double scale_z, int sigma_units,
                                     lgn_stats_t *st, lgn_prune_params_t *p, lgn_fp_params_t *f,
                                     hipStream_t stream)
{
    void *ws = nullptr;
    hipError_t e = scratch_address(&ws);
    if (e != hipSuccess) return e;
    // The array keeps whatever the last call on this GPU left: the ticket must start at zero (a
    // fill kernel, not a memset, so that the sequence can be captured in a graph); the records
    // are overwritten before they are read.
    e = launch_workspace_init(ws, stream);
    if (e != hipSuccess) return e;
    return launch_stats_solve(g, mask, mask_kind, n, dtype, target_sparsity, alpha_dtype, n_bits, e_bits,
                              scale_mode, scale_z, sigma_units, st, p, f, ws, stream);
}

size_t stats_scratch_bytes() { return kScratchBytes; }

}  // namespace lgn

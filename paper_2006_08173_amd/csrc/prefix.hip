// Prefix code of a pruned tensor (appendix "Encoding", table of codewords):
//     0 -> "0",   +alpha -> "100",   -alpha -> "101",   any other value -> "11" + the value.
// After stochastic pruning most elements are 0 or +-alpha, so the stream is a few bits per value.
//
// An element is its raw pattern of W bits (fp32 32, bf16 16, FP-n code N); the top bit is the
// sign and `special` the magnitude pattern of alpha.  Only the all-zero pattern takes the one-bit
// codeword, so the code is lossless for any input.  Stream bit k is bit (k & 7) of byte k >> 3,
// codewords are written first symbol first, the value after "11" least significant bit first.
//
// Container: chunks of 4096 elements, each starting on a 32-bit boundary listed in a table
// (table[c] = first word of chunk c, table[nchunks] = total words, table[nchunks+1] = status).
// Variable-length output needs the chunk sizes before anything can be placed, hence three
// launches: count (words per chunk), scan (one workgroup, in place), emit.  One workgroup owns a
// chunk; thread t owns its elements 16t .. 16t+15, a block-wide exclusive scan of the threads'
// bit counts gives each thread its offset, the chunk is assembled in LDS (first and last word of
// a thread with LDS atomic OR, interior words with plain stores) and copied out coalesced.
#include "fpcode_device.hpp"

namespace lgn {

constexpr int kChunk = LGN_PREFIX_CHUNK;          // elements per chunk
constexpr int kPerThread = kChunk / kBlock;       // 16 consecutive elements per thread
constexpr int kChunkWordsMax = (kChunk * 34 + 31) / 32;  // fp32: 2 + 32 bits per element

static_assert(kPerThread == 16, "a thread reads its elements as 16-byte vectors");

struct PrefixArgs {
    const void *in;      // elements (encode) / stream (decode)
    void *out;           // stream (encode) / elements (decode)
    uint64_t n;
    uint64_t capacity_words;
    uint64_t *table;
    const lgn_prune_params_t *p;
    const lgn_fp_params_t *f;
};

// WIDTH_CLASS: 0 = FP-n codes in bytes (W = n_bits of *f), 1 = bf16 patterns, 2 = fp32 patterns.
template <int WC>
struct Elem;
template <>
struct Elem<0> { using T = uint8_t; };
template <>
struct Elem<1> { using T = uint16_t; };
template <>
struct Elem<2> { using T = uint32_t; };

// Width in bits and the magnitude pattern of alpha (0: no special class).
template <int WC>
__device__ __forceinline__ void prefix_consts(const PrefixArgs &a, int &width, uint32_t &special)
{
    float alpha = 0.0f;
    if (a.p) alpha = a.p->alpha;
    const uint32_t ab = __float_as_uint(alpha) & 0x7fffffffu;
    if (WC == 2) {
        width = 32;
        special = ab;
    } else if (WC == 1) {
        width = 16;
        special = bf16_round_hi(ab) >> 16;
    } else {
        QuantConst q = {8, 1, 6, 0, 0, 1, 255u};
        if (a.f) load_quant_const(a.f, q);
        width = q.n_bits;
        // the code alpha itself takes with nearest rounding: with stochastic rounding the
        // survivors of pruning split between this code and its neighbour, this one gets more
        special = (ab != 0u && a.f) ? (quant_code<LGN_ROUND_NEAREST_EVEN>(ab, 0u, q) & q.maxmag) : 0u;
    }
    width = __builtin_amdgcn_readfirstlane(width);
    special = (uint32_t)__builtin_amdgcn_readfirstlane((int)special);
}

__device__ __forceinline__ int symbol_len(uint32_t v, int width, uint32_t special)
{
    const uint32_t mag = v & ((1u << (width - 1)) - 1u);
    if (v == 0u) return 1;
    if (special != 0u && mag == special) return 3;
    return 2 + width;
}

// The 16 elements of a thread; elements at or beyond n are marked absent (pattern irrelevant).
template <int WC>
__device__ __forceinline__ int load_thread_elems(const void *in, uint64_t first, uint64_t n,
                                                 uint32_t v[kPerThread])
{
    using T = typename Elem<WC>::T;
    const T *src = reinterpret_cast<const T *>(in);
    if (first + kPerThread <= n) {
        constexpr int kVecs = kPerThread * (int)sizeof(T) / 16;
        const uint4 *vp = reinterpret_cast<const uint4 *>(src + first);  // 16-byte aligned: first % 16 == 0
#pragma unroll
        for (int k = 0; k < kVecs; ++k) {
            const uint4 x = vp[k];
            const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (WC == 2) {
                    v[k * 4 + j] = w[j];
                } else if (WC == 1) {
                    v[(k * 4 + j) * 2] = w[j] & 0xffffu;
                    v[(k * 4 + j) * 2 + 1] = w[j] >> 16;
                } else {
                    v[j * 4] = w[j] & 0xffu;
                    v[j * 4 + 1] = (w[j] >> 8) & 0xffu;
                    v[j * 4 + 2] = (w[j] >> 16) & 0xffu;
                    v[j * 4 + 3] = w[j] >> 24;
                }
            }
        }
        return kPerThread;
    }
    int count = 0;
#pragma unroll
    for (int j = 0; j < kPerThread; ++j) {
        v[j] = 0u;
        if (first + j < n) {
            v[j] = src[first + j];
            count = j + 1;
        }
    }
    return count;
}

// Exclusive scan of one value per thread over the workgroup; also returns the total.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t x, uint32_t &total)
{
    __shared__ uint32_t wave_sum[kBlock / kWave];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    uint32_t incl = x;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const uint32_t up = __shfl_up(incl, off);
        if (lane >= off) incl += up;
    }
    __syncthreads();  // previous use of wave_sum is over
    if (lane == kWave - 1) wave_sum[wave] = incl;
    __syncthreads();
    uint32_t base = 0, sum = 0;
#pragma unroll
    for (int w = 0; w < kBlock / kWave; ++w) {
        if (w < wave) base += wave_sum[w];
        sum += wave_sum[w];
    }
    total = sum;
    return base + incl - x;
}

// ---- launch 1: words per chunk -> table[c + 1] ----------------------------------------------
template <int WC>
__global__ __launch_bounds__(kBlock) void prefix_count_kernel(PrefixArgs a)
{
    int width;
    uint32_t special;
    prefix_consts<WC>(a, width, special);
    const uint64_t nchunks = (a.n + kChunk - 1) / kChunk;
    for (uint64_t c = blockIdx.x; c < nchunks; c += gridDim.x) {
        uint32_t v[kPerThread];
        const int count = load_thread_elems<WC>(a.in, c * kChunk + (uint64_t)threadIdx.x * kPerThread, a.n, v);
        uint32_t bits = 0;
#pragma unroll
        for (int j = 0; j < kPerThread; ++j)
            if (j < count) bits += (uint32_t)symbol_len(v[j], width, special);
        uint32_t total;
        block_exclusive_scan(bits, total);
        if (threadIdx.x == 0) a.table[c + 1] = (total + 31u) / 32u;
    }
}

// ---- launch 2: in-place exclusive scan of the table (one workgroup) --------------------------
constexpr int kScanThreads = 1024;

__global__ __launch_bounds__(kScanThreads) void prefix_scan_kernel(uint64_t *table, uint64_t nchunks)
{
    __shared__ uint64_t part[kScanThreads];
    const uint64_t per = (nchunks + kScanThreads - 1) / kScanThreads;
    const uint64_t lo = min((uint64_t)threadIdx.x * per, nchunks), hi = min(lo + per, nchunks);
    uint64_t sum = 0;
    for (uint64_t c = lo; c < hi; ++c) sum += table[c + 1];
    part[threadIdx.x] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint64_t run = 0;
        for (int t = 0; t < kScanThreads; ++t) {
            const uint64_t x = part[t];
            part[t] = run;
            run += x;
        }
        table[0] = 0;
        table[nchunks + 1] = 0;  // status: cleared here, set by the emit pass on overflow
    }
    __syncthreads();
    uint64_t run = part[threadIdx.x];
    for (uint64_t c = lo; c < hi; ++c) {
        run += table[c + 1];
        table[c + 1] = run;  // entry c + 1 = first word of chunk c + 1 = end of chunk c
    }
}

// ---- launch 3: assemble each chunk in LDS and copy it out ------------------------------------
struct BitWriter {
    uint32_t *lds;
    uint64_t acc;     // bits not yet written; the low `fill` bits are in place
    uint32_t fill;    // < 32 between puts
    uint32_t word;    // index of the word the low bits of acc belong to
    bool first;       // the next flushed word may be shared with the previous thread

    __device__ __forceinline__ void put(uint32_t bits, int len)  // len <= 32
    {
        acc |= (uint64_t)bits << fill;
        fill += (uint32_t)len;
        if (fill >= 32u) {
            const uint32_t w = (uint32_t)acc;
            if (first) atomicOr(lds + word, w);
            else lds[word] = w;
            first = false;
            acc >>= 32;
            fill -= 32u;
            ++word;
        }
    }
    __device__ __forceinline__ void finish()
    {
        if (fill) atomicOr(lds + word, (uint32_t)acc);  // shared with the next thread
    }
};

template <int WC>
__global__ __launch_bounds__(kBlock) void prefix_emit_kernel(PrefixArgs a)
{
    __shared__ uint32_t buf[kChunkWordsMax];
    int width;
    uint32_t special;
    prefix_consts<WC>(a, width, special);
    const uint64_t nchunks = (a.n + kChunk - 1) / kChunk;
    uint32_t *out = reinterpret_cast<uint32_t *>(a.out);
    for (uint64_t c = blockIdx.x; c < nchunks; c += gridDim.x) {
        const uint64_t w0 = a.table[c];
        // what the count pass found for this chunk; never more than the LDS buffer holds
        const uint32_t nwords = (uint32_t)min(a.table[c + 1] - w0, (uint64_t)kChunkWordsMax);
        for (uint32_t i = threadIdx.x; i < nwords; i += kBlock) buf[i] = 0u;
        uint32_t v[kPerThread];
        const int count = load_thread_elems<WC>(a.in, c * kChunk + (uint64_t)threadIdx.x * kPerThread, a.n, v);
        uint32_t bits = 0;
#pragma unroll
        for (int j = 0; j < kPerThread; ++j)
            if (j < count) bits += (uint32_t)symbol_len(v[j], width, special);
        uint32_t total;
        const uint32_t off = block_exclusive_scan(bits, total);  // its barriers also cover the zeroing
        BitWriter bw = {buf, 0ull, off & 31u, off >> 5, true};
#pragma unroll
        for (int j = 0; j < kPerThread; ++j) {
            if (j < count) {
                const int len = symbol_len(v[j], width, special);
                if (len == 1) {
                    bw.put(0u, 1);
                } else if (len == 3) {
                    bw.put(1u | (((v[j] >> (width - 1)) & 1u) << 2), 3);
                } else {
                    bw.put(3u, 2);
                    bw.put(width == 32 ? v[j] : (v[j] & ((1u << width) - 1u)), width);
                }
            }
        }
        bw.finish();
        __syncthreads();
        if (w0 + nwords <= a.capacity_words) {
            for (uint32_t i = threadIdx.x; i < nwords; i += kBlock) out[w0 + i] = buf[i];
        } else if (threadIdx.x == 0) {
            a.table[nchunks + 1] = 1;  // stream buffer too small: this chunk is not written
        }
        __syncthreads();  // buf is reused by the next chunk
    }
}

// ---- decode: one thread per chunk (sequential by nature; not on the hot path) ----------------
template <int WC>
__global__ __launch_bounds__(kBlock) void prefix_decode_kernel(PrefixArgs a)
{
    using T = typename Elem<WC>::T;
    int width;
    uint32_t special;
    prefix_consts<WC>(a, width, special);
    const uint64_t nchunks = (a.n + kChunk - 1) / kChunk;
    const uint32_t *in = reinterpret_cast<const uint32_t *>(a.in);
    T *out = reinterpret_cast<T *>(a.out);
    const uint64_t c = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (c >= nchunks) return;
    const uint64_t first = c * kChunk, last = min(first + kChunk, a.n);
    const uint64_t wend = a.table[c + 1];
    uint64_t w = a.table[c];
    uint64_t acc = 0;   // bits fetched and not yet consumed, low bits first
    uint32_t have = 0;
    auto need = [&](uint32_t k) {  // make at least k <= 32 bits available (zeros past the chunk)
        if (have < k) {
            const uint32_t x = w < wend ? in[w] : 0u;
            ++w;
            acc |= (uint64_t)x << have;
            have += 32u;
        }
    };
    auto take = [&](uint32_t k) {
        need(k);
        const uint32_t r = k == 32u ? (uint32_t)acc : ((uint32_t)acc & ((1u << k) - 1u));
        acc >>= k;
        have -= k;
        return r;
    };
    for (uint64_t i = first; i < last; ++i) {
        uint32_t v = 0u;
        if (take(1)) {
            if (take(1)) v = take((uint32_t)width);
            else v = special | (take(1) << (width - 1));
        }
        out[i] = (T)v;
    }
}

static int prefix_grid(uint64_t nchunks)
{
    const uint64_t cap = 256 * 8;
    return (int)(nchunks < 1 ? 1 : (nchunks < cap ? nchunks : cap));
}

template <int WC>
static hipError_t encode_launches(const PrefixArgs &a, hipStream_t stream)
{
    const uint64_t nchunks = (a.n + kChunk - 1) / kChunk;
    if (nchunks) {
        prefix_count_kernel<WC><<<prefix_grid(nchunks), kBlock, 0, stream>>>(a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    prefix_scan_kernel<<<1, kScanThreads, 0, stream>>>(a.table, nchunks);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || !nchunks) return e;
    prefix_emit_kernel<WC><<<prefix_grid(nchunks), kBlock, 0, stream>>>(a);
    return hipGetLastError();
}

hipError_t launch_prefix_encode(int width_class, const void *in, uint64_t n, const lgn_prune_params_t *p,
                                const lgn_fp_params_t *f, void *out, uint64_t capacity_words,
                                uint64_t *table, hipStream_t stream)
{
    const PrefixArgs a = {in, out, n, capacity_words, table, p, f};
    if (width_class == 2) return encode_launches<2>(a, stream);
    if (width_class == 1) return encode_launches<1>(a, stream);
    return encode_launches<0>(a, stream);
}

hipError_t launch_prefix_decode(int width_class, const void *in, const uint64_t *table, uint64_t n,
                                const lgn_prune_params_t *p, const lgn_fp_params_t *f, void *out,
                                hipStream_t stream)
{
    const uint64_t nchunks = (n + kChunk - 1) / kChunk;
    if (!nchunks) return hipSuccess;
    const PrefixArgs a = {in, out, n, 0, const_cast<uint64_t *>(table), p, f};
    const int blocks = (int)((nchunks + kBlock - 1) / kBlock);
    if (width_class == 2) prefix_decode_kernel<2><<<blocks, kBlock, 0, stream>>>(a);
    else if (width_class == 1) prefix_decode_kernel<1><<<blocks, kBlock, 0, stream>>>(a);
    else prefix_decode_kernel<0><<<blocks, kBlock, 0, stream>>>(a);
    return hipGetLastError();
}

}  // namespace lgn

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
// (table[c] = first word of chunk c, table[nchunks] = total words, table[nchunks+1] = status),
// and behind the table the bit lengths of every chunk's 16 sub-blocks of 256 elements (16-bit
// numbers), so that the decoder can start a parser at every 256th element.
// Variable-length output needs the chunk sizes before anything can be placed, hence three
// launches.  Count: words per chunk, one wave per chunk, and their sum per workgroup.  Scan: one
// small workgroup turns the per-workgroup sums into first-word offsets.  Emit: a workgroup walks
// its contiguous run of chunks; an exclusive scan of the bit counts gives every thread (16-bit
// and 32-bit patterns: 16 elements per thread, a workgroup per chunk) or lane (byte codes: 64 per
// lane, a wave per chunk) its position, and the chunk is assembled in a zero-initialised LDS
// image with atomic ORs -- only non-zero elements write anything, the codeword "0" is the zero
// bit that is already there -- then copied out coalesced while the image is cleared for the next
// chunk.
#include "launch.hpp"
#include "fpcode_device.hpp"

namespace lgn {

constexpr int kChunk = LGN_PREFIX_CHUNK;          // elements per chunk
constexpr int kPerThread = kChunk / kBlock;       // 16 consecutive elements per thread
constexpr int kChunkWordsMax = (kChunk * 34 + 31) / 32;  // fp32: 2 + 32 bits per element
constexpr int kSub = 256;                         // elements per sub-block
constexpr int kSubsPerChunk = kChunk / kSub;      // 16

static_assert(kSub == kPerThread * 16, "a sub-block is the elements of 16 consecutive threads of the emit pass");
static_assert(kSub * 34 < 65536, "a sub-block's length fits 16 bits");

// The sub-block lengths live behind the chunk table and the encoder's scratch entries.
__host__ __device__ __forceinline__ uint16_t *sub_lengths(uint64_t *table, uint64_t nchunks)
{
    return reinterpret_cast<uint16_t *>(table + nchunks + 2 + LGN_PREFIX_MAX_BLOCKS);
}

static_assert(kPerThread == 16, "a thread reads its elements as 16-byte vectors");

struct PrefixArgs {
    const void *in;      // elements (encode) / stream (decode)
    void *out;           // stream (encode) / elements (decode)
    uint64_t n;
    uint64_t capacity_words;
    uint64_t *table;
    const lgn_prune_params_t *p;
    const lgn_fp_params_t *f;
    int dtype;           // element type of VALUE input (tells bf16 from fp16 among the 16-bit patterns)
};

// WIDTH_CLASS: 0 = FP-n codes in bytes (W = n_bits of *f), 1 = 16-bit patterns (bf16 or fp16),
// 2 = fp32 patterns.
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
        special = a.dtype == LGN_F16 ? (f32_bits_to_f16(ab) & 0x7fffu) : (bf16_round_hi(ab) >> 16);
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

template <typename T>
__device__ __forceinline__ T wave_inclusive_scan(T x)
{
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const T up = __shfl_up(x, off);
        if (lane >= off) x += up;
    }
    return x;
}

// Chunks are dealt to workgroups in contiguous runs, so that a workgroup knows the offsets of its
// own chunks from a running sum and only one number per workgroup has to be scanned globally.
struct ChunkRun {
    uint64_t first, last;  // chunks [first, last) of this workgroup
};

__device__ __forceinline__ ChunkRun chunk_run(uint64_t nchunks)
{
    const uint64_t per = (nchunks + gridDim.x - 1) / gridDim.x;
    ChunkRun r;
    r.first = min((uint64_t)blockIdx.x * per, nchunks);
    r.last = min(r.first + per, nchunks);
    return r;
}

// ---- launch 1: words per chunk -> table[c + 1], words per workgroup -> scratch[block] --------
// Wave-synchronous: a wave sums the codeword lengths of whole chunks (order does not matter for
// a sum, so the loads are lane-contiguous 16-byte vectors); no barrier until the final total.
template <int WC>
__global__ __launch_bounds__(kBlock) void prefix_count_kernel(PrefixArgs a, uint64_t *scratch)
{
    using T = typename Elem<WC>::T;
    constexpr int EPV = 16 / (int)sizeof(T);             // elements per 16-byte vector
    constexpr int kVecsPerLane = kChunk / (EPV * kWave);  // 4 (codes), 8 (bf16), 16 (fp32)
    __shared__ uint64_t wave_words[kBlock / kWave];
    int width;
    uint32_t special;
    prefix_consts<WC>(a, width, special);
    const uint64_t nchunks = (a.n + kChunk - 1) / kChunk;
    const ChunkRun run = chunk_run(nchunks);
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const T *src = reinterpret_cast<const T *>(a.in);
    uint64_t words = 0;  // wave-uniform
    for (uint64_t c = run.first + wave; c < run.last; c += kBlock / kWave) {
        const uint64_t e0 = c * kChunk;
        uint32_t bits = 0;
        if (e0 + kChunk <= a.n) {
            const uint4 *vp = reinterpret_cast<const uint4 *>(src + e0) + lane;
#pragma unroll
            for (int k = 0; k < kVecsPerLane; ++k) {
                const uint4 x = vp[k * kWave];
                const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (WC == 2) {
                        bits += (uint32_t)symbol_len(w[j], width, special);
                    } else if (WC == 1) {
                        bits += (uint32_t)symbol_len(w[j] & 0xffffu, width, special);
                        bits += (uint32_t)symbol_len(w[j] >> 16, width, special);
                    } else {
#pragma unroll
                        for (int t = 0; t < 4; ++t)
                            bits += (uint32_t)symbol_len((w[j] >> (8 * t)) & 0xffu, width, special);
                    }
                }
            }
        } else {  // the ragged last chunk, element by element
            for (uint64_t i = e0 + lane; i < a.n; i += kWave)
                bits += (uint32_t)symbol_len(src[i], width, special);
        }
        const uint32_t total = __shfl(wave_inclusive_scan(bits), kWave - 1);
        const uint32_t w32 = (total + 31u) / 32u;
        if (lane == 0) a.table[c + 1] = w32;
        words += w32;
    }
    if (lane == 0) wave_words[wave] = words;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint64_t sum = 0;
        for (int w = 0; w < kBlock / kWave; ++w) sum += wave_words[w];
        scratch[blockIdx.x] = sum;
    }
}

// ---- launch 2: exclusive scan of the per-workgroup totals (one workgroup) --------------------
constexpr int kScanThreads = 1024;
constexpr int kMaxPrefixBlocks = LGN_PREFIX_MAX_BLOCKS;  // two totals per scanning thread

__global__ __launch_bounds__(kScanThreads) void prefix_scan_kernel(uint64_t *table, uint64_t nchunks,
                                                                   uint64_t *scratch, int nblocks)
{
    __shared__ uint64_t wave_sum[kScanThreads / kWave];
    const int i0 = 2 * threadIdx.x, i1 = i0 + 1;
    const uint64_t x0 = i0 < nblocks ? scratch[i0] : 0, x1 = i1 < nblocks ? scratch[i1] : 0;
    const uint64_t incl = wave_inclusive_scan(x0 + x1);
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    if (lane == kWave - 1) wave_sum[wave] = incl;
    __syncthreads();
    uint64_t base = 0;
    for (int w = 0; w < wave; ++w) base += wave_sum[w];
    const uint64_t excl = base + incl - (x0 + x1);
    if (i0 < nblocks) scratch[i0] = excl;        // first word of the workgroup's first chunk
    if (i1 < nblocks) scratch[i1] = excl + x0;
    if (threadIdx.x == 0) {
        table[0] = 0;
        table[nchunks + 1] = 0;  // status: cleared here, set by the emit pass on overflow
    }
}

// ---- launch 3: assemble each chunk in LDS and copy it out ------------------------------------
// ORs `len` <= 32 bits into the zero-initialised LDS image of the chunk at bit position `pos`.
__device__ __forceinline__ void lds_put(uint32_t *buf, uint32_t pos, uint32_t bits)
{
    const uint64_t x = (uint64_t)bits << (pos & 31u);
    const uint32_t lo = (uint32_t)x, hi = (uint32_t)(x >> 32);
    atomicOr(buf + (pos >> 5), lo);
    if (hi) atomicOr(buf + (pos >> 5) + 1, hi);
}

// 16-bit and 32-bit patterns: a workgroup per chunk, 16 elements per thread.
template <int WC>
__global__ __launch_bounds__(kBlock) void prefix_emit_kernel(PrefixArgs a, const uint64_t *scratch)
{
    static_assert(WC == 1 || WC == 2, "byte codes have a kernel of their own");
    __shared__ uint32_t buf[kChunkWordsMax + 1];  // + 1: the word after the last bit may be ORed with 0
    __shared__ uint32_t wave_sum[kBlock / kWave];
    int width;
    uint32_t special;
    prefix_consts<WC>(a, width, special);
    const uint32_t payload_mask = width == 32 ? 0xffffffffu : (1u << width) - 1u;
    const uint64_t nchunks = (a.n + kChunk - 1) / kChunk;
    const ChunkRun run = chunk_run(nchunks);
    uint32_t *out = reinterpret_cast<uint32_t *>(a.out);
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    for (uint32_t i = threadIdx.x; i < (uint32_t)kChunkWordsMax + 1u; i += kBlock) buf[i] = 0u;
    uint64_t w0 = scratch[blockIdx.x];  // first word of the current chunk
    bool overflow = false;
    __syncthreads();
    for (uint64_t c = run.first; c < run.last; ++c) {
        const uint64_t first = c * kChunk + (uint64_t)threadIdx.x * kPerThread;
        uint32_t v[kPerThread];
        uint32_t bits = 0;
        const int count = load_thread_elems<WC>(a.in, first, a.n, v);
#pragma unroll
        for (int j = 0; j < kPerThread; ++j)
            if (j < count) bits += (uint32_t)symbol_len(v[j], width, special);
        const uint32_t incl = wave_inclusive_scan(bits);
        if (lane == kWave - 1) wave_sum[wave] = incl;
        {
            // length of each sub-block: 16 consecutive threads, four sub-blocks per wave
            const uint32_t start = __shfl(incl - bits, lane & ~15);
            if ((lane & 15) == 15)
                sub_lengths(a.table, nchunks)[c * kSubsPerChunk + (uint64_t)(wave * 4 + (lane >> 4))] =
                    (uint16_t)(incl - start);
        }
        __syncthreads();
        uint32_t pos = incl - bits, total = 0;
#pragma unroll
        for (int w = 0; w < kBlock / kWave; ++w) {
            if (w < wave) pos += wave_sum[w];
            total += wave_sum[w];
        }
        // zero symbols are the zero bits the image already holds: only the others are written
#pragma unroll
        for (int j = 0; j < kPerThread; ++j) {
            if (j < count) {
                const uint32_t x = v[j];
                const bool is_special = special != 0u && (x & ((1u << (width - 1)) - 1u)) == special;
                const uint32_t head = is_special ? (1u | (((x >> (width - 1)) & 1u) << 2)) : 3u;
                if (WC == 2) {
                    if (x != 0u) lds_put(buf, pos, head);
                    if (x != 0u && !is_special) lds_put(buf, pos + 2u, x);
                } else {
                    // at most 2 + 16 bits
                    if (x != 0u) lds_put(buf, pos, is_special ? head : (3u | ((x & payload_mask) << 2)));
                }
                pos += x == 0u ? 1u : (is_special ? 3u : 2u + (uint32_t)width);
            }
        }
        __syncthreads();
        const uint32_t nwords = (total + 31u) / 32u;  // = what the count pass stored in table[c + 1]
        const bool fits = w0 + nwords <= a.capacity_words;
        for (uint32_t i = threadIdx.x; i < nwords; i += kBlock) {
            if (fits) out[w0 + i] = buf[i];
            buf[i] = 0u;
        }
        overflow |= !fits;
        w0 += nwords;
        if (threadIdx.x == 0) a.table[c + 1] = w0;  // end of chunk c = first word of chunk c + 1
        __syncthreads();  // the image and wave_sum are reused by the next chunk
    }
    if (overflow && threadIdx.x == 0) a.table[nchunks + 1] = 1;  // stream buffer too small
}

// ---- launch 3 for byte codes: one wave per chunk ----------------------------------------------
// After pruning some 85 % of the codes are zero and cost nothing, so the emit pass is bound by the
// loop over the non-zero ones, which runs as often as the busiest lane of a wave needs.  With 64
// consecutive codes per lane instead of 16 the busiest lane is much closer to the average one
// (binomial counts: about 16 of 64 against 7 of 16 at 15 % non-zero), and a chunk is one wave's
// work: no workgroup barrier, one scan, one LDS image per wave.  A wave walks every fourth chunk
// of its workgroup's run; the chunks' first words come from the table, which wave 0 first turns
// from words per chunk into running ends for the whole run.
constexpr int kLaneCodes = kChunk / kWave;                // 64 consecutive codes per lane
constexpr int kByteImageWords = (kChunk * 10 + 31) / 32;  // at most 2 + 8 bits per code
static_assert(kSub % kLaneCodes == 0, "a sub-block is the codes of whole lanes");

// The 64 codes of a lane as sixteen words; codes at or beyond n read as zero.
__device__ __forceinline__ void load_lane_codes(const uint8_t *src, uint64_t first, uint64_t n, uint4 x[4])
{
    if (first + kLaneCodes <= n) {
        const uint4 *vp = reinterpret_cast<const uint4 *>(src + first);  // first % 64 == 0
#pragma unroll
        for (int k = 0; k < 4; ++k) x[k] = vp[k];
        return;
    }
    uint32_t w[16];
    for (int k = 0; k < 16; ++k) {
        w[k] = 0u;
        for (int t = 0; t < 4; ++t) {
            const uint64_t i = first + (uint64_t)(4 * k + t);
            if (i < n) w[k] |= (uint32_t)src[i] << (8 * t);
        }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) x[k] = make_uint4(w[4 * k], w[4 * k + 1], w[4 * k + 2], w[4 * k + 3]);
}

__global__ __launch_bounds__(kBlock) void prefix_emit_bytes_kernel(PrefixArgs a, const uint64_t *scratch)
{
    constexpr int kWaves = kBlock / kWave;
    __shared__ uint32_t image[kWaves][kByteImageWords + 1];  // + 1: the word after the last bit may be ORed with 0
    // a lane's codes, for the loop over the non-zero ones: word k of lane l at [k * 64 + l], so
    // that a lane only ever touches its own column and no two lanes share a bank
    __shared__ uint32_t codes[kWaves][(kLaneCodes / 4) * kWave];
    int width;
    uint32_t special;
    prefix_consts<0>(a, width, special);
    const uint32_t payload_mask = (1u << width) - 1u;
    const uint32_t mag_mask = (1u << (width - 1)) - 1u;  // <= 0x7f: the per-byte sums below cannot carry
    const uint32_t mag4 = mag_mask * 0x01010101u, sp4 = special * 0x01010101u;
    const uint32_t special_or_none = special ? special : 0x100u;  // 0x100: no masked byte equals it
    const uint64_t nchunks = (a.n + kChunk - 1) / kChunk;
    const ChunkRun run = chunk_run(nchunks);
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
    const uint8_t *src = static_cast<const uint8_t *>(a.in);
    uint32_t *out = reinterpret_cast<uint32_t *>(a.out);
    uint32_t *img = image[wave];
    uint32_t *mine = codes[wave] + lane;
    for (int i = lane; i < kByteImageWords + 1; i += kWave) img[i] = 0u;

    uint64_t c = run.first + (uint64_t)wave;
    uint4 x[4] = {make_uint4(0u, 0u, 0u, 0u), make_uint4(0u, 0u, 0u, 0u), make_uint4(0u, 0u, 0u, 0u),
                  make_uint4(0u, 0u, 0u, 0u)};
    if (c < run.last) load_lane_codes(src, c * kChunk + (uint64_t)lane * kLaneCodes, a.n, x);  // in flight during the scan

    if (wave == 0) {  // words per chunk -> end of each chunk, for this workgroup's run
        uint64_t carry = scratch[blockIdx.x];
        for (uint64_t base = run.first; base < run.last; base += kWave) {
            const uint64_t idx = base + (uint64_t)lane;
            const uint64_t words = idx < run.last ? a.table[idx + 1] : 0;
            const uint64_t incl = wave_inclusive_scan(words);
            if (idx < run.last) a.table[idx + 1] = carry + incl;
            carry += __shfl(incl, kWave - 1);
        }
    }
    __syncthreads();

    bool overflow = false;
    for (; c < run.last; c += kWaves) {
        const uint32_t d[16] = {x[0].x, x[0].y, x[0].z, x[0].w, x[1].x, x[1].y, x[1].z, x[1].w,
                                x[2].x, x[2].y, x[2].z, x[2].w, x[3].x, x[3].y, x[3].z, x[3].w};
        const uint64_t lane_first = c * kChunk + (uint64_t)lane * kLaneCodes;
        if (c + kWaves < run.last)  // the next chunk of this wave, in flight while this one is assembled
            load_lane_codes(src, lane_first + (uint64_t)kWaves * kChunk, a.n, x);
        const uint64_t w0 = c == run.first ? scratch[blockIdx.x] : a.table[c];

        // which codes are non-zero (a 64-bit mask in element order) and how many are +-alpha
        uint32_t nz_lo = 0u, nz_hi = 0u, n_sp = 0u;
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            mine[k * kWave] = d[k];
            // bit 7 of a byte: that byte of d is non-zero
            const uint32_t nz = (((d[k] & 0x7f7f7f7fu) + 0x7f7f7f7fu) | d[k]) & 0x80808080u;
            // a zero byte of t: that code's magnitude is alpha's
            const uint32_t t = (d[k] & mag4) ^ sp4;
            n_sp += (uint32_t)__popc(~(t + 0x7f7f7f7fu) & 0x80808080u);
            // bits 7, 15, 23, 31 gathered into a nibble
            const uint32_t nib = (((nz >> 7) * 0x00204081u) >> 21) & 0xfu;
            if (k < 8) nz_lo |= nib << (4 * k);
            else nz_hi |= nib << (4 * (k - 8));
        }
        if (special == 0u) n_sp = 0u;
        const uint32_t n_nz = (uint32_t)__popc(nz_lo) + (uint32_t)__popc(nz_hi);
        const uint32_t present =
            lane_first + kLaneCodes <= a.n ? (uint32_t)kLaneCodes : (lane_first < a.n ? (uint32_t)(a.n - lane_first) : 0u);
        const uint32_t bits = present + n_nz * (1u + (uint32_t)width) - n_sp * ((uint32_t)width - 1u);
        const uint32_t incl = wave_inclusive_scan(bits);
        const uint32_t total = __shfl(incl, kWave - 1);
        const uint32_t pos = incl - bits;
        {
            // length of each sub-block: the codes of four consecutive lanes
            const uint32_t start = __shfl(pos, lane & ~3);
            if ((lane & 3) == 3)
                sub_lengths(a.table, nchunks)[c * kSubsPerChunk + (uint64_t)(lane >> 2)] = (uint16_t)(incl - start);
        }

        // zero symbols are the zero bits the image already holds: only the others are written
        uint64_t todo = ((uint64_t)nz_hi << 32) | nz_lo;
        uint32_t extra = 0;  // bits beyond one per code, of the codes before the current one
        const uint8_t *bytes = reinterpret_cast<const uint8_t *>(mine);
        while (todo) {
            const uint32_t j = (uint32_t)__ffsll((unsigned long long)todo) - 1u;
            todo &= todo - 1ull;
            const uint32_t v = bytes[(j >> 2) * (kWave * 4u) + (j & 3u)];
            const bool sp = (v & mag_mask) == special_or_none;
            // "1", then "0" and the sign (+-alpha) or "1" and the code
            const uint32_t rest = sp ? ((v >> (width - 1)) & 1u) << 1 : ((v & payload_mask) << 1) | 1u;
            const uint32_t p = pos + j + extra;
            const uint64_t w = (uint64_t)((rest << 1) | 1u) << (p & 31u);
            atomicOr(img + (p >> 5), (uint32_t)w);
            atomicOr(img + (p >> 5) + 1, (uint32_t)(w >> 32));  // often zero: cheaper than asking
            extra += sp ? 2u : 1u + (uint32_t)width;
        }

        // the image is complete once every lane's ORs are done: LDS serves a wave's requests in order
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        const uint32_t nwords = (total + 31u) / 32u;  // = what the count pass found for this chunk
        const bool fits = w0 + nwords <= a.capacity_words;
        for (uint32_t i = (uint32_t)lane; i < nwords; i += kWave) {
            if (fits) out[w0 + i] = img[i];
            img[i] = 0u;
        }
        overflow |= !fits;
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
    if (overflow && lane == 0) a.table[nchunks + 1] = 1;  // stream buffer too small
}

// ---- decode: one thread per sub-block of 256 elements (a prefix code is sequential by nature; the
// listed sub-block lengths give sixteen starting points per chunk) --------------------------------
template <int WC>
__global__ __launch_bounds__(kBlock) void prefix_decode_kernel(PrefixArgs a)
{
    using T = typename Elem<WC>::T;
    constexpr int EPV = 16 / (int)sizeof(T);
    int width;
    uint32_t special;
    prefix_consts<WC>(a, width, special);
    const uint64_t nchunks = (a.n + kChunk - 1) / kChunk;
    const uint32_t *in = reinterpret_cast<const uint32_t *>(a.in);
    T *out = reinterpret_cast<T *>(a.out);
    const uint32_t tid = threadIdx.x;
    const uint64_t nsub = (a.n + kSub - 1) / kSub;
    const uint64_t sb = (uint64_t)blockIdx.x * kBlock + tid;  // this thread's sub-block
    const uint64_t c = sb / kSubsPerChunk;
    const uint32_t j = (uint32_t)(sb % kSubsPerChunk);
    // a thread without a sub-block reads nothing and decodes zeros; it still helps to copy out
    const uint64_t wend = sb < nsub ? a.table[c + 1] : 0;
    uint32_t skip = 0;  // bits of the chunk before this sub-block
    if (sb < nsub) {
        const uint2 *lp = reinterpret_cast<const uint2 *>(sub_lengths(a.table, nchunks) + c * kSubsPerChunk);
#pragma unroll
        for (uint32_t k = 0; k < 4; ++k) {
            const uint2 x = lp[k];
            const uint32_t len[4] = {x.x & 0xffffu, x.x >> 16, x.y & 0xffffu, x.y >> 16};
#pragma unroll
            for (uint32_t t = 0; t < 4; ++t) skip += 4 * k + t < j ? len[t] : 0u;
        }
    }
    uint64_t w = sb < nsub ? a.table[c] + (skip >> 5) : 0;  // next word to request

    // The threads of a wave sit in different symbols of different chunks, and a wait for memory
    // holds the whole wave, so nothing that waits may sit in a branch only some threads take.
    // Input therefore goes through a ring of 16 words per thread in LDS (word j of thread t at
    // j * kBlock + t: a thread only ever touches its own column, and the bank is fixed by t).
    // Once per step, at the same point for every thread, the free slots of the ring (at most six:
    // a step consumes at most 160 bits) are requested from memory, and they are stored into the
    // ring at the end of the step, after the step's symbols have been decoded.  Words past the
    // end of the chunk read as zero.
    constexpr uint32_t kRing = 16, kTop = 6;
    __shared__ uint32_t ring[kRing * kBlock];
    uint32_t rd = 0, wr = kRing;  // words moved to the accumulator / words stored in the ring
#pragma unroll
    for (uint32_t j = 0; j < kRing; ++j) ring[j * kBlock + tid] = w + j < wend ? in[w + j] : 0u;
    w += kRing;
    uint64_t acc = 0;   // bits not yet consumed, low bits first
    uint32_t have = 0;  // how many
    uint32_t next = ring[tid];  // word `rd` of the chunk, read ahead of its use
    // Tops the accumulator up to at least 32 bits; selects, no branch, and the ring is read at
    // every call so that the read is waited for at the next call, not in a branch.
    auto refill = [&]() {
        const bool need = have < 32u;
        const uint64_t moved = (uint64_t)next << (have & 31u);
        acc |= need ? moved : 0ull;
        have += need ? 32u : 0u;
        rd += need ? 1u : 0u;
        next = ring[(rd & (kRing - 1u)) * kBlock + tid];
    };
    const uint32_t payload_mask = width == 32 ? 0xffffffffu : (1u << width) - 1u;
    // A symbol is classified from its first two bits, again with selects.  A top-up leaves at
    // least 32 bits, and a byte code takes at most 2 + 8 of them, so for byte codes only every
    // third symbol needs one.
    auto symbol = [&](bool top_up) {
        if (top_up) refill();
        const uint32_t lo = (uint32_t)acc;
        const bool nonzero = (lo & 1u) != 0u, value = (lo & 3u) == 3u;
        uint32_t v = nonzero ? special | (((lo >> 2) & 1u) << (width - 1)) : 0u;
        if (WC != 2) {  // 2 + width <= 18 bits: the whole symbol is in `lo`
            const uint32_t len = nonzero ? (value ? 2u + (uint32_t)width : 3u) : 1u;
            v = value ? (lo >> 2) & payload_mask : v;
            acc >>= len;
            have -= len;
        } else {  // 2 + 32 bits: the head, then the payload after a second top-up
            const uint32_t head = nonzero ? (value ? 2u : 3u) : 1u;
            acc >>= head;
            have -= head;
            refill();
            v = value ? (uint32_t)acc : v;
            const uint32_t len = value ? 32u : 0u;
            acc >>= len;
            have -= len;
        }
        return v;
    };

    // the sub-block starts inside its first word
    refill();
    acc >>= (skip & 31u);
    have -= (skip & 31u);

    // Output: a thread produces 16 bytes per step, 256 elements apart from its neighbours'.
    // kLine steps are collected in LDS (16 * kLine bytes per thread, slots rotated by the thread
    // index to spread the banks) and then written by the wave as whole lines: lane l writes piece
    // l % kLine of the thread l / kLine + (64 / kLine) k.  Only wave-level ordering is needed.
    // Four steps (64-byte lines) rather than eight: the smaller buffer lets a fourth workgroup
    // fit a compute unit, and the parsers are bound by latency, not by the stores.
    constexpr int kLine = 4, kRows = kWave / kLine;
    __shared__ uint4 stage[kBlock * kLine];
    const int lane = (int)tid & (kWave - 1);
    const int wave_first = (int)tid - lane;                      // first thread of this wave
    const uint64_t wave_sub = (uint64_t)blockIdx.x * kBlock + (uint64_t)wave_first;
    constexpr int kSteps = kSub / EPV;
    static_assert(kSteps % kLine == 0, "whole lines");
    bool dense = false;  // byte codes: which of the two forms of a step this wave takes next (wave-uniform)
    for (int step = 0; step < kSteps; ++step) {
        const uint32_t fresh = min(kRing - (wr - rd), kTop);  // free slots of the ring
        uint32_t top[kTop];
#pragma unroll
        for (uint32_t j = 0; j < kTop; ++j) top[j] = (j < fresh && w + j < wend) ? in[w + j] : 0u;
        uint4 *slot = stage + tid * kLine + ((step + (int)tid) & (kLine - 1));
        if (WC == 0 && !dense) {
            // Byte codes, most of them zero: the step's sixteen bytes start as zeros in LDS, a run
            // of "0" codewords is skipped in one go (count of trailing zero bits, at most up to
            // the end of the step) and only the non-zero codes are parsed and stored.  The loop
            // runs once per non-zero code of the busiest lane (and ends after at most sixteen
            // rounds whatever the bits are); a top-up at every round keeps at least 32 bits,
            // enough for sixteen zeros and one codeword of at most ten.
            *slot = make_uint4(0u, 0u, 0u, 0u);
            uint8_t *bytes = reinterpret_cast<uint8_t *>(slot);
            uint32_t pos = 0, busy = 0;
            while (pos < (uint32_t)EPV) {
                refill();
                const uint32_t lo = (uint32_t)acc;
                const uint32_t room = (uint32_t)EPV - pos;
                uint32_t first_one;  // index of the lowest set bit; 0xffffffff if there is none
                asm("v_ffbl_b32 %0, %1" : "=v"(first_one) : "v"(lo));
                const uint32_t z = min(first_one, room);
                const bool more = z < room;  // then bit z is a "1"
                const uint32_t sym = lo >> z;
                const bool value = (sym & 2u) != 0u;
                const uint32_t v = value ? (sym >> 2) & payload_mask : special | (((sym >> 2) & 1u) << (width - 1));
                const uint32_t used = z + (more ? (value ? 2u + (uint32_t)width : 3u) : 0u);
                acc >>= used;
                have -= used;
                if (more) bytes[pos + z] = (uint8_t)v;
                pos += z + 1u;
                ++busy;
            }
            // a round costs about twice a symbol of the other form: that one is the better
            // choice from about ten non-zero codes among sixteen in the busiest lane
            dense = __builtin_amdgcn_ballot_w64(busy > 10u) != 0ull;
        } else {
            uint32_t q[4] = {0u, 0u, 0u, 0u};
            uint32_t busy = 0;
#pragma unroll
            for (int j = 0; j < EPV; ++j) {
                const uint32_t v = symbol(WC != 0 || j % 3 == 0);
                if (WC == 2) q[j] = v;
                else if (WC == 1) q[j / 2] |= v << (16 * (j % 2));
                else q[j / 4] |= v << (8 * (j % 4));
                if (WC == 0) busy += v != 0u ? 1u : 0u;
            }
            *slot = make_uint4(q[0], q[1], q[2], q[3]);
            if (WC == 0) dense = __builtin_amdgcn_ballot_w64(busy > 8u) != 0ull;
        }
#pragma unroll
        for (uint32_t j = 0; j < kTop; ++j)
            if (j < fresh) ring[((wr + j) & (kRing - 1u)) * kBlock + tid] = top[j];
        wr += fresh;
        w += fresh;
        if ((step & (kLine - 1)) != kLine - 1) continue;
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        const int piece = lane & (kLine - 1);             // 16-byte piece of the line
        const int pstep = (step & ~(kLine - 1)) + piece;  // the step that produced it
#pragma unroll
        for (int k = 0; k < kLine; ++k) {
            const int t = wave_first + k * kRows + lane / kLine;  // thread whose line this lane writes
            const uint64_t block = wave_sub + (uint64_t)(k * kRows + lane / kLine);
            const uint4 x = stage[t * kLine + ((pstep + t) & (kLine - 1))];
            if (block >= nsub) continue;
            const uint64_t e0 = block * kSub + (uint64_t)pstep * EPV;  // first element of the piece
            if (e0 + EPV <= a.n) {
                *reinterpret_cast<uint4 *>(out + e0) = x;
            } else if (e0 < a.n) {  // the ragged end of the tensor, element by element
                const uint32_t xs[4] = {x.x, x.y, x.z, x.w};
                for (int j = 0; e0 + j < a.n; ++j) {
                    if (WC == 2) out[e0 + j] = (T)xs[j];
                    else if (WC == 1) out[e0 + j] = (T)(xs[j / 2] >> (16 * (j % 2)));
                    else out[e0 + j] = (T)(xs[j / 4] >> (8 * (j % 4)));
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

static int prefix_grid(uint64_t nchunks)
{
    const uint64_t cap = kMaxPrefixBlocks;
    return (int)(nchunks < 1 ? 1 : (nchunks < cap ? nchunks : cap));
}

template <int WC>
static hipError_t encode_launches(const PrefixArgs &a, hipStream_t stream)
{
    const uint64_t nchunks = (a.n + kChunk - 1) / kChunk;
    uint64_t *scratch = a.table + nchunks + 2;  // per-workgroup totals, then first words
    const int blocks = prefix_grid(nchunks);
    if (nchunks) {
        prefix_count_kernel<WC><<<blocks, kBlock, 0, stream>>>(a, scratch);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    prefix_scan_kernel<<<1, kScanThreads, 0, stream>>>(a.table, nchunks, scratch, nchunks ? blocks : 0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || !nchunks) return e;
    if constexpr (WC == 0) prefix_emit_bytes_kernel<<<blocks, kBlock, 0, stream>>>(a, scratch);
    else prefix_emit_kernel<WC><<<blocks, kBlock, 0, stream>>>(a, scratch);
    return hipGetLastError();
}

hipError_t launch_prefix_encode(int width_class, int dtype, const void *in, uint64_t n,
                                const lgn_prune_params_t *p, const lgn_fp_params_t *f, void *out,
                                uint64_t capacity_words, uint64_t *table, hipStream_t stream)
{
    const PrefixArgs a = {in, out, n, capacity_words, table, p, f, dtype};
    if (width_class == 2) return encode_launches<2>(a, stream);
    if (width_class == 1) return encode_launches<1>(a, stream);
    return encode_launches<0>(a, stream);
}

hipError_t launch_prefix_decode(int width_class, int dtype, const void *in, const uint64_t *table,
                                uint64_t n, const lgn_prune_params_t *p, const lgn_fp_params_t *f,
                                void *out, hipStream_t stream)
{
    const uint64_t nchunks = (n + kChunk - 1) / kChunk;
    if (!nchunks) return hipSuccess;
    const PrefixArgs a = {in, out, n, 0, const_cast<uint64_t *>(table), p, f, dtype};
    const uint64_t nsub = (n + kSub - 1) / kSub;
    const int blocks = (int)((nsub + kBlock - 1) / kBlock);
    if (width_class == 2) prefix_decode_kernel<2><<<blocks, kBlock, 0, stream>>>(a);
    else if (width_class == 1) prefix_decode_kernel<1><<<blocks, kBlock, 0, stream>>>(a);
    else prefix_decode_kernel<0><<<blocks, kBlock, 0, stream>>>(a);
    return hipGetLastError();
}

}  // namespace lgn

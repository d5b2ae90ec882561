// The streaming operators: stochastic pruning T_{alpha,eps} (Section 5, first equation), the
// FP(1,e,m) quantizer with power-of-two scale (Section 4.1; Alg. 1), and both in one pass.
//
// One kernel template covers prune-only, quantize-only and the fused pass.  A wave owns tiles of
// 256 consecutive elements; lane l owns elements 4l..4l+3 of the tile, i.e. exactly one Philox
// block (one word per element: upper half prunes, lower half rounds), one 16-byte load (fp32) and
// one 16-byte / 4-byte store.  Everything is
// integer work on fp32 bit patterns (bf16 widens by a shift, fp16 by the exact conversion), except
// the one single-precision product alpha * u that the pruning rule is defined with.
//
// Two code paths per tile.  The fast path covers full tiles whose global quad indices share the
// upper counter word, with elem_offset a multiple of four, a normal-range alpha and a scale that
// flushes fp32 subnormals (the case for any sane gradient scale): there the first Philox rounds
// run partly on the scalar unit, the three-way xors are single v_bitop3 instructions, and the
// per-element work is ten instructions (stochastic rounding, re-biasing and the sign are one
// 64-bit multiply-add).  Everything else (ragged tail tile, unaligned offsets, exotic scales)
// takes the general path; both give identical bits.
//
// PACKED output: the four N-bit codes of a lane form a 4N-bit chunk; the 64 chunks of a tile are
// one contiguous run of 8N dwords.  Lane k < 8N assembles dword k from the (at most five) chunks
// that overlap it, fetched with cross-lane reads, and the wave stores 8N consecutive dwords.
//
// This header holds the kernel template; stream_f32.hip, stream_bf16.hip and stream_f16.hip
// instantiate it for one element type each (they compile in parallel), stream.hip launches.
#pragma once

#include "launch.hpp"
#include "lgn_device.hpp"
#include "fpcode_device.hpp"

namespace lgn {

// Words of the four elements j0..j0+3; j0 need not be a multiple of four.
__device__ __forceinline__ void quad_words(uint64_t j0, PhiloxKey key, uint32_t w[4])
{
    const uint32_t r = (uint32_t)j0 & 3u;  // wave-uniform: tiles start at multiples of four
    uint32_t a[4];
    philox_block(j0 >> 2, key, a);
    if (r == 0u) {
        w[0] = a[0]; w[1] = a[1]; w[2] = a[2]; w[3] = a[3];
    } else {
        uint32_t b[4];
        philox_block((j0 >> 2) + 1, key, b);
        if (r == 1u) { w[0] = a[1]; w[1] = a[2]; w[2] = a[3]; w[3] = b[0]; }
        else if (r == 2u) { w[0] = a[2]; w[1] = a[3]; w[2] = b[0]; w[3] = b[1]; }
        else { w[0] = a[3]; w[1] = b[0]; w[2] = b[1]; w[3] = b[2]; }
    }
}

// T_{alpha,u}: |x| > alpha keeps x; |x| < fl32(alpha u) gives 0; otherwise sign(x) alpha, with
// u = ((w >> 16) + 1/2) / 2^16 in (0, 1): the upper half of the element's word.  Zero stays
// (+)zero whatever alpha u rounds to; NaN and Inf compare above any finite alpha and pass.
__device__ __forceinline__ uint32_t prune_bits(uint32_t bits, uint32_t w, uint32_t alpha_bits,
                                               float alpha)
{
    const uint32_t a = bits & 0x7fffffffu;
    const float u = (float)((w & 0xffff0000u) | 0x8000u) * 0x1p-32f;  // exact: 17 significant bits
    const uint32_t t = __float_as_uint(alpha * u);                    // one rounding
    const uint32_t small = (a < t || a == 0u) ? 0u : (alpha_bits | (bits & 0x80000000u));
    return a > alpha_bits ? bits : small;
}

// PACKED output of one 256-element tile: lane i holds the 4N-bit chunk of its four codes, and the
// tile's run of 32N bytes is the chunks end to end.  The lane in whose chunk a dword of the run
// begins assembles that dword: the rest of its own chunk from bit `o` on, then the chunks of the
// next one to three lanes.  Lanes fall into aligned groups of 8 / gcd(N, 8) whose chunks make up
// whole dwords, so the neighbours a dword needs are in the same row of 16 lanes and come over
// with row shifts (plain vector instructions, no LDS).  Everything here depends on the lane and
// on N only and is computed once per kernel.
struct PackLane {
    bool owns;        // a dword begins in this lane's chunk
    uint32_t dword;   // its index in the tile's run
    uint32_t o;       // first bit of it inside the chunk
    uint32_t s1, s2, s3;  // left shifts of the chunks of lanes i+1, i+2, i+3 (32 or more: not part of it)
    int neighbours;   // how many of them some lane needs (wave-uniform)
};

__device__ __forceinline__ PackLane pack_lane(int n_bits, int lane)
{
    PackLane p;
    const uint32_t cb = 4u * (uint32_t)n_bits, first = cb * (uint32_t)lane;
    p.dword = (first + 31u) / 32u;
    p.owns = 32u * p.dword < first + cb;
    p.o = p.owns ? 32u * p.dword - first : 0u;
    p.s1 = cb - p.o;
    p.s2 = 2u * cb - p.o;
    p.s3 = 3u * cb - p.o;
    p.neighbours = n_bits <= 3 ? 3 : (n_bits == 5 ? 2 : (n_bits == 8 ? 0 : 1));
    return p;
}

// The value lane i + K of the same row of 16 holds (0 past the end of the row).
template <int K>
__device__ __forceinline__ uint32_t from_lane_above(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x100 + K, 0xf, 0xf, true);  // row_shl:K
}

__device__ __forceinline__ void pack_store_n(const PackLane &p, int lane, uint32_t chunk,
                                             uint8_t *tile_out, uint64_t bytes_valid)
{
    uint32_t dword = chunk >> p.o;
    // 64-bit shifts: a shift of 32 or more leaves nothing in the low word.  The first neighbour is
    // merged unconditionally (for N = 8, where no dword spans two lanes, its shift is 32): the
    // common formats then run without a branch here.
    dword |= (uint32_t)((uint64_t)from_lane_above<1>(chunk) << p.s1);
    if (p.neighbours >= 2) dword |= (uint32_t)((uint64_t)from_lane_above<2>(chunk) << p.s2);
    if (p.neighbours >= 3) dword |= (uint32_t)((uint64_t)from_lane_above<3>(chunk) << p.s3);
    if (p.owns) {
        const uint64_t byte = 4ull * p.dword;
        if (byte + 4 <= bytes_valid) {
            __builtin_nontemporal_store(dword, reinterpret_cast<uint32_t *>(tile_out) + p.dword);
        } else {
            for (uint64_t b = byte; b < bytes_valid; ++b)
                tile_out[b] = (uint8_t)(dword >> (8 * (b - byte)));
        }
    }
}

// ---- fast path ------------------------------------------------------------------------------
// Wave-uniform constants of the fast path.
struct FastConst {
    uint32_t alpha_bits;
    float alpha16;     // alpha * 2^-16 and alpha * 2^-17 (exact for the alphas the fast path
    float alpha17;     // accepts): fl32(alpha u) = fma(k, alpha16, alpha17) for u = (k + 1/2) / 2^16
    uint32_t sub;      // cbias << 23: subtracting it re-biases the exponent field
    uint32_t sub_hi;   // -(cbias << m) mod 2^32: the same subtraction applied to a magnitude code
    uint32_t lo_bits;  // smallest magnitude pattern that is not flushed
    uint32_t sat_bits; // smallest magnitude pattern that gives the largest code without rounding
    uint32_t floor_bits;  // lower clamp of the magnitude: min(alpha, sat_bits) when pruning, else 0
    uint32_t cut;      // 23 - m
    uint32_t rmul;     // 2^(9+m)
    uint32_t sshift;   // e + m: position of the sign bit in a code
    uint32_t rnd;      // 2^(cut-1) - 1, the nearest-even increment before the parity bit
};

// One element of the fused / quantize-only fast path; returns the code (sign included).
// `a` is |x| as a bit pattern, clamped to [floor_bits, sat_bits] by the caller: the lower clamp
// raises what pruning keeps to alpha, the upper clamp is the saturation rule (a magnitude clamped
// to sat_bits has no remainder, so rounding cannot carry past the largest code; Inf and NaN
// patterns lie above sat_bits).  `keep` is false where pruning zeroed the element.  Stochastic
// rounding is one 64-bit multiply-add: with r the lower half of the element's word, the upper half
// of y * 2^(9+m) + (r * 2^16 + 2^15) is (y + (r + 1/2) 2^(7-m)) >> (23-m), i.e. y goes up iff its
// cut-off fraction plus (r + 1/2) / 2^16 reaches one.
// CHECK_LO = false is used when every magnitude that reaches the quantizer is known to be at or
// above the flush threshold (fused pass with alpha >= 2^(E_min+s)).
template <int ROUND, bool CHECK_LO>
__device__ __forceinline__ uint32_t fast_code(uint32_t bits, uint32_t a, bool keep, uint32_t w,
                                              const FastConst &c)
{
    uint32_t code;
    if (ROUND == LGN_ROUND_STOCHASTIC) {
        // upper word of  a * 2^(9+m) + w  plus, in the upper word of the addend, the sign bit at
        // its place in the code minus the re-biasing (cbias << m): sub * 2^(9+m) is a multiple of
        // 2^32, and the re-biased magnitude code stays below the sign bit, so nothing carries.
        // Written as asm so that the sum stays one v_mad_u64_u32 with a ready-made addend.
        const uint64_t addend = ((uint64_t)(((bits >> 31) << c.sshift) + c.sub_hi) << 32) | ((w << 16) | 0x8000u);
        uint64_t r, carry;  // the carry-out goes to a scalar pair of the allocator's choice, not vcc
        asm("v_mad_u64_u32 %0, %1, %2, %3, %4" : "=v"(r), "=s"(carry) : "v"(a), "s"(c.rmul), "v"(addend));
        code = (uint32_t)(r >> 32);
    } else {
        const uint32_t y = a - c.sub;
        const uint32_t mag = (y + c.rnd + ((y >> c.cut) & 1u)) >> c.cut;
        code = ((bits >> 31) << c.sshift) | mag;
    }
    const bool valid = CHECK_LO ? (a >= c.lo_bits && keep) : keep;
    return valid ? code : 0u;
}

// clamp(x, lo, hi) for lo <= hi: the median of the three, one instruction.  The compiler forms
// v_med3_u32 only for constant bounds, hence the asm; one bound sits in a vector register because
// an instruction of this family reads at most one scalar register.
__device__ __forceinline__ uint32_t clamp_u32(uint32_t x, uint32_t lo, uint32_t hi)
{
    uint32_t r;
    asm("v_med3_u32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "v"(lo), "s"(hi));
    return r;
}

// Four byte-sized codes into one dword with three byte permutes (selector 0x0c yields zero).
__device__ __forceinline__ uint32_t merge_bytes(const uint32_t code[4])
{
    const uint32_t lo = __builtin_amdgcn_perm(code[1], code[0], 0x0c0c0400u);
    const uint32_t hi = __builtin_amdgcn_perm(code[3], code[2], 0x04000c0cu);
    return lo | hi;
}

template <int DTYPE>
__device__ __forceinline__ const char *tile_in(const StreamArgs &a, uint64_t tile)
{
    return reinterpret_cast<const char *>(a.g) + tile * (uint64_t)(kWave * (DTYPE == LGN_F32 ? 16 : 8));
}

// A full tile whose loads are already in b[].
// PRUNE: the call prunes; DO_PRUNE: alpha is non-zero, so pruning actually draws random words.
template <int DTYPE, bool PRUNE, bool DO_PRUNE, bool QUANT, int ROUND, int OUT, bool CHECK_LO>
__device__ __forceinline__ void fast_tile(const StreamArgs &a, uint64_t tile, uint64_t qbase,
                                          int lane, PhiloxKey key, const FastConst &c,
                                          const QuantConst &q, const PackLane &pk, uint32_t b[4])
{
    constexpr int QB = DTYPE == LGN_F32 ? 16 : 8;  // bytes per quad
    const uint32_t q_lo = (uint32_t)qbase + (uint32_t)lane;  // no carry: checked by the caller
    const uint32_t q_hi = (uint32_t)(qbase >> 32);
    // one word per element: upper half for pruning, lower half for stochastic rounding
    uint32_t w[4] = {0u, 0u, 0u, 0u};
    if (DO_PRUNE || (QUANT && ROUND == LGN_ROUND_STOCHASTIC)) {
        const uint64_t p0 = (uint64_t)kPhiloxM0 * q_lo;
        philox_finish((uint32_t)(p0 >> 32), (uint32_t)p0, q_hi, key, w);
        // Two of the four words are low halves of products; without this the compiler turns their
        // later shift by 16 into a second multiply by M << 16 plus an or (two instructions where
        // one shift-or does).
#pragma unroll
        for (int t = 0; t < 4; ++t) asm volatile("" : "+v"(w[t]));
    }

    uint32_t mag_in[4];
    bool keep[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const uint32_t ab = b[t] & 0x7fffffffu;
        mag_in[t] = ab;
        keep[t] = true;
        if (DO_PRUNE) {
            const float kf = (float)(w[t] >> 16);
            const uint32_t thr = __float_as_uint(__builtin_fmaf(kf, c.alpha16, c.alpha17));
            keep[t] = !(ab < thr);
            if (!QUANT) {
                const uint32_t small = keep[t] ? (c.alpha_bits | (b[t] & 0x80000000u)) : 0u;
                b[t] = ab > c.alpha_bits ? b[t] : small;
            }
        } else if (PRUNE && !QUANT) {
            b[t] = ab ? b[t] : 0u;  // alpha = 0: only -0 changes
        }
        // below alpha the survivor is +-alpha; above the range the code saturates
        if (QUANT) mag_in[t] = clamp_u32(ab, c.floor_bits, c.sat_bits);
    }
    if (!QUANT) {
        char *gout = reinterpret_cast<char *>(a.out) + tile * (uint64_t)(kWave * QB);
        store_quad<DTYPE>(gout, (uint32_t)lane, b);
        return;
    }
    uint32_t code[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
        code[t] = fast_code<ROUND, CHECK_LO>(b[t], mag_in[t], keep[t], w[t], c);
    if (OUT == LGN_OUT_VALUE) {
        uint32_t v[4];
#pragma unroll
        for (int t = 0; t < 4; ++t)
            v[t] = (b[t] & 0x7fffffffu) > 0x7f800000u ? b[t] : code_value_bits(code[t], q);
        char *gout = reinterpret_cast<char *>(a.out) + tile * (uint64_t)(kWave * QB);
        store_quad<DTYPE>(gout, (uint32_t)lane, v);
    } else if (OUT == LGN_OUT_CODE8) {
        uint32_t *gout = reinterpret_cast<uint32_t *>(a.out) + tile * (uint64_t)kWave;
        __builtin_nontemporal_store(merge_bytes(code), gout + (uint32_t)lane);
    } else {
        const int N = q.n_bits;
        const uint32_t chunk = code[0] | (code[1] << N) | (code[2] << (2 * N)) | (code[3] << (3 * N));
        pack_store_n(pk, lane, chunk, reinterpret_cast<uint8_t *>(a.out) + tile * 32ull * (uint64_t)N,
                     ~0ull);
    }
}

// ---- general path: any tile, any offset, any scale ------------------------------------------
template <int DTYPE, bool PRUNE, bool QUANT, int ROUND, int OUT>
__device__ __forceinline__ void general_tile(const StreamArgs &a, uint64_t tile, int lane,
                                             PhiloxKey key, float alpha, const QuantConst &q,
                                             const PackLane &pk, uint64_t packed_total)
{
    const uint64_t n = a.n;
    const uint32_t alpha_bits = __float_as_uint(alpha);
    const uint64_t quad = tile * kWave + lane;  // index of this lane's four elements
    const uint64_t i0 = quad * 4;
    const bool full = (tile + 1) * 256 <= n;    // wave-uniform
    uint32_t b[4];
    if (full) {
        load_quad<DTYPE>(a.g, quad, b);
    } else {
#pragma unroll
        for (int t = 0; t < 4; ++t) b[t] = i0 + t < n ? load_elem<DTYPE>(a.g, i0 + t) : 0u;
    }
    const uint64_t j0 = a.elem_offset + i0;
    uint32_t w[4] = {0u, 0u, 0u, 0u};
    if ((PRUNE && alpha_bits != 0u) || (QUANT && ROUND == LGN_ROUND_STOCHASTIC)) quad_words(j0, key, w);
    if (PRUNE && alpha_bits != 0u) {
#pragma unroll
        for (int t = 0; t < 4; ++t) b[t] = prune_bits(b[t], w[t], alpha_bits, alpha);
    } else if (PRUNE) {
#pragma unroll
        for (int t = 0; t < 4; ++t) b[t] = (b[t] & 0x7fffffffu) ? b[t] : 0u;
    }
    if (!QUANT) {
        if (full) {
            store_quad<DTYPE>(a.out, quad, b);
        } else {
#pragma unroll
            for (int t = 0; t < 4; ++t)
                if (i0 + t < n) store_elem<DTYPE>(a.out, i0 + t, b[t]);
        }
        return;
    }
    uint32_t code[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) code[t] = quant_code<ROUND>(b[t], w[t], q);
    if (OUT == LGN_OUT_VALUE) {
        uint32_t v[4];
#pragma unroll
        for (int t = 0; t < 4; ++t)
            v[t] = (b[t] & 0x7fffffffu) > 0x7f800000u ? b[t] : code_value_bits(code[t], q);
        if (full) {
            store_quad<DTYPE>(a.out, quad, v);
        } else {
#pragma unroll
            for (int t = 0; t < 4; ++t)
                if (i0 + t < n) store_elem<DTYPE>(a.out, i0 + t, v[t]);
        }
    } else if (OUT == LGN_OUT_CODE8) {
        if (full) {
            reinterpret_cast<uint32_t *>(a.out)[quad] =
                code[0] | (code[1] << 8) | (code[2] << 16) | (code[3] << 24);
        } else {
#pragma unroll
            for (int t = 0; t < 4; ++t)
                if (i0 + t < n) reinterpret_cast<uint8_t *>(a.out)[i0 + t] = (uint8_t)code[t];
        }
    } else {
        const int N = q.n_bits;
        const uint32_t chunk = code[0] | (code[1] << N) | (code[2] << (2 * N)) | (code[3] << (3 * N));
        const uint64_t tile_byte = tile * 32ull * (uint64_t)N;
        pack_store_n(pk, lane, chunk, reinterpret_cast<uint8_t *>(a.out) + tile_byte,
                     packed_total - tile_byte);
    }
}

// Waves per SIMD the register allocator is asked to leave room for.  Eight (64 VGPRs) is what
// the streaming skeleton likes; the two heaviest variants would spill at that size.
constexpr int stream_min_waves(bool prune, bool quant, int round, int out)
{
    const bool heavy = prune && quant && round == LGN_ROUND_STOCHASTIC;
    return out == LGN_OUT_PACKED ? (heavy ? 4 : 5) : (heavy ? 6 : 7);
}

// Everything a wave needs that does not depend on the tile.
struct WalkState {
    StreamArgs a;
    PhiloxKey key;
    float alpha;
    QuantConst q;
    PackLane pk;
    FastConst c;
    uint64_t ntiles, nwaves, wave, packed_total, qoff;
    int lane;
    bool fast_ok;
};

// The tile loops of one wave.  A wave walks PAIRS of consecutive tiles (2 KiB of fp32 input): both
// loads of the next pair are issued before the current pair is processed, so every wave keeps
// 2 KiB in flight while its Philox and quantizer arithmetic runs.  With eight waves per SIMD that
// is 16 KiB per SIMD, twice what the measured latency x bandwidth product asks for; one tile per
// step was not enough.  DO_PRUNE and CHECK_LO select the fast-tile variant once per kernel, so
// the loops carry no variant dispatch.
//
// First loop: the fast pairs, with 32-bit scalar bookkeeping only (pair index, the low word of the
// quad counter, one compare each) and two register sets used alternately, so that no prefetched
// value is ever copied.  A pair is fast if both tiles are full and its 128 quad indices share the
// upper counter word.  Second loop: whatever the first one left out (the ragged tail, a pair that
// straddles a 2^34-element boundary, everything if the call does not qualify) on the general path.
template <int DTYPE, bool PRUNE, bool DO_PRUNE, bool QUANT, int ROUND, int OUT, bool CHECK_LO>
__device__ __forceinline__ void walk_pairs(const WalkState &s)
{
    const uint64_t n = s.a.n;
    const uint64_t npairs = (s.ntiles + 1) / 2;
    // pairs [0, fast_pairs) consist of full tiles; 32-bit bookkeeping covers tensors below 2^40 elements
    const bool small = npairs <= 0x7fffffffull && s.nwaves <= 0x00ffffffull;
    const uint32_t fast_pairs = (s.fast_ok && small) ? (uint32_t)((n / 256) / 2) : 0u;
    const uint32_t nw = (uint32_t)s.nwaves;
    const uint32_t qstep = nw * 128u;  // quads between two pairs of this wave (mod 2^32)
    auto q_first = [&](uint32_t pair) { return (uint32_t)s.qoff + pair * 128u; };
    auto no_wrap = [](uint32_t q0) { return q0 <= 0xffffff7fu; };  // q0 + 127 stays in the word
    auto load_pair = [&](uint32_t pair, uint32_t *r) {
        const char *base = tile_in<DTYPE>(s.a, 2ull * pair);
        constexpr int QB = DTYPE == LGN_F32 ? 16 : 8;
        load_quad<DTYPE>(base, (uint32_t)s.lane, r);
        load_quad<DTYPE>(base + kWave * QB, (uint32_t)s.lane, r + 4);
    };
    auto run_pair = [&](uint32_t pair, uint32_t *r) {
        const uint64_t t = 2ull * pair;
        const uint64_t qbase = s.qoff + t * kWave;  // global quad index of lane 0
        fast_tile<DTYPE, PRUNE, DO_PRUNE, QUANT, ROUND, OUT, CHECK_LO>(s.a, t, qbase, s.lane, s.key,
                                                                       s.c, s.q, s.pk, r);
        // keep the two tiles' instruction streams apart: interleaving them doubles the live
        // registers and costs two waves of occupancy
        __builtin_amdgcn_sched_barrier(0);
        fast_tile<DTYPE, PRUNE, DO_PRUNE, QUANT, ROUND, OUT, CHECK_LO>(s.a, t + 1, qbase + kWave, s.lane,
                                                                       s.key, s.c, s.q, s.pk, r + 4);
    };

    {
        // Runs of consecutive fast pairs of this wave.  Inside a run every load is unconditional,
        // so the compiler waits for exactly the older pair while the younger one stays in flight.
        uint32_t ra[8], rb[8];
        uint32_t pair = (uint32_t)min(s.wave, (uint64_t)fast_pairs), q0 = q_first(pair);
        while (pair < fast_pairs) {
            if (!no_wrap(q0)) {  // left to the second loop
                pair += nw; q0 += qstep;
                continue;
            }
            load_pair(pair, ra);
            for (;;) {
                // current pair in set A
                uint32_t next = pair + nw, qn = q0 + qstep;
                if (!(next < fast_pairs && no_wrap(qn))) {
                    run_pair(pair, ra);
                    pair = next; q0 = qn;
                    break;
                }
                load_pair(next, rb);
                run_pair(pair, ra);
                pair = next; q0 = qn;
                // current pair in set B
                next = pair + nw; qn = q0 + qstep;
                if (!(next < fast_pairs && no_wrap(qn))) {
                    run_pair(pair, rb);
                    pair = next; q0 = qn;
                    break;
                }
                load_pair(next, ra);
                run_pair(pair, rb);
                pair = next; q0 = qn;
            }
        }
    }

    for (uint64_t pair = s.wave; pair < npairs; pair += s.nwaves) {
        if (pair < fast_pairs && no_wrap(q_first((uint32_t)pair))) continue;  // done above
        general_tile<DTYPE, PRUNE, QUANT, ROUND, OUT>(s.a, 2 * pair, s.lane, s.key, s.alpha, s.q, s.pk,
                                                      s.packed_total);
        if (2 * pair + 1 < s.ntiles)
            general_tile<DTYPE, PRUNE, QUANT, ROUND, OUT>(s.a, 2 * pair + 1, s.lane, s.key, s.alpha, s.q,
                                                          s.pk, s.packed_total);
    }
}

// One workgroup's share of a tensor: workgroup `block` of the `nblocks` that walk it.
template <int DTYPE, bool PRUNE, bool QUANT, int ROUND, int OUT>
__device__ __forceinline__ void stream_body(const StreamArgs &a, uint32_t block, uint32_t nblocks)
{
    WalkState s;
    s.a = a;
    s.key = {a.k0, a.k1};
    s.alpha = 0.0f;
    if (PRUNE) s.alpha = a.p->alpha;
    const uint32_t alpha_bits = __float_as_uint(s.alpha);
    s.q = {8, 1, 6, 0, 0, 1, 255u};
    if (QUANT) load_quant_const(a.f, s.q);
    const QuantConst &q = s.q;
    s.ntiles = (a.n + 255) / 256;
    s.nwaves = (uint64_t)nblocks * (kBlock / kWave);
    s.lane = threadIdx.x & (kWave - 1);
    s.wave = (uint64_t)block * (kBlock / kWave) +
             (uint64_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
    s.packed_total = (a.n * (uint64_t)q.n_bits + 7) / 8;
    s.pk = pack_lane(q.n_bits, s.lane);

    // Fast-path eligibility that does not depend on the tile (all wave-uniform).
    const bool do_prune = PRUNE && alpha_bits != 0u;
    FastConst &c = s.c;
    c.alpha_bits = alpha_bits;
    c.alpha16 = s.alpha * 0x1p-16f;
    c.alpha17 = s.alpha * 0x1p-17f;
    c.sub = (uint32_t)max(q.cbias, 0) << 23;
    c.lo_bits = (uint32_t)min(max(q.cbias + 1, 0), 256) << 23;
    c.cut = 23u - (uint32_t)q.m;
    c.sub_hi = 0u - (c.sub >> c.cut);
    c.sat_bits = (uint32_t)__builtin_amdgcn_readfirstlane((int)(c.sub + (q.maxmag << c.cut)));
    c.floor_bits = do_prune ? min(alpha_bits, c.sat_bits) : 0u;
    c.rmul = 1u << (9u + (uint32_t)q.m);
    c.rmul = (uint32_t)__builtin_amdgcn_readfirstlane((int)c.rmul);  // scalar operand of the asm
    // kept in a vector register: (sign << sshift) + sub_hi is then one shift-and-add (an
    // instruction reads at most one scalar register, and the shift count is the other one)
    asm volatile("" : "+v"(c.sub_hi));
    asm volatile("" : "+v"(c.floor_bits));  // vector operand of the clamp, kept live across tiles
    c.sshift = (uint32_t)(q.e + q.m);
    c.rnd = (1u << (c.cut - 1u)) - 1u;
    // pruning raises every surviving magnitude to alpha: no flush test needed if alpha is in range
    const bool check_lo = !(do_prune && alpha_bits >= c.lo_bits);
    s.fast_ok = (a.elem_offset & 3ull) == 0ull &&
                // the saturation pattern must stay below the Inf pattern, so that the clamp also
                // catches Inf and NaN
                (!QUANT || (q.cbias >= 0 && q.cbias + q.cmax <= 254)) &&
                (!do_prune || (alpha_bits >= 0x12000000u && alpha_bits < 0x7f800000u));
    s.qoff = a.elem_offset >> 2;

    if (PRUNE && do_prune && !check_lo)
        walk_pairs<DTYPE, PRUNE, PRUNE, QUANT, ROUND, OUT, false>(s);
    else if (PRUNE && do_prune)
        walk_pairs<DTYPE, PRUNE, PRUNE, QUANT, ROUND, OUT, true>(s);
    else
        walk_pairs<DTYPE, PRUNE, false, QUANT, ROUND, OUT, true>(s);
}


template <int DTYPE, bool PRUNE, bool QUANT, int ROUND, int OUT>
__global__ __launch_bounds__(kBlock, stream_min_waves(PRUNE, QUANT, ROUND, OUT)) void stream_kernel(StreamArgs a)
{
    stream_body<DTYPE, PRUNE, QUANT, ROUND, OUT>(a, blockIdx.x, gridDim.x);
}

// ---- many tensors, one launch: the fused pass ------------------------------------------------
// The grid is the concatenation of the grids the one-tensor launches would use; a workgroup finds
// its tensor in a table of first workgroup indices (kernel argument) and then does exactly what it
// would do in that tensor's own launch, so the output is the same, bit for bit.
struct BatchStreamTensor {
    const void *g;
    void *out;
    uint64_t n;
    const lgn_prune_params_t *p;
    const lgn_fp_params_t *f;
    uint32_t k0, k1;
    uint32_t blocks, reserved;
};

struct BatchStreamArgs {
    uint32_t first_block[kBatchMax];  // of tensor i; 0xffffffff past the last tensor
    BatchStreamTensor t[kBatchMax];
};
static_assert(sizeof(BatchStreamArgs) <= 4096, "must fit the kernel argument segment");

template <int DTYPE, int ROUND, int OUT>
__global__ __launch_bounds__(kBlock, stream_min_waves(true, true, ROUND, OUT)) void stream_batch_kernel(BatchStreamArgs a)
{
    const uint32_t b = blockIdx.x;
    int t = 0;
#pragma unroll
    for (int i = 1; i < kBatchMax; ++i) t += a.first_block[i] <= b ? 1 : 0;  // uniform: scalar unit
    t = __builtin_amdgcn_readfirstlane(t);
    const BatchStreamTensor &T = a.t[t];
    const StreamArgs one = {T.g, T.out, T.n, 0ull, T.p, T.f, T.k0, T.k1};
    stream_body<DTYPE, true, true, ROUND, OUT>(one, b - a.first_block[t], T.blocks);
}

using StreamBatchKernel = void (*)(BatchStreamArgs);

template <int DTYPE>
StreamBatchKernel pick_batch_kernel(int rounding, int out_kind)
{
    if (rounding == LGN_ROUND_STOCHASTIC) {
        if (out_kind == LGN_OUT_VALUE) return stream_batch_kernel<DTYPE, LGN_ROUND_STOCHASTIC, LGN_OUT_VALUE>;
        if (out_kind == LGN_OUT_CODE8) return stream_batch_kernel<DTYPE, LGN_ROUND_STOCHASTIC, LGN_OUT_CODE8>;
        return stream_batch_kernel<DTYPE, LGN_ROUND_STOCHASTIC, LGN_OUT_PACKED>;
    }
    if (out_kind == LGN_OUT_VALUE) return stream_batch_kernel<DTYPE, LGN_ROUND_NEAREST_EVEN, LGN_OUT_VALUE>;
    if (out_kind == LGN_OUT_CODE8) return stream_batch_kernel<DTYPE, LGN_ROUND_NEAREST_EVEN, LGN_OUT_CODE8>;
    return stream_batch_kernel<DTYPE, LGN_ROUND_NEAREST_EVEN, LGN_OUT_PACKED>;
}

using StreamKernel = void (*)(StreamArgs);

template <int DTYPE, bool PRUNE, bool QUANT>
StreamKernel pick_round_out(int rounding, int out_kind)
{
    if (!QUANT) return stream_kernel<DTYPE, PRUNE, false, LGN_ROUND_NEAREST_EVEN, LGN_OUT_VALUE>;
    if (rounding == LGN_ROUND_STOCHASTIC) {
        if (out_kind == LGN_OUT_VALUE) return stream_kernel<DTYPE, PRUNE, true, LGN_ROUND_STOCHASTIC, LGN_OUT_VALUE>;
        if (out_kind == LGN_OUT_CODE8) return stream_kernel<DTYPE, PRUNE, true, LGN_ROUND_STOCHASTIC, LGN_OUT_CODE8>;
        return stream_kernel<DTYPE, PRUNE, true, LGN_ROUND_STOCHASTIC, LGN_OUT_PACKED>;
    }
    if (out_kind == LGN_OUT_VALUE) return stream_kernel<DTYPE, PRUNE, true, LGN_ROUND_NEAREST_EVEN, LGN_OUT_VALUE>;
    if (out_kind == LGN_OUT_CODE8) return stream_kernel<DTYPE, PRUNE, true, LGN_ROUND_NEAREST_EVEN, LGN_OUT_CODE8>;
    return stream_kernel<DTYPE, PRUNE, true, LGN_ROUND_NEAREST_EVEN, LGN_OUT_PACKED>;
}

template <int DTYPE>
StreamKernel pick_kernel(bool prune, bool quant, int rounding, int out_kind)
{
    return prune ? (quant ? pick_round_out<DTYPE, true, true>(rounding, out_kind)
                          : pick_round_out<DTYPE, true, false>(rounding, out_kind))
                 : pick_round_out<DTYPE, false, true>(rounding, out_kind);
}


// one translation unit per element type
StreamKernel pick_stream_kernel_f32(bool prune, bool quant, int rounding, int out_kind);
StreamKernel pick_stream_kernel_bf16(bool prune, bool quant, int rounding, int out_kind);
StreamKernel pick_stream_kernel_f16(bool prune, bool quant, int rounding, int out_kind);
StreamBatchKernel pick_stream_batch_kernel_f32(int rounding, int out_kind);
StreamBatchKernel pick_stream_batch_kernel_bf16(int rounding, int out_kind);
StreamBatchKernel pick_stream_batch_kernel_f16(int rounding, int out_kind);

}  // namespace lgn

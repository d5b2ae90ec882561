// Device-side helpers shared by the HIP kernels of the lognormal gradient-compression library
// (gfx950 / CDNA4, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/lgn.h"

namespace lgn {

constexpr int kWave = 64;
constexpr int kBlock = 256;            // threads per workgroup (4 waves, one per SIMD)
constexpr int kMaxStatsBlocks = 2048;  // cap of stage-1 partials (fills 256 CUs x 8 waves/SIMD)
constexpr int kBatchMax = 32;          // tensors per launch of the batched entry points

// ---------------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11).  One block = four 32-bit words.  The multiplications are
// written as 64-bit products so the compiler emits one v_mad_u64_u32 per product (both halves).
// The key schedule depends only on the seed and is therefore wave-uniform (scalar registers).
// ---------------------------------------------------------------------------------------------
struct PhiloxKey {
    uint32_t k0, k1;
};

__device__ __forceinline__ void philox_round(uint32_t &c0, uint32_t &c1, uint32_t &c2, uint32_t &c3,
                                             uint32_t k0, uint32_t k1)
{
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
}

// Words of the block with counter (lo32(q), hi32(q), 0, 0): the words of elements 4q..4q+3.
__device__ __forceinline__ void philox_block(uint64_t q, PhiloxKey key, uint32_t w[4])
{
    uint32_t c0 = (uint32_t)q, c1 = (uint32_t)(q >> 32), c2 = 0u, c3 = 0u;
    uint32_t k0 = key.k0, k1 = key.k1;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        philox_round(c0, c1, c2, c3, k0, k1);
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    w[0] = c0;
    w[1] = c1;
    w[2] = c2;
    w[3] = c3;
}

// Three-way xor in one instruction (gfx950 v_bitop3_b32, truth table 0x96).
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c)
{
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

constexpr uint32_t kPhiloxM0 = 0xD2511F53u, kPhiloxM1 = 0xCD9E8D57u;
constexpr uint32_t kPhiloxW0 = 0x9E3779B9u, kPhiloxW1 = 0xBB67AE85u;

// Rounds 1..10 for counter (q_lo, q_hi, 0, 0) when q_hi is wave-uniform and the round-1 product
// hi0:lo0 = M0 * q_lo is already known.  In round 1 the second product is zero, in round 2 the
// first product has uniform operands: the compiler keeps those on the scalar unit, leaving 17
// vector multiplies instead of 20.
__device__ __forceinline__ void philox_finish(uint32_t hi0, uint32_t lo0, uint32_t q_hi,
                                              PhiloxKey key, uint32_t w[4])
{
    uint32_t k0 = key.k0, k1 = key.k1;
    // round 1: (c0, c1, c2, c3) = (q_lo, q_hi, 0, 0)
    uint32_t c0 = q_hi ^ k0;  // uniform
    uint32_t c1 = 0u;
    uint32_t c2 = hi0 ^ k1;
    uint32_t c3 = lo0;
    k0 += kPhiloxW0; k1 += kPhiloxW1;
    {   // round 2: c0 and c1 are uniform
        const uint64_t a = (uint64_t)kPhiloxM0 * c0;
        const uint64_t b = (uint64_t)kPhiloxM1 * c2;
        const uint32_t n0 = (uint32_t)(b >> 32) ^ (c1 ^ k0);
        const uint32_t n2 = c3 ^ ((uint32_t)(a >> 32) ^ k1);
        c1 = (uint32_t)b; c3 = (uint32_t)a; c0 = n0; c2 = n2;
        k0 += kPhiloxW0; k1 += kPhiloxW1;
    }
    {   // round 3: c3 is uniform
        const uint64_t a = (uint64_t)kPhiloxM0 * c0;
        const uint64_t b = (uint64_t)kPhiloxM1 * c2;
        const uint32_t n0 = xor3((uint32_t)(b >> 32), c1, k0);
        const uint32_t n2 = (uint32_t)(a >> 32) ^ (c3 ^ k1);
        c1 = (uint32_t)b; c3 = (uint32_t)a; c0 = n0; c2 = n2;
        k0 += kPhiloxW0; k1 += kPhiloxW1;
    }
#pragma unroll
    for (int r = 3; r < 10; ++r) {
        const uint64_t a = (uint64_t)kPhiloxM0 * c0;
        const uint64_t b = (uint64_t)kPhiloxM1 * c2;
        const uint32_t n0 = xor3((uint32_t)(b >> 32), c1, k0);
        const uint32_t n2 = xor3((uint32_t)(a >> 32), c3, k1);
        c1 = (uint32_t)b; c3 = (uint32_t)a; c0 = n0; c2 = n2;
        k0 += kPhiloxW0; k1 += kPhiloxW1;
    }
    w[0] = c0; w[1] = c1; w[2] = c2; w[3] = c3;
}

// ---------------------------------------------------------------------------------------------
// Element access.  A "quad" is four consecutive elements: 16 bytes of fp32 or 8 bytes of bf16.
// Elements are handled as fp32 bit patterns (bf16 widens exactly by a 16-bit shift, fp16 by the
// exact hardware conversion).
// ---------------------------------------------------------------------------------------------
// Streaming accesses: every byte is touched once per pass, so loads and stores carry the
// non-temporal hint (measured on MI355X: +10..15 % bandwidth for the read-16-write-4 pattern at
// four to eight workgroups per CU).
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint4 load_stream16(const void *p)
{
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

// fp16 <-> fp32 patterns with the hardware conversions (v_cvt_f32_f16 is exact, subnormals
// included; v_cvt_f16_f32 rounds to nearest even, overflows to infinity).
__device__ __forceinline__ uint32_t f16_to_f32_bits(uint32_t h)
{
    return __float_as_uint((float)__builtin_bit_cast(_Float16, (unsigned short)h));
}

__device__ __forceinline__ uint32_t f32_bits_to_f16(uint32_t b)
{
    return (uint32_t)__builtin_bit_cast(unsigned short, (_Float16)__uint_as_float(b));
}

// The two 16-bit elements of a dword as fp32 patterns (low half first).
template <int DTYPE>
__device__ __forceinline__ void widen_pair(uint32_t w, uint32_t &lo, uint32_t &hi)
{
    if (DTYPE == LGN_BF16) {
        lo = w << 16;
        hi = w & 0xffff0000u;
    } else {
        lo = f16_to_f32_bits(w & 0xffffu);
        hi = f16_to_f32_bits(w >> 16);
    }
}

template <int DTYPE>
__device__ __forceinline__ void load_quad(const void *g, uint64_t quad, uint32_t b[4])
{
    if (DTYPE == LGN_F32) {
        const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(g) + quad);
        b[0] = v.x; b[1] = v.y; b[2] = v.z; b[3] = v.w;
    } else {
        const u32x2_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x2_t *>(g) + quad);
        widen_pair<DTYPE>(v.x, b[0], b[1]);
        widen_pair<DTYPE>(v.y, b[2], b[3]);
    }
}

template <int DTYPE>
__device__ __forceinline__ uint32_t load_elem(const void *g, uint64_t i)
{
    if (DTYPE == LGN_F32) return reinterpret_cast<const uint32_t *>(g)[i];
    const uint32_t h = reinterpret_cast<const uint16_t *>(g)[i];
    return DTYPE == LGN_BF16 ? h << 16 : f16_to_f32_bits(h);
}

// fp32 pattern -> bf16 pattern in the upper half, round to nearest even.  Everything the kernels
// store is exactly representable in bf16 (a no-op then) except a saturated value whose scale puts
// it below the bf16 subnormal range.
__device__ __forceinline__ uint32_t bf16_round_hi(uint32_t b)
{
    return (b + 0x7fffu + ((b >> 16) & 1u)) & 0xffff0000u;
}

template <int DTYPE>
__device__ __forceinline__ void store_quad(void *out, uint64_t quad, const uint32_t b[4])
{
    if (DTYPE == LGN_F32) {
        u32x4_t v = {b[0], b[1], b[2], b[3]};
        __builtin_nontemporal_store(v, reinterpret_cast<u32x4_t *>(out) + quad);
    } else if (DTYPE == LGN_BF16) {
        u32x2_t v = {(bf16_round_hi(b[0]) >> 16) | bf16_round_hi(b[1]),
                     (bf16_round_hi(b[2]) >> 16) | bf16_round_hi(b[3])};
        __builtin_nontemporal_store(v, reinterpret_cast<u32x2_t *>(out) + quad);
    } else {
        u32x2_t v = {f32_bits_to_f16(b[0]) | (f32_bits_to_f16(b[1]) << 16),
                     f32_bits_to_f16(b[2]) | (f32_bits_to_f16(b[3]) << 16)};
        __builtin_nontemporal_store(v, reinterpret_cast<u32x2_t *>(out) + quad);
    }
}

template <int DTYPE>
__device__ __forceinline__ void store_elem(void *out, uint64_t i, uint32_t b)
{
    if (DTYPE == LGN_F32) reinterpret_cast<uint32_t *>(out)[i] = b;
    else if (DTYPE == LGN_BF16) reinterpret_cast<uint16_t *>(out)[i] = (uint16_t)(bf16_round_hi(b) >> 16);
    else reinterpret_cast<uint16_t *>(out)[i] = (uint16_t)f32_bits_to_f16(b);
}

}  // namespace lgn

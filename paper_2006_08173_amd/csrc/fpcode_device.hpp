// FP(1,e,m) code <-> value on fp32 bit patterns (Section 4.1 with the N-bit encoding described in
// include/lgn.h), shared by the streaming kernels, the dequantizer and the prefix coder.
#pragma once

#include "lgn_device.hpp"

namespace lgn {

// wave-uniform quantizer constants
struct QuantConst {
    int n_bits, e, m, s;
    int cbias;        // biased fp32 exponent that maps to exponent field 0
    int cmax;         // largest exponent field, 2^e - 1
    uint32_t maxmag;  // largest magnitude code, 2^(e+m) - 1
};

// Reads the format from device memory.  The fields are clamped to their legal ranges so that a
// struct that was never filled in cannot cause out-of-range shifts; sizing a PACKED output for
// the n_bits in the struct stays the caller's contract.
__device__ __forceinline__ void load_quant_const(const lgn_fp_params_t *f, QuantConst &q)
{
    q.n_bits = min(max(f->n_bits, 2), 8);
    q.e = min(max(f->e_bits, 1), q.n_bits - 1);
    q.m = q.n_bits - 1 - q.e;
    q.s = min(max(f->scale_exp, -400), 400);
    q.cbias = 127 + q.s - (1 << (q.e - 1));
    q.cmax = (1 << q.e) - 1;
    q.maxmag = (1u << (q.e + q.m)) - 1u;
}

// Magnitude-and-sign code of one element (Section 4.1 with the N-bit encoding of the header).
template <int ROUND>
__device__ __forceinline__ uint32_t quant_code(uint32_t bits, uint32_t w, const QuantConst &q)
{
    const uint32_t a = bits & 0x7fffffffu;
    uint32_t frac = a & 0x7fffffu;
    int be = (int)(a >> 23);
    if (be == 0 && frac != 0u) {  // subnormal input: normalise with integer ops
        const int sh = __clz(frac) - 8;
        frac = (frac << sh) & 0x7fffffu;
        be = 1 - sh;
    }
    const int c = be - q.cbias;
    const int cut = 23 - q.m;
    const uint32_t y = ((uint32_t)c << 23) | frac;  // meaningful only when 1 <= c <= cmax
    uint32_t mag = y >> cut;
    const uint32_t rem = y & ((1u << cut) - 1u);
    bool up;
    if (ROUND == LGN_ROUND_STOCHASTIC) {
        // cut-off fraction + (r + 1/2) / 2^16 >= 1, r the lower half of the element's word
        up = rem + ((w & 0xffffu) << (cut - 16)) + (1u << (cut - 17)) >= (1u << cut);
    } else {
        const uint32_t half = 1u << (cut - 1);
        up = rem > half || (rem == half && (mag & 1u));
    }
    mag += up ? 1u : 0u;
    mag = min(mag, q.maxmag);                        // carry out of the top binade saturates
    if (a == 0u) return 0u;
    if (c > q.cmax || a >= 0x7f800000u) mag = q.maxmag;  // above the range, Inf, NaN
    else if (c < 1) return 0u;                           // flush, decided before rounding
    return ((bits >> 31) << (q.e + q.m)) | mag;
}

// fp32 bit pattern of 2^s * (value of code); NaN inputs are passed through by the caller.
__device__ __forceinline__ uint32_t code_value_bits(uint32_t code, const QuantConst &q)
{
    const uint32_t mag = code & q.maxmag;
    const uint32_t c = mag >> q.m;
    if (c == 0u) return 0u;
    const uint32_t k = mag & ((1u << q.m) - 1u);
    const uint32_t sign = (code >> (q.e + q.m)) << 31;
    const int ef = (int)c + q.cbias;  // biased fp32 exponent of the result
    const uint32_t mant = k << (23 - q.m);
    if (ef >= 255) return sign | 0x7f800000u;
    if (ef >= 1) return sign | ((uint32_t)ef << 23) | mant;
    // The result is subnormal in fp32 and may need more bits than fp32 has there: rounded to
    // nearest, ties to even, as a conversion of the exact value would (a carry gives 2^-126).
    const int sh = 1 - ef;
    if (sh > 24) return sign;  // below half of the smallest subnormal
    const uint32_t x = 0x800000u | mant;
    const uint32_t r = x >> sh, rem = x & ((1u << sh) - 1u), half = 1u << (sh - 1);
    return sign | (r + ((rem > half || (rem == half && (r & 1u) != 0u)) ? 1u : 0u));
}

}  // namespace lgn

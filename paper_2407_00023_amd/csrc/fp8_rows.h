// The fp8 form of the KV pool (dtype PA_BF16_KV8): device-side encode and decode of one row.
//
// A row = the D elements of one (token, KV head, K or V).  It is kept as D one-byte codes of the 8-bit floating-point
// format with 4 exponent bits (bias 7), 3 mantissa bits, no infinities and largest value 448, plus one exponent k per
// row: stored value = decode(code) * 2^k.  k is the smallest integer with max|row| * 2^-k <= 448 (0 for a row of
// zeros, kept within [-100, 119]); code = x * 2^-k rounded to nearest, ties to the even mantissa, anything still above
// 448 stored as 448.  Every stored value is exactly a finite bfloat16.  Inputs are finite bfloat16 values.
//
// Layout in the pool: the codes first, arranged like the elements of the bfloat16 pool (pool_row with one byte per
// element), then, from byte num_slots * 2 * Hkv * D on, the exponents as int8 in the same order of rows
// ([page][K | V][kv head][token in page]).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace pa {

constexpr int kFp8ExpMin = -100, kFp8ExpMax = 119;

// The row exponent from the largest magnitude of the row, given as bfloat16 bits without the sign.
__host__ __device__ inline int fp8_row_exponent(unsigned amax_bits) {
    if (amax_bits == 0) return 0;
    // amax = (1 + m / 128) * 2^(E - 127); 448 = 1.75 * 2^8
    const int E = static_cast<int>(amax_bits >> 7), m = static_cast<int>(amax_bits & 127);
    const int k = E - 135 + (m > 96 ? 1 : 0);
    return k < kFp8ExpMin ? kFp8ExpMin : k > kFp8ExpMax ? kFp8ExpMax : k;
}

// One bfloat16 (bits) times 2^-k as a code; integer arithmetic only, so that rounding is the same everywhere.
__host__ __device__ inline unsigned fp8_encode(unsigned bits, int k) {
    const unsigned sign = (bits >> 8) & 0x80u;
    const int E = static_cast<int>((bits >> 7) & 0xFF), m = static_cast<int>(bits & 127);
    if (E == 0) return sign;  // zero, or a subnormal bfloat16: far below half the smallest code for every k allowed
    const int Es = E - k;     // biased exponent of the scaled value (1 + m / 128) * 2^(Es - 127)
    int code;
    if (Es >= 121) {
        // a normal code: exponent field Es - 120, mantissa m rounded from 7 to 3 bits; a carry out of the mantissa
        // moves into the exponent field by itself
        const int t = ((Es - 120) << 7) | m;
        code = (t + 7 + ((t >> 4) & 1)) >> 4;
        if (code > 126) code = 126;
    } else {
        // below 2^-6: a multiple of 2^-9, q = (128 + m) * 2^(Es - 125) rounded to an integer (8 = the smallest normal code)
        const int sh = 125 - Es;
        const int M = 128 + m;
        code = sh > 9 ? 0 : (M + (1 << (sh - 1)) - 1 + ((M >> sh) & 1)) >> sh;
    }
    return sign | static_cast<unsigned>(code);
}

// 2^k as a float, k in [kFp8ExpMin, kFp8ExpMax].
__device__ __forceinline__ float fp8_scale(int k) { return __int_as_float((k + 127) << 23); }

// Four codes (one 32-bit word, first code in the low byte) times `scale` (a power of two) -> four bfloat16, in order.
// The conversion instruction multiplies the decoded pair by the scale and rounds to bfloat16; here the product is
// exactly representable, so nothing is rounded.
__device__ __forceinline__ uint2 fp8_decode4(unsigned word, float scale) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    const bf16x2_t lo = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(word, scale, false);
    const bf16x2_t hi = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(word, scale, true);
    return make_uint2(__builtin_bit_cast(unsigned, lo), __builtin_bit_cast(unsigned, hi));
}

}  // namespace pa

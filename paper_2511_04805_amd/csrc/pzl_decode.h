// Algorithm 1 as every kernel of the library runs it: on 32-bit words, two packed elements at a
// time, without a branch.  The streaming GEMM, the tiled GEMM and pzl_unpack all include this one
// routine, so the exhaustive 65536-word x 2-position comparison of pzl_unpack with the CPU
// definition covers the decode that runs inside the matmuls.
//
// Packed half-word (Sec. 3.3.2; bit positions as Algorithm 1 reads them):
//   15: S0   14: S1   13: M0   12: M1   11..7: exponent - 112   6..0: mantissa
#pragma once
#include <stdint.h>

namespace pzl {

typedef short dec_s16x2 __attribute__((ext_vector_type(2)));

// Exponent and mantissa of both halves as bf16 fields: the stored five bits plus 112, shifted to
// bf16's exponent position (112 << 7 = 0x3800).  No carry can cross the halves:
// 0x0FFF + 0x3800 < 0x8000.
__device__ __forceinline__ uint32_t decode_body(uint32_t x) { return (x & 0x0FFF0FFFu) + 0x38003800u; }

// The same two elements as IEEE half precision, each multiplied by 2.  The stored exponent field
// e (value 2^(e-15) (1 + m/128)) is half precision's own biased exponent, and the 7 mantissa bits
// are the top of its 10; moved up by three bits the 12 stored bits are the half-precision number
// itself, except that half precision reads field 0 as subnormal and field 31 as infinity.  One
// more in the exponent (x 2, exact) makes field 0 a normal number; fields 30 and 31 then do not
// fit, so only tensors whose largest used field is at most 29 (|w| < 2^15) may be decoded this way.
__device__ __forceinline__ uint32_t decode_body_half_x2(uint32_t x) { return ((x & 0x0FFF0FFFu) << 3) + 0x04000400u; }

// Sign and mask of position POS applied to `body` (either of the above): the mask bit (13 - POS)
// of each half is moved to the half's top bit and smeared over the half by a packed arithmetic
// shift (a masked-out element is +0, as Algorithm 1 assigns 0 before looking at the sign); the
// sign bit (15 - POS) is moved to bit 15.
template <int POS>
__device__ __forceinline__ uint32_t decode_pair(uint32_t x, uint32_t body)
{
    const uint32_t xs = POS ? (x << 1) : x;
    dec_s16x2 t = __builtin_bit_cast(dec_s16x2, x << (2 + POS));
    t = t >> 15;
    const uint32_t m = __builtin_bit_cast(uint32_t, t);
    return ((xs & 0x80008000u) | body) & m;
}

typedef unsigned short dec_u16x2 __attribute__((ext_vector_type(2)));

// Two plain bf16 weights (a dense expert) as IEEE half precision times 2^(112 - B), B = `bias`:
// the tensor's largest exponent field minus 30 (at least 0), so that its largest weights land on
// half precision's largest exponent and everything down to 2^-30 of them stays a normal number.
// Per half: exponent field clamped from below to B (smaller weights, and zeros, become zero or a
// subnormal of no weight in a sum), the 15 bits moved up by three (the exponent's top bits fall
// off the half), B subtracted from what is now the exponent's place modulo 64 -- exact, since the
// true difference is within 0..30 -- and the sign put back.  clamp2 = B << 7 and bias2 =
// (B << 10) mod 2^16, each in both halves.  Tensors with an infinity or a NaN are not decoded
// this way.
__device__ __forceinline__ uint32_t dense_pair_to_half_scaled(uint32_t x, uint32_t clamp2, uint32_t bias2)
{
    dec_u16x2 t = __builtin_bit_cast(dec_u16x2, x & 0x7FFF7FFFu);
    t = __builtin_elementwise_max(t, __builtin_bit_cast(dec_u16x2, clamp2));
    t = (t << 3) - __builtin_bit_cast(dec_u16x2, bias2);
    return (x & 0x80008000u) | (__builtin_bit_cast(uint32_t, t) & 0x7FFF7FFFu);
}

}  // namespace pzl

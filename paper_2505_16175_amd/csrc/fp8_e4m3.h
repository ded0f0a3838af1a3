// 8-bit E4M3 (OCP 8-bit floating point: 1 sign bit, 4 exponent bits with bias 7, 3 mantissa bits, no infinities,
// largest value 448, subnormals down to 2^-9) for the pruned cache's 8-bit format: conversions from and to bf16 bit
// patterns in integer arithmetic, the same code on the host and on the device.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace qp {

// One bf16 value (its 16 bits) to the 8-bit E4M3 code: nearest, ties to even, magnitudes beyond 448 saturate, NaN
// gives the NaN code. Exact integer arithmetic on the bf16 fields (1 sign, 8 exponent bits with bias 127, 7 mantissa
// bits) into E4M3's (1, 4 with bias 7, 3): normal results for unbiased exponents -6 .. 8, below that multiples of 2^-9.
__host__ __device__ inline uint32_t bf16_to_e4m3(uint32_t h) {
  const uint32_t sign = (h >> 8) & 0x80u;
  const uint32_t a = h & 0x7fffu;
  if (a > 0x7f80u) return sign | 0x7fu;                 // NaN
  const int e = (int)(a >> 7) - 127;                     // unbiased exponent (bf16 subnormals: far below 2^-10 -> 0)
  const uint32_t m = a & 0x7fu;
  uint32_t code;
  if (e >= -6) {
    // 7 mantissa bits -> 3: keep the top 3, round on the lower 4
    uint32_t q = ((uint32_t)(e + 7) << 3) | (m >> 4);    // exponent and mantissa as one integer: a carry moves up
    const uint32_t rem = m & 0xfu;
    q += (rem > 8u || (rem == 8u && (q & 1u))) ? 1u : 0u;
    code = q > 0x7eu ? 0x7eu : q;                        // 0x7e = 448; beyond it (or infinity) saturates
  } else if (e >= -10 && (a >> 7) != 0) {
    // subnormal result: value = (128 + m) * 2^(e - 7), in units of 2^-9: (128 + m) >> sh with sh = -e - 2 in 5 .. 8
    const uint32_t sig = 128u + m;
    const int sh = -e - 2;
    const uint32_t q = sig >> sh, rem = sig & ((1u << sh) - 1u), half = 1u << (sh - 1);
    code = q + ((rem > half || (rem == half && (q & 1u))) ? 1u : 0u);  // 8 = the smallest normal: the carry is right
  } else {
    code = 0;                                            // below half of 2^-9 (2^-10 itself is a tie: to even, 0)
  }
  return sign | code;
}

// The E4M3 code's value as a bf16 bit pattern (exact: 3 mantissa bits and the exponent range fit).
__host__ __device__ inline uint32_t e4m3_to_bf16(uint32_t c) {
  const uint32_t sign = (c & 0x80u) << 8;
  const uint32_t e = (c >> 3) & 0xfu, m = c & 7u;
  if (e == 0xfu && m == 7u) return sign | 0x7fc0u;                    // NaN
  if (e != 0) return sign | ((e + 120u) << 7) | (m << 4);             // (1 + m/8) 2^(e-7): bf16 exponent e - 7 + 127
  if (m == 0) return sign;
  const uint32_t top = m >= 4u ? 2u : (m >= 2u ? 1u : 0u);            // m 2^-9 = (1 + frac) 2^(top - 9)
  return sign | ((118u + top) << 7) | (((m << (7 - top)) & 0x7fu));
}

}  // namespace qp

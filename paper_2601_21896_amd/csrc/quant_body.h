// E4M3 quantisation of bf16 values (8-bit storage of the K/V cache; beyond the paper, which states no storage
// precision: App. A), shared by the quantisation kernel and by the compaction kernel that quantises the chunk's rows
// behind the retained ones.  E4M3 = 1 sign, 4 exponent bits with bias 7, 3 mantissa bits, no infinities,
// S.1111.111 = NaN; round to nearest even; magnitudes beyond 448 saturate.  Integer arithmetic, so that every code is
// a defined function of the input bits.
#pragma once
#include "pafu_internal.h"

namespace pafu {
namespace {

// x * inv_scale (exact: inv_scale is a power of two) -> E4M3 code
__device__ __forceinline__ unsigned e4m3_code(float x, float inv_scale) {
  const float v = x * inv_scale;
  const unsigned u = __float_as_uint(v);
  const unsigned sign = (u >> 24) & 0x80u;
  const unsigned au = u & 0x7fffffffu;
  if (au > 0x7f800000u) return sign | 0x7fu;  // NaN
  const float a = fminf(__uint_as_float(au), 448.0f);
  unsigned code;
  if (a < 0.015625f) {  // below the smallest normal 2^-6: the grid is k * 2^-9, k = 0..8 (8 = the smallest normal)
    code = (unsigned)__builtin_rintf(a * 512.0f);
  } else {
    unsigned b = __float_as_uint(a);
    b += 0x7ffffu + ((b >> 20) & 1u);        // nearest even at 3 mantissa bits (a carry moves into the exponent)
    code = ((b >> 20) & 0x7ffu) - (120u << 3);  // exponent bias 127 -> 7
  }
  return sign | code;
}

__device__ __forceinline__ float bf16_lo(unsigned w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(unsigned w) { return __uint_as_float(w & 0xffff0000u); }

// 8 bf16 values (four 32-bit words) -> 8 codes (two words)
__device__ __forceinline__ void e4m3_codes8(const unsigned (&w)[4], float inv, unsigned (&o)[2]) {
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    o[e] = e4m3_code(bf16_lo(w[2 * e]), inv) | (e4m3_code(bf16_hi(w[2 * e]), inv) << 8) |
           (e4m3_code(bf16_lo(w[2 * e + 1]), inv) << 16) | (e4m3_code(bf16_hi(w[2 * e + 1]), inv) << 24);
  }
}

}  // namespace
}  // namespace pafu

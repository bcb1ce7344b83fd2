// The tensor's 16-bit format, fixed per translation unit: every kernel source is compiled once for
// bf16 and once (ADACC_F16=1) for IEEE binary16, the format the paper compresses (Section 3.2, "from
// FP16 to INT4"); the two sets of kernels live in the namespaces adacc::bf16 and adacc::f16.
//
// Both formats have the sign in bit 15 and a magnitude in the 15 low bits that grows with |x| when
// read as an integer, with Inf and NaN on top; they differ in how a pattern widens to binary32
// (exactly, in both), where "not finite" begins, and in the rounding back from binary32.
#pragma once

#include "adacc_common.hpp"

#ifndef ADACC_F16
#define ADACC_F16 0
#endif
#if ADACC_F16
#define ADACC_DT_NS f16
#else
#define ADACC_DT_NS bf16
#endif

namespace adacc {
namespace ADACC_DT_NS {

typedef float f32x2_t __attribute__((ext_vector_type(2)));

#if ADACC_F16
constexpr uint32_t kNonfiniteMag = 0x7C00u;  // binary16: 5 exponent bits, 10 fraction bits
__device__ __forceinline__ float widen_lo(uint32_t w) { return (float)__builtin_bit_cast(_Float16, (uint16_t)w); }
__device__ __forceinline__ float widen_hi(uint32_t w) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16)); }
// binary32 bits of the magnitude `mag` (15 bits)
__device__ __forceinline__ uint32_t mag_bits32(uint32_t mag) { return __float_as_uint(widen_lo(mag)); }
// two binary32 values -> two 16-bit values in one word (first value in the low half), round to
// nearest even, too large becomes infinite
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t narrow_pair(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2_t));
}
#else
constexpr uint32_t kNonfiniteMag = 0x7F80u;  // bf16: the upper half of a binary32 word
__device__ __forceinline__ float widen_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float widen_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }
__device__ __forceinline__ uint32_t mag_bits32(uint32_t mag) { return mag << 16; }
// the conversion instruction of gfx950
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t narrow_pair(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
#endif

}  // namespace ADACC_DT_NS
}  // namespace adacc

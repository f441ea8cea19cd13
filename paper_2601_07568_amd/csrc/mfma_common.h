// Shared by the matrix-core (MFMA) kernel files: vector types, the 16x16x32 product, bfloat16 packing,
// workspace access.
//
// v_mfma_f32_16x16x32_bf16 operand layout (lane l, c = l % 16, g = l / 16): A holds row c of a
// 16x32 tile, B holds column c of a 32x16 tile, each its 8 consecutive k-elements of group g;
// D holds column c, rows 4g..4g+3.  The k-order is immaterial as long as A and B agree, which is
// used throughout to give each lane contiguous bytes.
#pragma once
#include "common.h"
#include <math.h>
#include <string.h>
#include <stdlib.h>

namespace dllm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ inline f32x4 mfma16(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                 0, 0);
}

// two floats -> packed bfloat16 pair (round to nearest even, in hardware)
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t));
}

// Maximum over the four 16-lane rows of a wave, returned in every lane, without a trip through LDS: the
// row swap exchanges rows 1 and 3 of its first operand with rows 0 and 2 of its second, the half swap the
// upper half of the first with the lower half of the second, so the two results of a swap of x with
// itself hold, lane by lane, x of both rows (halves) of a pair.
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float rows_max(float x) {
  const uint32_t xi = __float_as_uint(x);
  const u32x2_t a = __builtin_amdgcn_permlane16_swap(xi, xi, false, false);
  const float m = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
  const uint32_t mi = __float_as_uint(m);
  const u32x2_t b = __builtin_amdgcn_permlane32_swap(mi, mi, false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}

#define WSM(c, field, type) ((type*)((c)->ws + (c)->map.field))

}  // namespace dllm

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

#define WSM(c, field, type) ((type*)((c)->ws + (c)->map.field))

}  // namespace dllm

// The two 16-bit float storage types of the MFMA path: bf16 (8 exponent bits) and fp16 (the
// precision the paper runs in, App. C).  Kernels take `bool F16` as their last template argument
// and get the element type, its 8-wide operand vector and the 32x32x16 matrix instruction here.
// Device code only (included by .hip files).
#pragma once
#include <type_traits>

#include "goose_internal.h"

typedef _Float16 f16_t;

template <bool F16>
struct Mma16;

template <>
struct Mma16<false> {
  typedef bf16_t T;
  typedef __bf16 v8 __attribute__((ext_vector_type(8)));
  typedef __bf16 v4 __attribute__((ext_vector_type(4)));
  typedef float acc16 __attribute__((ext_vector_type(16)));
  static __device__ inline acc16 mfma(v8 a, v8 b, acc16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  }
};

template <>
struct Mma16<true> {
  typedef f16_t T;
  typedef _Float16 v8 __attribute__((ext_vector_type(8)));
  typedef _Float16 v4 __attribute__((ext_vector_type(4)));
  typedef float acc16 __attribute__((ext_vector_type(16)));
  static __device__ inline acc16 mfma(v8 a, v8 b, acc16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
  }
};

// Storage types and MFMA operand vectors for gfx950 device code.
#pragma once
#include <hip/hip_runtime.h>

namespace flexco {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ inline float ld(const float* p) { return *p; }
__device__ inline float ld(const bf16_t* p) { return (float)*p; }
__device__ inline void st(float* p, float v) { *p = v; }
__device__ inline void st(bf16_t* p, float v) { *p = (bf16_t)v; }   // round to nearest even


// 16-byte row accesses of the element-wise kernels: N consecutive elements as floats
template <typename T> struct Vec;
template <> struct Vec<float> {
  static constexpr int N = 4;
  __device__ static void load(const float* p, float* v) {
    const f32x4 t = *reinterpret_cast<const f32x4*>(p);
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = t[i];
  }
  __device__ static void store(float* p, const float* v) {
    f32x4 t;
#pragma unroll
    for (int i = 0; i < 4; ++i) t[i] = v[i];
    *reinterpret_cast<f32x4*>(p) = t;
  }
};
template <> struct Vec<bf16_t> {
  static constexpr int N = 8;
  __device__ static void load(const bf16_t* p, float* v) {
    const bf16x8 t = *reinterpret_cast<const bf16x8*>(p);
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = (float)t[i];
  }
  __device__ static void store(bf16_t* p, const float* v) {
    bf16x8 t;
#pragma unroll
    for (int i = 0; i < 8; ++i) t[i] = (bf16_t)v[i];   // round to nearest even
    *reinterpret_cast<bf16x8*>(p) = t;
  }
};

}  // namespace flexco

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

}  // namespace flexco

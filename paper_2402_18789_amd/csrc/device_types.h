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

// Exchanges between the four rows of 16 lanes of a wavefront without the LDS crossbar: gfx950's row swaps.
// v_permlane16_swap a, b swaps the odd rows of a with the even rows of b; v_permlane32_swap the upper half of a
// with the lower half of b.  With a = b = v on entry, a then holds the value of the even row of each pair of rows
// (of the lower half) in both rows (halves) and b that of the odd row (upper half): a op b is v op (the value of
// lane ^ 16, lane ^ 32) in every lane, the same bits in both partners.  (One wait state around the swap for the
// vector ALU's read-after-write rules, which the compiler does not track through the asm.)
__device__ inline void row_pair_swap(float& a, float& b) {
  asm("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}
__device__ inline void half_swap(float& a, float& b) {
  asm("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}
__device__ inline float sum_xor16(float v) { float a = v, b = v; row_pair_swap(a, b); return a + b; }
__device__ inline float sum_xor32(float v) { float a = v, b = v; half_swap(a, b); return a + b; }
__device__ inline float max_xor16(float v) { float a = v, b = v; row_pair_swap(a, b); return fmaxf(a, b); }
__device__ inline float max_xor32(float v) { float a = v, b = v; half_swap(a, b); return fmaxf(a, b); }

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

// ReLU with a sign bitmask as its only saved state (Sec. 5.2 of the paper: the backward of a ReLU reads nothing
// of its output but the sign, so a ReLU whose output no other backward operator needs keeps 1 bit per element
// instead of the tensor).  mask: [n, ceil(width / 32)] 32-bit words, bit j of word w of a row = element 32 w + j
// of that row is positive; the unused high bits of a row's last word are zero.
#include "flexco_internal.h"
#include "device_types.h"

namespace flexco {

namespace {

// A lane owns N consecutive elements (16 bytes); 32 / N neighbouring lanes own one mask word and OR their
// pieces together with shuffles.  FWD: y = max(x, 0), mask written.  !FWD: dx = dy where the bit is set, else 0.
template <typename T, bool FWD>
__global__ __launch_bounds__(256) void relu_bitmask_kernel(const T* __restrict__ in, T* __restrict__ out,
                                                           uint32_t* __restrict__ mask, int width, int words,
                                                           size_t ld_in, size_t ld_out) {
  constexpr int N = Vec<T>::N, G = 32 / N;
  const int row = blockIdx.y;
  const int lane = threadIdx.x & 63;
  const int col = (blockIdx.x * 256 + threadIdx.x) * N;
  const bool valid = col < width;                           // width % N == 0: a lane is inside or outside as a whole
  float v[N];
#pragma unroll
  for (int i = 0; i < N; ++i) v[i] = 0.f;
  if (valid) Vec<T>::load(in + (size_t)row * ld_in + col, v);
  uint32_t* wp = mask + (size_t)row * words + (col >> 5);
  if (FWD) {
    uint32_t bits = 0;
#pragma unroll
    for (int i = 0; i < N; ++i) {
      bits |= (v[i] > 0.f ? 1u : 0u) << i;
      v[i] = fmaxf(v[i], 0.f);
    }
    uint32_t w = bits << ((lane % G) * N);
#pragma unroll
    for (int o = 1; o < G; o <<= 1) w |= __shfl_xor(w, o, 64);
    if (valid) {
      Vec<T>::store(out + (size_t)row * ld_out + col, v);
      if (lane % G == 0) *wp = w;
    }
  } else {
    if (!valid) return;
    const uint32_t bits = *wp >> ((lane % G) * N);
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] = (bits >> i & 1u) ? v[i] : 0.f;
    Vec<T>::store(out + (size_t)row * ld_out + col, v);
  }
}

// any width and alignment: one thread per mask word
template <typename T, bool FWD>
__global__ __launch_bounds__(256) void relu_bitmask_scalar_kernel(const T* __restrict__ in, T* __restrict__ out,
                                                                  uint32_t* __restrict__ mask, int width, int words,
                                                                  size_t ld_in, size_t ld_out) {
  const int row = blockIdx.y;
  const int w = blockIdx.x * 256 + threadIdx.x;
  if (w >= words) return;
  uint32_t bits = FWD ? 0u : mask[(size_t)row * words + w];
  for (int j = 0; j < 32; ++j) {
    const int col = w * 32 + j;
    if (col >= width) break;
    const float x = (float)in[(size_t)row * ld_in + col];
    if (FWD) {
      bits |= (x > 0.f ? 1u : 0u) << j;
      out[(size_t)row * ld_out + col] = (T)fmaxf(x, 0.f);
    } else {
      out[(size_t)row * ld_out + col] = (T)((bits >> j & 1u) ? x : 0.f);
    }
  }
  if (FWD) mask[(size_t)row * words + w] = bits;
}

template <bool FWD>
int32_t launch(const void* in, void* out, uint32_t* mask, int n, int width, int dtype, hipStream_t s) {
  if (n == 0 || width == 0) return FLEXCO_OK;
  const int words = (width + 31) / 32;
  const int vn = dtype == FLEXCO_BF16 ? 8 : 4;
  const bool vec = width % vn == 0 && aligned16(in) && aligned16(out);
  if (dtype == FLEXCO_BF16) {
    if (vec)
      hipLaunchKernelGGL((relu_bitmask_kernel<bf16_t, FWD>), dim3((width / 8 + 255) / 256, n), dim3(256), 0, s,
                         (const bf16_t*)in, (bf16_t*)out, mask, width, words, (size_t)width, (size_t)width);
    else
      hipLaunchKernelGGL((relu_bitmask_scalar_kernel<bf16_t, FWD>), dim3((words + 255) / 256, n), dim3(256), 0, s,
                         (const bf16_t*)in, (bf16_t*)out, mask, width, words, (size_t)width, (size_t)width);
  } else {
    if (vec)
      hipLaunchKernelGGL((relu_bitmask_kernel<float, FWD>), dim3((width / 4 + 255) / 256, n), dim3(256), 0, s,
                         (const float*)in, (float*)out, mask, width, words, (size_t)width, (size_t)width);
    else
      hipLaunchKernelGGL((relu_bitmask_scalar_kernel<float, FWD>), dim3((words + 255) / 256, n), dim3(256), 0, s,
                         (const float*)in, (float*)out, mask, width, words, (size_t)width, (size_t)width);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(FLEXCO_EHIP, "launch of relu_bitmask failed: %s", hipGetErrorString(e));
  return FLEXCO_OK;
}

int32_t check(const void* a, const void* b, const uint32_t* mask, int n, int width, int dtype) {
  FLEXCO_CHECK(a && b && mask, FLEXCO_EINVAL, "NULL argument");
  FLEXCO_CHECK(n >= 0 && width >= 0, FLEXCO_EINVAL, "negative size");
  FLEXCO_CHECK((size_t)n <= 65535, FLEXCO_ESHAPE, "at most 65535 rows per call (got %d)", n);
  FLEXCO_CHECK(dtype == FLEXCO_F32 || dtype == FLEXCO_BF16, FLEXCO_ESHAPE, "unknown dtype %d", dtype);
  FLEXCO_CHECK(((uintptr_t)mask & 3u) == 0, FLEXCO_EINVAL, "mask is not 4-byte aligned");
  return FLEXCO_OK;
}

}  // namespace

}  // namespace flexco

using namespace flexco;

extern "C" int32_t flexco_relu_bitmask_fwd(const void* x, void* y, uint32_t* mask, int32_t n, int32_t width,
                                           int32_t dtype, void* stream) {
  clear_error();
  FLEXCO_TRY(check(x, y, mask, n, width, dtype));
  return launch<true>(x, y, mask, n, width, dtype, (hipStream_t)stream);
}

extern "C" int32_t flexco_relu_bitmask_bwd(const void* dy, const uint32_t* mask, void* dx, int32_t n, int32_t width,
                                           int32_t dtype, void* stream) {
  clear_error();
  FLEXCO_TRY(check(dy, dx, mask, n, width, dtype));
  return launch<false>(dy, dx, const_cast<uint32_t*>(mask), n, width, dtype, (hipStream_t)stream);
}

// Machine-ceiling probes for the benchmark: what this GPU delivers for the two resources the
// rooflines are quoted against, measured with the simplest possible kernels.  They compute
// nothing of the method; bench.py times them with events on the stream they are launched on.
#include "flexco_internal.h"
#include "device_types.h"

namespace flexco {

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// back-to-back v_mfma_f32_32x32x16_bf16 on register operands: 16 independent accumulators per
// wavefront (the register shape of the 256 x 256 GEMM tile), one wavefront per SIMD
__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, float* sink) {
  const int lane = threadIdx.x & 63;
  bf16x8 a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      // operand values spread over [-1, 1) like activations and weights, not zeros: the clock the
      // chip sustains depends on how many bits toggle
      const unsigned h = (unsigned)(lane * 8 + j + 64 * i) * 2654435761u;
      a[i][j] = (bf16_t)((float)(h >> 8 & 0xffff) / 32768.f - 1.f);
      b[i][j] = (bf16_t)((float)(h >> 4 & 0xffff) / 32768.f - 1.f);
    }
  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) s += acc[i][j][0];
  if (s == 12345.678f) sink[0] = s;   // keeps the loop; never true in practice
}

// The same products with their operands fetched from LDS the way the projection kernels fetch them: a block of
// 4 wavefronts (2 x 2) owns a (64 MT) x (64 NT) tile, LDS holds one 64-column stage of both operand tiles (128-byte
// rows, 16-byte chunks XOR-swizzled by row), and every 16-column slice costs a wavefront MT + NT ds_read_b128 for
// MT x NT products.  No global memory traffic and no barriers inside the loop: what the matrix cores sustain when
// LDS feeds them (MT = NT = 2: the 128 x 128 tile, LDS reads as long as the products; 4: the 256 x 256 tile, half).
template <int MT, int NT>
__global__ __launch_bounds__(256) void probe_mfma_lds_kernel(int iters, float* sink) {
  constexpr int BM = 64 * MT, BN = 64 * NT;
  __shared__ __attribute__((aligned(1024))) bf16_t tile[(BM + BN) * 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int i = tid; i < (BM + BN) * 64; i += 256) {
    const unsigned h = (unsigned)i * 2654435761u;
    tile[i] = (bf16_t)((float)(h >> 8 & 0xffff) / 32768.f - 1.f);
  }
  __syncthreads();
  const int wm0 = (wave >> 1) * 32 * MT, wn0 = (wave & 1) * 32 * NT;
  const int l32 = lane & 31, kg = lane >> 5;
  f32x16 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      bf16x8 af[MT], bf[NT];
#pragma unroll
      for (int i = 0; i < MT; ++i) {
        const int r = wm0 + i * 32 + l32;
        af[i] = *reinterpret_cast<const bf16x8*>(tile + r * 64 + (((kk * 2 + kg) ^ ((r >> 1) & 7)) * 8));
      }
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const int r = wn0 + j * 32 + l32;
        bf[j] = *reinterpret_cast<const bf16x8*>(tile + (BM + r) * 64 + (((kk * 2 + kg) ^ ((r >> 1) & 7)) * 8));
      }
#pragma unroll
      for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[j], af[i], acc[i][j], 0, 0, 0);
    }
    asm volatile("" ::: "memory");      // the fragments are read again in every iteration
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j) s += acc[i][j][0];
  if (s == 12345.678f) sink[0] = s;
}

// every block streams its own contiguous piece with 16-byte loads, 8 in flight per lane
__global__ __launch_bounds__(256) void probe_read_kernel(const u32x4* __restrict__ src, size_t vec_per_block,
                                                         unsigned* sink) {
  const u32x4* p = src + (size_t)blockIdx.x * vec_per_block;
  u32x4 acc = {0, 0, 0, 0};
  for (size_t i = threadIdx.x; i + 7 * 256 < vec_per_block; i += 8 * 256) {
    u32x4 v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = p[i + j * 256];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc ^= v[j];
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[0] = acc.x;   // keeps the loads
}

}  // namespace

}  // namespace flexco

using namespace flexco;

extern "C" int32_t flexco_probe_mfma(int32_t blocks, int32_t iters, void* sink, double* flops, void* stream) {
  clear_error();
  FLEXCO_CHECK(blocks > 0 && iters > 0 && sink && flops, FLEXCO_EINVAL, "probe_mfma: bad argument");
  hipLaunchKernelGGL(probe_mfma_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, iters, (float*)sink);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(FLEXCO_EHIP, "launch of probe_mfma failed: %s", hipGetErrorString(e));
  *flops = (double)blocks * 4.0 * iters * 16.0 * (2.0 * 32 * 32 * 16);
  return FLEXCO_OK;
}

extern "C" int32_t flexco_probe_mfma_lds(int32_t blocks, int32_t iters, int32_t tile, void* sink, double* flops,
                                         void* stream) {
  clear_error();
  FLEXCO_CHECK(blocks > 0 && iters > 0 && sink && flops, FLEXCO_EINVAL, "probe_mfma_lds: bad argument");
  FLEXCO_CHECK(tile == 128 || tile == 256, FLEXCO_EINVAL, "probe_mfma_lds: tile must be 128 or 256");
  if (tile == 128)
    hipLaunchKernelGGL((probe_mfma_lds_kernel<2, 2>), dim3(blocks), dim3(256), 0, (hipStream_t)stream, iters, (float*)sink);
  else
    hipLaunchKernelGGL((probe_mfma_lds_kernel<4, 4>), dim3(blocks), dim3(256), 0, (hipStream_t)stream, iters, (float*)sink);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(FLEXCO_EHIP, "launch of probe_mfma_lds failed: %s", hipGetErrorString(e));
  const double per_slice = (tile == 128 ? 4.0 : 16.0) * (2.0 * 32 * 32 * 16);
  *flops = (double)blocks * 4.0 * iters * 4.0 * per_slice;
  return FLEXCO_OK;
}

extern "C" int32_t flexco_probe_read(const void* src, size_t bytes, int32_t blocks, void* sink, double* bytes_read,
                                     void* stream) {
  clear_error();
  FLEXCO_CHECK(src && sink && bytes_read && blocks > 0, FLEXCO_EINVAL, "probe_read: bad argument");
  FLEXCO_CHECK(aligned16(src), FLEXCO_EINVAL, "probe_read: misaligned pointer");
  const size_t vec_per_block = bytes / 16 / (size_t)blocks / 2048 * 2048;   // whole rounds of 8 loads x 256 lanes
  FLEXCO_CHECK(vec_per_block > 0, FLEXCO_ESHAPE, "probe_read: %zu bytes are too few for %d blocks", bytes, blocks);
  hipLaunchKernelGGL(probe_read_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (const u32x4*)src, vec_per_block,
                     (unsigned*)sink);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(FLEXCO_EHIP, "launch of probe_read failed: %s", hipGetErrorString(e));
  *bytes_read = (double)vec_per_block * 16.0 * blocks;
  return FLEXCO_OK;
}

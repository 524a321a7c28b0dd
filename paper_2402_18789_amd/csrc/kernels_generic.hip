// Element-wise, normalisation, RoPE/cache-append, LoRA and type-generic fallback kernels.
//
// Everything here computes in fp32 whatever the storage type, one thread block per row or
// per small tile.  These kernels carry the fp32 configuration end to end and the parts of
// the bf16 configurations that are bound by HBM traffic or are tiny (norms, RoPE, SwiGLU,
// rank-r LoRA products).  The dense bf16 contractions live in gemm_mfma.hip /
// attn_mfma.hip.
#include <cmath>
#include <initializer_list>
#include <mutex>
#include <vector>
#include "flexco_internal.h"
#include "device_types.h"

namespace flexco {

// --------------------------------------------------------------------------------------
// reductions
// --------------------------------------------------------------------------------------
// Every lane gets the result.  Within a row of 16 lanes the partner's value comes through the data-parallel
// primitives, as an operand modifier of the addition itself (lane ^ 1, lane ^ 2, then the other quad of eight lanes
// and the other half of the row by mirrored reads - the quads, then the halves, are uniform by then); only the two
// exchanges between rows go through the LDS crossbar (a rank-16 row product ends with sixteen of these sums per
// wavefront: 4.1 of the norm backward's 17.6 us were the 96 crossbar exchanges of the all-crossbar form; row swaps
// for the last two steps as well, as the attention kernels use them in their softmax chain, were 3 - 5 % slower
// here, where sixteen independent sums overlap their crossbar round trips).
template <int CTRL>
__device__ inline float dpp_read(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false));
}
constexpr int DPP_XOR1 = 0xB1, DPP_XOR2 = 0x4E, DPP_HALF_MIRROR = 0x141, DPP_MIRROR = 0x140;
__device__ inline float wave_sum(float v) {
  v += dpp_read<DPP_XOR1>(v);
  v += dpp_read<DPP_XOR2>(v);
  v += dpp_read<DPP_HALF_MIRROR>(v);
  v += dpp_read<DPP_MIRROR>(v);
  v += __shfl_xor(v, 16, 64);
  v += __shfl_xor(v, 32, 64);
  return v;
}
__device__ inline float wave_max(float v) {
  v = fmaxf(v, dpp_read<DPP_XOR1>(v));
  v = fmaxf(v, dpp_read<DPP_XOR2>(v));
  v = fmaxf(v, dpp_read<DPP_HALF_MIRROR>(v));
  v = fmaxf(v, dpp_read<DPP_MIRROR>(v));
  v = fmaxf(v, __shfl_xor(v, 16, 64));
  v = fmaxf(v, __shfl_xor(v, 32, 64));
  return v;
}
// sum over a block of 256 threads; every thread gets the result
__device__ inline float block_sum256(float v, float* red /* >= 4 floats of LDS */) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

// ---- rank-r products of a row with LoRA B matrices, inside the row kernel that produced the row ------------
// acc[q] += v * B[col][q]: one 2 R-byte row of B per element
template <int R>
__device__ inline void lora_acc_row(float (&acc)[R], float v, const bf16_t* __restrict__ brow) {
#pragma unroll
  for (int q8 = 0; q8 < R / 8; ++q8) {
    const bf16x8 b = *reinterpret_cast<const bf16x8*>(brow + 8 * q8);
#pragma unroll
    for (int q = 0; q < 8; ++q) acc[8 * q8 + q] += v * (float)b[q];
  }
}
// the same for N consecutive columns: every load is issued before the first multiply-add
template <int R, int N>
__device__ inline void lora_acc_cols(float (&acc)[R], const float (&v)[N], const bf16_t* __restrict__ brow0) {
  bf16x8 b[N][R / 8];
#pragma unroll
  for (int j = 0; j < N; ++j)
#pragma unroll
    for (int q8 = 0; q8 < R / 8; ++q8) b[j][q8] = *reinterpret_cast<const bf16x8*>(brow0 + (size_t)j * R + 8 * q8);
#pragma unroll
  for (int j = 0; j < N; ++j)
#pragma unroll
    for (int q8 = 0; q8 < R / 8; ++q8)
#pragma unroll
      for (int q = 0; q < 8; ++q) acc[8 * q8 + q] += v[j] * (float)b[j][q8][q];
}
// the two halves of lora_acc_cols apart, for kernels that request the rows of B before they have the values
template <int R, int N>
__device__ inline void lora_load_cols(bf16x8 (&b)[N][R / 8], const bf16_t* __restrict__ brow0) {
#pragma unroll
  for (int j = 0; j < N; ++j)
#pragma unroll
    for (int q8 = 0; q8 < R / 8; ++q8) b[j][q8] = *reinterpret_cast<const bf16x8*>(brow0 + (size_t)j * R + 8 * q8);
}
template <int R, int N>
__device__ inline void lora_fma_cols(float (&acc)[R], const float (&v)[N], const bf16x8 (&b)[N][R / 8]) {
#pragma unroll
  for (int j = 0; j < N; ++j)
#pragma unroll
    for (int q8 = 0; q8 < R / 8; ++q8)
#pragma unroll
      for (int q = 0; q < 8; ++q) acc[8 * q8 + q] += v[j] * (float)b[j][q8][q];
}
// sum of acc over the block's 256 threads (the lanes of a wavefront, then the four wavefronts in order) -> t and ext of `row`
template <int R, int NW = 4>
__device__ inline void lora_row_finish(float (&acc)[R], float* lds /* NW R floats */, float* t, bf16_t* ext, size_t row,
                                       float scale) {
#pragma unroll
  for (int q = 0; q < R; ++q) acc[q] = wave_sum(acc[q]);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) {
#pragma unroll
    for (int q = 0; q < R; ++q) lds[(threadIdx.x >> 6) * R + q] = acc[q];
  }
  __syncthreads();
  if (threadIdx.x < R) {
    float v = lds[threadIdx.x];
#pragma unroll
    for (int w = 1; w < NW; ++w) v += lds[w * R + threadIdx.x];
    t[row * R + threadIdx.x] = v;
    ext[row * R + threadIdx.x] = (bf16_t)(v * scale);
  }
}

// t = dy B of one target, one block of NW wavefronts per row (see RowLoraT)
template <int R, int NW>
__global__ __launch_bounds__(64 * NW) void lora_row_t_kernel(const bf16_t* __restrict__ dy, size_t lddy, int width, RowLoraT lt) {
  __shared__ float lds[NW * R];
  const size_t row = blockIdx.x;
  float acc[R];
#pragma unroll
  for (int q = 0; q < R; ++q) acc[q] = 0.f;
  const bf16_t* B = (const bf16_t*)lt.B[0];
  for (int i = threadIdx.x * 8; i < width; i += 64 * NW * 8) {
    const bf16x8 v = *reinterpret_cast<const bf16x8*>(dy + row * lddy + i);
    float vf[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) vf[j] = (float)v[j];
    lora_acc_cols<R, 8>(acc, vf, B + (size_t)i * R);
  }
  lora_row_finish<R, NW>(acc, lds, lt.t[0], (bf16_t*)lt.ext[0], row, lt.scale);
}

// --------------------------------------------------------------------------------------
// RMSNorm forward / backward (one block of 256 threads per row)
// --------------------------------------------------------------------------------------
// VEC: rows are read and written in 16-byte pieces (the host picks it when H is a multiple of the
// vector width and every pointer and row pitch is 16-byte aligned).
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const T* __restrict__ x, const T* __restrict__ g,
                                                      T* __restrict__ h, int H, float eps, T* __restrict__ save,
                                                      int save_row0, int save_rows) {
  __shared__ float red[4];
  constexpr int N = Vec<T>::N;
  const size_t row = blockIdx.x;
  const T* xr = x + row * H;
  // rows [save_row0, save_row0 + save_rows) also leave a copy of the INPUT row in `save` (the finetune
  // window's rows of an activation graph pruning keeps, written by the kernel that reads them anyway)
  T* sv = (save && (int)row >= save_row0 && (int)row < save_row0 + save_rows) ? save + (row - save_row0) * H : nullptr;
  float ss = 0.f;
  if (VEC) {
    for (int i = threadIdx.x * N; i < H; i += 256 * N) {
      float v[N];
      Vec<T>::load(xr + i, v);
      if (sv) Vec<T>::store(sv + i, v);
#pragma unroll
      for (int j = 0; j < N; ++j) ss += v[j] * v[j];
    }
  } else {
    for (int i = threadIdx.x; i < H; i += 256) {
      const float v = ld(xr + i);
      if (sv) st(sv + i, v);
      ss += v * v;
    }
  }
  ss = block_sum256(ss, red);
  const float rstd = 1.0f / sqrtf(ss / H + eps);
  if (VEC) {
    for (int i = threadIdx.x * N; i < H; i += 256 * N) {
      float v[N], gv[N];
      Vec<T>::load(xr + i, v);
      Vec<T>::load(g + i, gv);
#pragma unroll
      for (int j = 0; j < N; ++j) v[j] = v[j] * rstd * gv[j];
      Vec<T>::store(h + row * H + i, v);
    }
  } else {
    for (int i = threadIdx.x; i < H; i += 256) st(h + row * H + i, ld(xr + i) * rstd * ld(g + i));
  }
}

// v[0..N) = the N consecutive elements at `idx` of a product whose split-K partial sums still lie in
// part[split][stride]: added in split order and rounded to the storage type, exactly as the reduction
// kernel would have written them.
template <typename T, int N>
__device__ inline void load_split_sum(const float* __restrict__ part, int splits, size_t stride, size_t idx, float* v) {
#pragma unroll
  for (int j = 0; j < N; ++j) v[j] = 0.f;
  for (int sp = 0; sp < splits; ++sp) {
    const float* p = part + (size_t)sp * stride + idx;
    if (N % 4 == 0) {
#pragma unroll
      for (int q = 0; q < N / 4; ++q) {
        const f32x4 t = *reinterpret_cast<const f32x4*>(p + 4 * q);
#pragma unroll
        for (int j = 0; j < 4; ++j) v[4 * q + j] += t[j];
      }
    } else {
#pragma unroll
      for (int j = 0; j < N; ++j) v[j] += p[j];
    }
  }
#pragma unroll
  for (int j = 0; j < N; ++j) v[j] = (float)(T)v[j];
}

// dx = rstd * (g * dh) - x * rstd^3 * mean(x * g * dh)  (+ add);  hn (optional) = x rstd g, the row
// the forward norm produced (same arithmetic, same bits), for callers that need it again
// R > 0 (bf16, VEC): the produced row dx is also multiplied by a LoRA B matrix (see RowLoraT; one target = the whole row)
template <typename T, bool VEC, int R = 0>
__global__ __launch_bounds__(256) void rmsnorm_bwd_kernel(const T* __restrict__ x, const T* __restrict__ g,
                                                          const T* __restrict__ dh, const T* __restrict__ add,
                                                          T* __restrict__ dx, T* __restrict__ hn, int H, float eps,
                                                          const float* __restrict__ dh_part, int splits, size_t stride,
                                                          RowLoraT lt) {
  constexpr int RA = R > 0 ? R : 1;
  __shared__ float lt_lds[4 * RA];
  float lt_acc[RA];
#pragma unroll
  for (int q = 0; q < RA; ++q) lt_acc[q] = 0.f;
  // dh_part: dh still lies as split-K partial sums (see load_split_sum); the row's sums are kept in LDS
  // between the two passes (dynamic shared memory of H floats, only then)
  extern __shared__ float dh_row[];
  __shared__ float red[4];
  constexpr int N = Vec<T>::N;
  const size_t row = blockIdx.x;
  const T* xr = x + row * H;
  const T* dr = dh + row * H;
  float ss = 0.f, sd = 0.f;
  if (VEC) {
    for (int i = threadIdx.x * N; i < H; i += 256 * N) {
      float v[N], gv[N], dv[N];
      Vec<T>::load(xr + i, v);
      Vec<T>::load(g + i, gv);
      if (dh_part) {
        load_split_sum<T, N>(dh_part, splits, stride, row * H + i, dv);
#pragma unroll
        for (int j = 0; j < N; ++j) dh_row[i + j] = dv[j];
      } else {
        Vec<T>::load(dr + i, dv);
      }
#pragma unroll
      for (int j = 0; j < N; ++j) { ss += v[j] * v[j]; sd += v[j] * gv[j] * dv[j]; }
    }
  } else {
    for (int i = threadIdx.x; i < H; i += 256) {
      float v = ld(xr + i);
      float d1;
      if (dh_part) { load_split_sum<T, 1>(dh_part, splits, stride, row * H + i, &d1); dh_row[i] = d1; }
      else d1 = ld(dr + i);
      ss += v * v;
      sd += v * ld(g + i) * d1;
    }
  }
  ss = block_sum256(ss, red);
  sd = block_sum256(sd, red);
  const float rstd = 1.0f / sqrtf(ss / H + eps);
  const float coef = rstd * rstd * rstd * sd / H;
  if (VEC) {
    for (int i = threadIdx.x * N; i < H; i += 256 * N) {
      float v[N], gv[N], dv[N], av[N];
      Vec<T>::load(xr + i, v);
      Vec<T>::load(g + i, gv);
      if (dh_part) {           // (each thread reads back what it wrote itself)
#pragma unroll
        for (int j = 0; j < N; ++j) dv[j] = dh_row[i + j];
      } else {
        Vec<T>::load(dr + i, dv);
      }
      if (add) Vec<T>::load(add + row * H + i, av);
      if (hn) {
        float hv[N];
#pragma unroll
        for (int j = 0; j < N; ++j) hv[j] = v[j] * rstd * gv[j];
        Vec<T>::store(hn + row * H + i, hv);
      }
#pragma unroll
      for (int j = 0; j < N; ++j) {
        v[j] = rstd * gv[j] * dv[j] - v[j] * coef;
        if (add) v[j] += av[j];
      }
      Vec<T>::store(dx + row * H + i, v);
      if constexpr (R > 0) {   // (the values as they were just stored)
#pragma unroll
        for (int j = 0; j < N; ++j) v[j] = (float)(T)v[j];
        lora_acc_cols<R, N>(lt_acc, v, (const bf16_t*)lt.B[0] + (size_t)i * R);
      }
    }
    if constexpr (R > 0) lora_row_finish<R>(lt_acc, lt_lds, lt.t[0], (bf16_t*)lt.ext[0], row, lt.scale);
  } else {
    for (int i = threadIdx.x; i < H; i += 256) {
      if (hn) st(hn + row * H + i, ld(xr + i) * rstd * ld(g + i));
      float v = rstd * ld(g + i) * (dh_part ? dh_row[i] : ld(dr + i)) - ld(xr + i) * coef;
      if (add) v += ld(add + row * H + i);
      st(dx + row * H + i, v);
    }
  }
}

// The same backward for bf16 rows of up to 8192 elements, sixteen wavefronts per row: a thread owns four elements of
// each 4096-element stretch and keeps them in registers between the two passes, and every load of a row (x, g, the
// residual gradient, all split-K partial sums) is in flight at once.  A window of a few hundred rows gives the
// one-block-per-row kernel above one block of four wavefronts per CU, which waits out the latency of each of its
// loads in turn; here the chip holds four times as many wavefronts and each waits once.
// The sums over the row are taken in another order than above: hn may differ from the forward norm's row in the last
// bit of an element.
template <int R, int IT>
__global__ __launch_bounds__(1024) void rmsnorm_bwd_wide_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ g,
                                                                const bf16_t* __restrict__ dh,
                                                                const bf16_t* __restrict__ add, bf16_t* __restrict__ dx,
                                                                bf16_t* __restrict__ hn, int H, float eps,
                                                                const float* __restrict__ dh_part, int splits,
                                                                size_t stride, RowLoraT lt) {
  constexpr int RA = R > 0 ? R : 1;
  __shared__ float red[2][16];
  __shared__ float lt_lds[16 * RA];
  const size_t row = blockIdx.x;
  const int wave = threadIdx.x >> 6;
  float v[IT][4], gv[IT][4], dv[IT][4], av[IT][4];
  auto ld4 = [](const bf16_t* p, float (&o)[4]) {
    const bf16x4 t = *reinterpret_cast<const bf16x4*>(p);
#pragma unroll
    for (int j = 0; j < 4; ++j) o[j] = (float)t[j];
  };
  auto st4 = [](bf16_t* p, const float (&o)[4]) {
    bf16x4 t;
#pragma unroll
    for (int j = 0; j < 4; ++j) t[j] = (bf16_t)o[j];
    *reinterpret_cast<bf16x4*>(p) = t;
  };
  float ss = 0.f, sd = 0.f;
  bf16x8 bfrag[IT][4][R > 0 ? R / 8 : 1];   // the rows of B this thread's elements meet, fetched with the row
#pragma unroll
  for (int it = 0; it < IT; ++it) {
    const int i = (it * 1024 + (int)threadIdx.x) * 4;
#pragma unroll
    for (int j = 0; j < 4; ++j) v[it][j] = gv[it][j] = dv[it][j] = av[it][j] = 0.f;
    if (i < H) {
      if constexpr (R > 0) lora_load_cols<R, 4>(bfrag[it], (const bf16_t*)lt.B[0] + (size_t)i * R);
      ld4(x + row * H + i, v[it]);
      ld4(g + i, gv[it]);
      if (add) ld4(add + row * H + i, av[it]);
      if (dh_part) {   // split-K partial sums, added in split order and rounded to the storage type (see load_split_sum)
        const float* p = dh_part + row * H + i;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        int sp = 0;
        for (; sp + 4 <= splits; sp += 4) {
          const f32x4 t0 = *reinterpret_cast<const f32x4*>(p + (size_t)sp * stride);
          const f32x4 t1 = *reinterpret_cast<const f32x4*>(p + (size_t)(sp + 1) * stride);
          const f32x4 t2 = *reinterpret_cast<const f32x4*>(p + (size_t)(sp + 2) * stride);
          const f32x4 t3 = *reinterpret_cast<const f32x4*>(p + (size_t)(sp + 3) * stride);
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[j] = (((acc[j] + t0[j]) + t1[j]) + t2[j]) + t3[j];
        }
        for (; sp < splits; ++sp) {
          const f32x4 t0 = *reinterpret_cast<const f32x4*>(p + (size_t)sp * stride);
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[j] += t0[j];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) dv[it][j] = (float)(bf16_t)acc[j];
      } else {
        ld4(dh + row * H + i, dv[it]);
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) { ss += v[it][j] * v[it][j]; sd += v[it][j] * gv[it][j] * dv[it][j]; }
    }
  }
  ss = wave_sum(ss);
  sd = wave_sum(sd);
  if ((threadIdx.x & 63) == 0) { red[0][wave] = ss; red[1][wave] = sd; }
  __syncthreads();
  ss = sd = 0.f;
#pragma unroll
  for (int w = 0; w < 16; ++w) { ss += red[0][w]; sd += red[1][w]; }
  const float rstd = 1.0f / sqrtf(ss / H + eps);
  const float coef = rstd * rstd * rstd * sd / H;
  float lt_acc[RA];
#pragma unroll
  for (int q = 0; q < RA; ++q) lt_acc[q] = 0.f;
#pragma unroll
  for (int it = 0; it < IT; ++it) {
    const int i = (it * 1024 + (int)threadIdx.x) * 4;
    if (i < H) {
      if (hn) {
        float hv[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) hv[j] = v[it][j] * rstd * gv[it][j];
        st4(hn + row * H + i, hv);
      }
      float o[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        o[j] = rstd * gv[it][j] * dv[it][j] - v[it][j] * coef;
        if (add) o[j] += av[it][j];
      }
      st4(dx + row * H + i, o);
      if constexpr (R > 0) {   // (the values as they were just stored)
#pragma unroll
        for (int j = 0; j < 4; ++j) o[j] = (float)(bf16_t)o[j];
        lora_fma_cols<R, 4>(lt_acc, o, bfrag[it]);
      }
    }
  }
  if constexpr (R > 0) lora_row_finish<R, 16>(lt_acc, lt_lds, lt.t[0], (bf16_t*)lt.ext[0], row, lt.scale);
}

// Rotation angles.  Pair i of a head turns by pos * theta^(-2 i / d).  The host hands over the frequencies in
// revolutions, theta^(-2 i / d) / (2 pi), as doubles (a kernel argument: pow and a double-precision sincos per
// (token, i) on the device were a third of these kernels' run time).  The device takes the fractional part of
// pos * rev in double precision (exact to 1e-10 of a turn at any position) and the sine and cosine of that
// fraction of a turn in single precision (angle in [0, 2 pi): about 5e-7 absolute).
constexpr int ROPE_MAX_HALF = 128;   // head_dim <= 256
struct RopeFreq {
  double rev[ROPE_MAX_HALF];
};
__device__ inline void rope_cos_sin(const RopeFreq& f, int i, int pos, float* c, float* sn) {
  const double r = (double)pos * f.rev[i];
  const float turn = (float)(r - floor(r));
  sincosf(turn * 6.283185307179586f, sn, c);
}

// --------------------------------------------------------------------------------------
// RoPE + cache append (Alg. 2: Forward then Append of Q, K, V).  One block per token.
//   qkv row = [q heads | k heads | v heads]; q is rotated in place, k is rotated and
//   written to the K pages, v is written to the (position-minor) V pages, and rows of
//   the finetune window also store the rotated q in the sequence's Q cache.
// --------------------------------------------------------------------------------------
// VEC: a thread rotates Vec<T>::N neighbouring pairs of one head with 16-byte accesses (head_dim / 2 a
// multiple of the vector width, every pointer 16-byte aligned); same arithmetic, same results.
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void rope_append_kernel(T* __restrict__ qkv, const int32_t* __restrict__ tok_pos,
                                                          const int32_t* __restrict__ slot, T* __restrict__ kp,
                                                          T* __restrict__ vp, int nq, int nkv, int d, int ps,
                                                          RopeFreq freq, int ft_tok0, int n_ft, int ft_pos0,
                                                          T* __restrict__ q_cache) {
  extern __shared__ float cs[];   // cos[d/2], sin[d/2]
  const int t = blockIdx.x;
  const int pos = tok_pos[t];
  const int half = d >> 1;
  for (int i = threadIdx.x; i < half; i += 256) rope_cos_sin(freq, i, pos, &cs[i], &cs[half + i]);
  // the run of tokens this token's v row is written with (below): its first token and its length.  One lane per
  // neighbouring token looks at that token's slot and its predecessor's, all at once (a chain of dependent loads
  // along the run would cost more than the kernel's whole run time)
  constexpr int RUN = 16;
  __shared__ int run_info[2];
  if constexpr (VEC) {
    if (threadIdx.x < 64) {
      const int k = threadIdx.x, tt = t - (RUN - 1) + k;     // lanes 0 .. 31: tokens t - 15 .. t + 16
      bool first = false;                                     // tt begins a run (or lies past the batch)
      if (k < 2 * RUN) {
        if (tt >= (int)gridDim.x) first = true;
        else if (tt >= 0) {
          const int s1 = slot[tt];
          first = tt == 0 || slot[tt - 1] + 1 != s1 || (s1 % ps) % RUN == 0;
        }
      }
      const unsigned long long m = __ballot(first);
      if (k == 0) {
        const int k0 = 31 - __clz((unsigned)(m & 0xFFFFu));              // the last beginning at or before t
        const unsigned after = (unsigned)((m >> RUN) & 0xFFFFu);
        const int k1 = after ? RUN + __ffs(after) - 1 : 2 * RUN;         // the first beginning after t
        run_info[0] = t - (RUN - 1) + k0;
        run_info[1] = k1 - k0;
      }
    }
  }
  __syncthreads();
  const int qkv_dim = (nq + 2 * nkv) * d;
  T* row = qkv + (size_t)t * qkv_dim;
  const int sl = slot[t];
  const size_t page = sl / ps;
  const int pip = sl % ps;
  const bool is_ft = (t >= ft_tok0 && t < ft_tok0 + n_ft);
  // rotate q and k heads
  const T* vrow = row + (nq + nkv) * d;
  if constexpr (VEC) {
    constexpr int N = Vec<T>::N;
    const int hv = half / N;
    for (int idx = threadIdx.x; idx < (nq + nkv) * hv; idx += 256) {
      const int head = idx / hv, i = (idx % hv) * N;
      T* hp = row + head * d;
      float lo[N], hi[N], rlo[N], rhi[N];
      Vec<T>::load(hp + i, lo);
      Vec<T>::load(hp + half + i, hi);
#pragma unroll
      for (int j = 0; j < N; ++j) {
        const float c = cs[i + j], sn = cs[half + i + j];
        rlo[j] = lo[j] * c - hi[j] * sn;
        rhi[j] = hi[j] * c + lo[j] * sn;
      }
      if (head < nq) {
        Vec<T>::store(hp + i, rlo);
        Vec<T>::store(hp + half + i, rhi);
        if (is_ft) {
          T* qc = q_cache + (size_t)(ft_pos0 + (t - ft_tok0)) * nq * d + head * d;
          Vec<T>::store(qc + i, rlo);
          Vec<T>::store(qc + half + i, rhi);
        }
      } else {
        const int kh = head - nq;
        T* dst = kp + ((page * nkv + kh) * ps + pip) * (size_t)d;
        Vec<T>::store(dst + i, rlo);
        Vec<T>::store(dst + half + i, rhi);
      }
    }
    // v: a channel's positions are the contiguous index of a V page, so one token's row is nkv d scattered elements
    // (these stores were half of the kernel's time).  Tokens whose slots follow each other inside a page (a chunk's
    // rows) form a run; a run begins at a page's first position, at a multiple of 16 positions, and where the slot
    // is not the one after the previous token's.  The blocks of a run's tokens share its v rows out by channels:
    // each reads its channels of every row of the run (no block ever writes them) and stores, per channel, the
    // run's positions side by side - 16-byte pieces for a run of 16, a contiguous stretch of the page per block.
    const int t0 = run_info[0], len = run_info[1];
    const int j = t - t0;
    const int pip0 = pip - j;
    const int nv = nkv * d / N;                       // 16-byte pieces of a v row
    const int v_lo = (int)((long)nv * j / len), v_hi = (int)((long)nv * (j + 1) / len);
    const bool whole = len == RUN && ps % N == 0;
    const T* vrow0 = qkv + (size_t)t0 * qkv_dim + (nq + nkv) * d;
    for (int vi = v_lo + threadIdx.x; vi < v_hi; vi += 256) {
      const int idx = vi * N, kh = idx / d, i = idx % d;
      T* dst = vp + ((page * nkv + kh) * (size_t)d + i) * ps + pip0;
      if (whole) {        // (all sixteen loads in flight before the first store)
        float rows[RUN][N];
#pragma unroll
        for (int jj = 0; jj < RUN; ++jj) Vec<T>::load(vrow0 + (size_t)jj * qkv_dim + idx, rows[jj]);
#pragma unroll
        for (int c = 0; c < N; ++c) {
          float col[RUN];
#pragma unroll
          for (int jj = 0; jj < RUN; ++jj) col[jj] = rows[jj][c];
#pragma unroll
          for (int piece = 0; piece < RUN / N; ++piece) Vec<T>::store(dst + (size_t)c * ps + piece * N, &col[piece * N]);
        }
      } else {
        for (int jj = 0; jj < len; ++jj) {
          float v[N];
          Vec<T>::load(vrow0 + (size_t)jj * qkv_dim + idx, v);
#pragma unroll
          for (int c = 0; c < N; ++c) dst[(size_t)c * ps + jj] = (T)v[c];
        }
      }
    }
  } else {
    for (int idx = threadIdx.x; idx < (nq + nkv) * half; idx += 256) {
      const int head = idx / half, i = idx % half;
      T* hp = row + head * d;
      const float lo = ld(hp + i), hi = ld(hp + half + i);
      const float c = cs[i], sn = cs[half + i];
      const float rlo = lo * c - hi * sn, rhi = hi * c + lo * sn;
      if (head < nq) {
        st(hp + i, rlo);
        st(hp + half + i, rhi);
        if (is_ft) {
          T* qc = q_cache + (size_t)(ft_pos0 + (t - ft_tok0)) * nq * d + head * d;
          st(qc + i, rlo);
          st(qc + half + i, rhi);
        }
      } else {
        const int kh = head - nq;
        T* dst = kp + ((page * nkv + kh) * ps + pip) * (size_t)d;
        st(dst + i, rlo);
        st(dst + half + i, rhi);
      }
    }
    for (int idx = threadIdx.x; idx < nkv * d; idx += 256) {
      const int kh = idx / d, i = idx % d;
      vp[((page * nkv + kh) * (size_t)d + i) * ps + pip] = vrow[idx];
    }
  }
}

// Backward of the q/k/v rotation for a window: dqkv[n, (nq+2nkv)d] = [rope^T(dq) | rope^T(dk) | dv]
// dq rows are in the storage type, dk/dv rows are the (float) accumulator rows of the window.
// R > 0 (bf16): the packed row is also multiplied by the LoRA B matrices of q, k, v (see RowLoraT; entry 0 = q,
// 1 = k, 2 = v, B = NULL where the projection carries no LoRA)
// N consecutive floats with 16-byte loads
template <int N>
__device__ inline void load_f32_run(const float* p, float (&v)[N]) {
#pragma unroll
  for (int q4 = 0; q4 < N / 4; ++q4) {
    const f32x4 t = *reinterpret_cast<const f32x4*>(p + 4 * q4);
#pragma unroll
    for (int q = 0; q < 4; ++q) v[4 * q4 + q] = t[q];
  }
}

// VEC as in rope_append_kernel
template <typename T, int R = 0, bool VEC = false>
__global__ __launch_bounds__(256) void rope_bwd_pack_kernel(const T* __restrict__ dq, const float* __restrict__ dk,
                                                            const float* __restrict__ dv, T* __restrict__ dqkv,
                                                            int nq, int nkv, int d, RopeFreq freq, int win_start,
                                                            RowLoraT lt) {
  extern __shared__ float cs[];
  constexpr int RA = R > 0 ? R : 1;
  __shared__ float lt_lds[4 * RA];
  float acc_q[RA], acc_k[RA], acc_v[RA];
#pragma unroll
  for (int q = 0; q < RA; ++q) acc_q[q] = acc_k[q] = acc_v[q] = 0.f;
  const int r = blockIdx.x;
  const int pos = win_start + r;
  const int half = d >> 1;
  // a grid of two blocks per row (short windows: the row's chain of loads is the whole run time) gives the
  // query heads to block 0 and the key heads and v to block 1
  const int part = gridDim.y == 2 ? (int)blockIdx.y : -1;
  const int h_lo = part == 1 ? nq : 0, h_hi = part == 0 ? nq : nq + nkv;
  for (int i = threadIdx.x; i < half; i += 256) rope_cos_sin(freq, i, pos, &cs[i], &cs[half + i]);
  __syncthreads();
  T* out = dqkv + (size_t)r * (nq + 2 * nkv) * d;
  if constexpr (VEC) {
    constexpr int N = Vec<T>::N;
    const int hv = half / N;
    for (int idx = h_lo * hv + threadIdx.x; idx < h_hi * hv; idx += 256) {
      const int head = idx / hv, i = (idx % hv) * N;
      float lo[N], hi[N], rlo[N], rhi[N];
      if (head < nq) {
        const T* p = dq + (size_t)r * nq * d + head * d;
        Vec<T>::load(p + i, lo);
        Vec<T>::load(p + half + i, hi);
      } else {
        const float* p = dk + (size_t)r * nkv * d + (head - nq) * d;
        load_f32_run<N>(p + i, lo);
        load_f32_run<N>(p + half + i, hi);
      }
#pragma unroll
      for (int j = 0; j < N; ++j) {
        const float c = cs[i + j], sn = cs[half + i + j];
        // transpose of the rotation: turn by the negative angle
        rlo[j] = lo[j] * c + hi[j] * sn;
        rhi[j] = hi[j] * c - lo[j] * sn;
      }
      Vec<T>::store(out + head * d + i, rlo);
      Vec<T>::store(out + head * d + half + i, rhi);
      if constexpr (R > 0) {   // (the values as they were just stored)
#pragma unroll
        for (int j = 0; j < N; ++j) {
          rlo[j] = (float)(T)rlo[j];
          rhi[j] = (float)(T)rhi[j];
        }
        if (head < nq) {
          if (lt.B[0]) {
            const bf16_t* b = (const bf16_t*)lt.B[0] + (size_t)(head * d + i) * R;
            lora_acc_cols<R, N>(acc_q, rlo, b);
            lora_acc_cols<R, N>(acc_q, rhi, b + (size_t)half * R);
          }
        } else if (lt.B[1]) {
          const bf16_t* b = (const bf16_t*)lt.B[1] + (size_t)((head - nq) * d + i) * R;
          lora_acc_cols<R, N>(acc_k, rlo, b);
          lora_acc_cols<R, N>(acc_k, rhi, b + (size_t)half * R);
        }
      }
    }
    for (int idx = threadIdx.x * N; part != 0 && idx < nkv * d; idx += 256 * N) {
      float v[N];
      load_f32_run<N>(dv + (size_t)r * nkv * d + idx, v);
      Vec<T>::store(out + (nq + nkv) * d + idx, v);
      if constexpr (R > 0) {
        if (lt.B[2]) {
#pragma unroll
          for (int j = 0; j < N; ++j) v[j] = (float)(T)v[j];
          lora_acc_cols<R, N>(acc_v, v, (const bf16_t*)lt.B[2] + (size_t)idx * R);
        }
      }
    }
  } else {
  for (int idx = h_lo * half + threadIdx.x; idx < h_hi * half; idx += 256) {
    const int head = idx / half, i = idx % half;
    float lo, hi;
    if (head < nq) {
      const T* p = dq + (size_t)r * nq * d + head * d;
      lo = ld(p + i); hi = ld(p + half + i);
    } else {
      const float* p = dk + (size_t)r * nkv * d + (head - nq) * d;
      lo = p[i]; hi = p[half + i];
    }
    const float c = cs[i], sn = cs[half + i];
    // transpose of the rotation: turn by the negative angle
    const float rlo = lo * c + hi * sn, rhi = hi * c - lo * sn;
    st(out + head * d + i, rlo);
    st(out + head * d + half + i, rhi);
    if constexpr (R > 0) {   // (the values as they were just stored)
      const float vlo = (float)(T)rlo, vhi = (float)(T)rhi;
      if (head < nq) {
        if (lt.B[0]) {
          const bf16_t* b = (const bf16_t*)lt.B[0] + (size_t)(head * d + i) * R;
          lora_acc_row<R>(acc_q, vlo, b);
          lora_acc_row<R>(acc_q, vhi, b + (size_t)half * R);
        }
      } else if (lt.B[1]) {
        const bf16_t* b = (const bf16_t*)lt.B[1] + (size_t)((head - nq) * d + i) * R;
        lora_acc_row<R>(acc_k, vlo, b);
        lora_acc_row<R>(acc_k, vhi, b + (size_t)half * R);
      }
    }
  }
  for (int idx = threadIdx.x; part != 0 && idx < nkv * d; idx += 256) {
    const float v = dv[(size_t)r * nkv * d + idx];
    st(out + (nq + nkv) * d + idx, v);
    if constexpr (R > 0) {
      if (lt.B[2]) lora_acc_row<R>(acc_v, (float)(T)v, (const bf16_t*)lt.B[2] + (size_t)idx * R);
    }
  }
  }
  if constexpr (R > 0) {
    if (lt.B[0] && part != 1) lora_row_finish<R>(acc_q, lt_lds, lt.t[0], (bf16_t*)lt.ext[0], r, lt.scale);
    if (lt.B[1] && part != 0) lora_row_finish<R>(acc_k, lt_lds, lt.t[1], (bf16_t*)lt.ext[1], r, lt.scale);
    if (lt.B[2] && part != 0) lora_row_finish<R>(acc_v, lt_lds, lt.t[2], (bf16_t*)lt.ext[2], r, lt.scale);
  }
}

// --------------------------------------------------------------------------------------
// (IA)^3 bypass network (Sec. 4.1: Y = X + X (.) (l - 1) = X (.) l on the adapter's rows).
// Forward: one block per listed token; up to two column ranges of the row, each with its own vector;
// rows of the finetune window first keep the unscaled values (the other operand of the product, which
// the vector's gradient needs).
// --------------------------------------------------------------------------------------
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void ia3_scale_rows_kernel(T* __restrict__ buf, size_t ldb,
                                                             const int32_t* __restrict__ tok, Ia3ScaleArgs a) {
  constexpr int N = VEC ? Vec<T>::N : 1;
  const int t = tok[blockIdx.x];
  T* row = buf + (size_t)t * ldb;
  const bool is_ft = t >= a.ft_tok0 && t < a.ft_tok0 + a.n_ft;
  for (int sg = 0; sg < a.n_seg; ++sg) {
    const T* l = (const T*)a.l[sg];
    T* sv = (is_ft && a.save[sg]) ? (T*)a.save[sg] + (size_t)(a.ft_pos0 + (t - a.ft_tok0)) * a.ld_save[sg] : nullptr;
    T* p = row + a.col0[sg];
    for (int c = threadIdx.x * N; c < a.width[sg]; c += 256 * N) {
      float v[N], lv[N];
      if (VEC) {
        Vec<T>::load(p + c, v);
        Vec<T>::load(l + c, lv);
        if (sv) Vec<T>::store(sv + c, v);          // (a value of type T passes through float unchanged)
#pragma unroll
        for (int j = 0; j < N; ++j) v[j] *= lv[j];
        Vec<T>::store(p + c, v);
      } else {
        v[0] = ld(p + c);
        if (sv) st(sv + c, v[0]);
        st(p + c, v[0] * ld(l + c));
      }
    }
  }
}

// Backward of the product Y = X (.) l over a window of n rows: G holds dY.  Per chunk of IA3_CHUNK rows and
// per column, part[chunk][c] = sum_r G[r, c] X[r, c] (the chunk's share of dl[c]), and G[r, c] <- G[r, c] l[c]
// (= dX) in place.  The second kernel adds the chunks in order into dl: no atomics, a fixed order.
constexpr int IA3_CHUNK = 8;
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void ia3_colgrad_kernel(T* __restrict__ G, size_t ldg, const T* __restrict__ X,
                                                          size_t ldx, const T* __restrict__ l,
                                                          float* __restrict__ part, int n, int C) {
  constexpr int N = VEC ? Vec<T>::N : 1;
  const int c = (blockIdx.x * 256 + threadIdx.x) * N;
  if (c >= C) return;
  const int r0 = blockIdx.y * IA3_CHUNK;
  float lv[N], acc[N], g[IA3_CHUNK][N], x[IA3_CHUNK][N];
  if (VEC) Vec<T>::load(l + c, lv); else lv[0] = ld(l + c);
#pragma unroll
  for (int j = 0; j < N; ++j) acc[j] = 0.f;
#pragma unroll
  for (int i = 0; i < IA3_CHUNK; ++i) {            // every load of the chunk in flight before the first use
    const int r = min(r0 + i, n - 1);
    if (VEC) { Vec<T>::load(G + (size_t)r * ldg + c, g[i]); Vec<T>::load(X + (size_t)r * ldx + c, x[i]); }
    else { g[i][0] = ld(G + (size_t)r * ldg + c); x[i][0] = ld(X + (size_t)r * ldx + c); }
  }
#pragma unroll
  for (int i = 0; i < IA3_CHUNK; ++i) {
    if (r0 + i >= n) break;
#pragma unroll
    for (int j = 0; j < N; ++j) { acc[j] += g[i][j] * x[i][j]; g[i][j] *= lv[j]; }
    if (VEC) Vec<T>::store(G + (size_t)(r0 + i) * ldg + c, g[i]); else st(G + (size_t)(r0 + i) * ldg + c, g[i][0]);
  }
#pragma unroll
  for (int j = 0; j < N; ++j) part[(size_t)blockIdx.y * C + c + j] = acc[j];
}

__global__ __launch_bounds__(256) void ia3_colgrad_finalize_kernel(const float* __restrict__ part, int chunks, int C,
                                                                   float* __restrict__ dl) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= C) return;
  float acc = 0.f;
  for (int k0 = 0; k0 < chunks; k0 += 8) {   // eight loads in flight, added in chunk order
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = k0 + i < chunks ? part[(size_t)(k0 + i) * C + c] : 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) acc += v[i];
  }
  dl[c] += acc;
}

// --------------------------------------------------------------------------------------
// SwiGLU forward / backward
// --------------------------------------------------------------------------------------
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void swiglu_kernel(const T* __restrict__ gu, T* __restrict__ act, int F) {
  constexpr int N = VEC ? Vec<T>::N : 1;
  const size_t row = blockIdx.y;
  const int i = (blockIdx.x * 256 + threadIdx.x) * N;
  if (i >= F) return;
  float g[N], u[N];
  if (VEC) { Vec<T>::load(gu + row * 2 * F + i, g); Vec<T>::load(gu + row * 2 * F + F + i, u); }
  else { g[0] = ld(gu + row * 2 * F + i); u[0] = ld(gu + row * 2 * F + F + i); }
#pragma unroll
  for (int j = 0; j < N; ++j) g[j] = g[j] / (1.0f + __expf(-g[j])) * u[j];
  if (VEC) Vec<T>::store(act + row * F + i, g); else st(act + row * F + i, g[0]);
}

// from saved gate, up and dact: dgu = [dgate | dup]
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void swiglu_bwd_kernel(const T* __restrict__ gate, const T* __restrict__ up,
                                                         const T* __restrict__ dact, T* __restrict__ dgu,
                                                         T* __restrict__ act, int F, const float* __restrict__ dact_part,
                                                         int splits, size_t stride) {
  constexpr int N = VEC ? Vec<T>::N : 1;
  const size_t row = blockIdx.y;
  const int i = (blockIdx.x * 256 + threadIdx.x) * N;
  if (i >= F) return;
  float g[N], u[N], da[N];
  if (VEC) { Vec<T>::load(gate + row * F + i, g); Vec<T>::load(up + row * F + i, u); }
  else { g[0] = ld(gate + row * F + i); u[0] = ld(up + row * F + i); }
  if (dact_part) load_split_sum<T, N>(dact_part, splits, stride, row * F + i, da);   // dact still lies as split-K partial sums
  else if (VEC) Vec<T>::load(dact + row * F + i, da);
  else da[0] = ld(dact + row * F + i);
  float dg[N], du[N];
#pragma unroll
  for (int j = 0; j < N; ++j) {
    const float sg = 1.0f / (1.0f + __expf(-g[j]));
    dg[j] = da[j] * u[j] * (sg + g[j] * sg * (1.0f - sg));
    du[j] = da[j] * g[j] * sg;
  }
  if (VEC) { Vec<T>::store(dgu + row * 2 * F + i, dg); Vec<T>::store(dgu + row * 2 * F + F + i, du); }
  else { st(dgu + row * 2 * F + i, dg[0]); st(dgu + row * 2 * F + F + i, du[0]); }
  if (act) {   // the rematerialised SwiGLU output (as swiglu_remat_kernel computes it), for callers that need it again
#pragma unroll
    for (int j = 0; j < N; ++j) g[j] = g[j] / (1.0f + __expf(-g[j])) * u[j];
    if (VEC) Vec<T>::store(act + row * F + i, g); else st(act + row * F + i, g[0]);
  }
}

// act = silu(gate) * up from the saved gate and up (rematerialisation, Alg. 1)
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void swiglu_remat_kernel(const T* __restrict__ gate, const T* __restrict__ up,
                                                           T* __restrict__ act, int F) {
  constexpr int N = VEC ? Vec<T>::N : 1;
  const size_t row = blockIdx.y;
  const int i = (blockIdx.x * 256 + threadIdx.x) * N;
  if (i >= F) return;
  float g[N], u[N];
  if (VEC) { Vec<T>::load(gate + row * F + i, g); Vec<T>::load(up + row * F + i, u); }
  else { g[0] = ld(gate + row * F + i); u[0] = ld(up + row * F + i); }
#pragma unroll
  for (int j = 0; j < N; ++j) g[j] = g[j] / (1.0f + __expf(-g[j])) * u[j];
  if (VEC) Vec<T>::store(act + row * F + i, g); else st(act + row * F + i, g[0]);
}

// --------------------------------------------------------------------------------------
// strided row copy: dst row i = src row i, `width` units of V (uint4 = 16 bytes, or 4-byte words)
// --------------------------------------------------------------------------------------
// several strided row copies in one launch (blockIdx.z picks the copy); widths in 16-byte units
__global__ __launch_bounds__(256) void copy_rows_batch_kernel(CopyRowsBatch b) {
  const int e = blockIdx.z;
  const size_t row = blockIdx.y;
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= b.width16[e]) return;
  reinterpret_cast<uint4*>(b.dst[e] + row * b.ld_dst[e])[i] = reinterpret_cast<const uint4*>(b.src[e] + row * b.ld_src[e])[i];
}

template <typename V>
__global__ __launch_bounds__(256) void copy_rows_kernel(const char* __restrict__ src, size_t ld_src,
                                                        char* __restrict__ dst, size_t ld_dst, int width) {
  const size_t row = blockIdx.y;
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= width) return;
  reinterpret_cast<V*>(dst + row * ld_dst)[i] = reinterpret_cast<const V*>(src + row * ld_src)[i];
}

// --------------------------------------------------------------------------------------
// LoRA building blocks on a row range.  S(i, j) denotes element (long index i, rank index j)
// of a LoRA matrix, addressed as S[i * s_i + j * s_j], so that the same kernels serve
// A [r, in] (s_i = 1, s_j = in) and B [out, r] (s_i = r, s_j = 1).
// --------------------------------------------------------------------------------------
// out[m, j] = sum_i X[m, i] * S(i, j)        one block per row m; R = rank bound
template <typename T, int R>
__global__ __launch_bounds__(256) void lora_reduce_long_kernel(const T* __restrict__ X, size_t ldx,
                                                               const T* __restrict__ S, size_t s_i, size_t s_j,
                                                               float* __restrict__ out, int n_long, int r,
                                                               const int32_t* __restrict__ row_idx) {
  __shared__ float red[4][R];
  const size_t mo = blockIdx.x;
  const size_t m = row_idx ? (size_t)row_idx[mo] : mo;
  float acc[R];
#pragma unroll
  for (int j = 0; j < R; ++j) acc[j] = 0.f;
  for (int i = threadIdx.x; i < n_long; i += 256) {
    const float xv = ld(X + m * ldx + i);
#pragma unroll
    for (int j = 0; j < R; ++j)
      if (j < r) acc[j] += xv * ld(S + (size_t)i * s_i + (size_t)j * s_j);
  }
#pragma unroll
  for (int j = 0; j < R; ++j) {
    const float v = wave_sum(acc[j]);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6][j] = v;
  }
  __syncthreads();
  if (threadIdx.x < r) out[mo * r + threadIdx.x] = red[0][threadIdx.x] + red[1][threadIdx.x] + red[2][threadIdx.x] + red[3][threadIdx.x];
}

// Y[m, i] += scale * sum_j U[m, j] * S(i, j)     grid (ceil(n_long/256), ceil(n/16))
template <typename T, int R>
__global__ __launch_bounds__(256) void lora_expand_kernel(const float* __restrict__ U, const T* __restrict__ S,
                                                          size_t s_i, size_t s_j, T* __restrict__ Y, size_t ldy,
                                                          int n, int n_long, int r, float scale,
                                                          const int32_t* __restrict__ row_idx) {
  __shared__ float us[16][R];
  const int m0 = blockIdx.y * 16;
  for (int idx = threadIdx.x; idx < 16 * R; idx += 256) {
    const int mm = idx / R, j = idx % R;
    us[mm][j] = (m0 + mm < n && j < r) ? U[(size_t)(m0 + mm) * r + j] : 0.f;
  }
  __syncthreads();
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= n_long) return;
  float sv[R];
#pragma unroll
  for (int j = 0; j < R; ++j) sv[j] = (j < r) ? ld(S + (size_t)i * s_i + (size_t)j * s_j) : 0.f;
  for (int mm = 0; mm < 16 && m0 + mm < n; ++mm) {
    float a = 0.f;
#pragma unroll
    for (int j = 0; j < R; ++j) a += us[mm][j] * sv[j];
    const size_t yr = row_idx ? (size_t)row_idx[m0 + mm] : (size_t)(m0 + mm);
    T* y = Y + yr * ldy + i;
    st(y, ld(y) + scale * a);
  }
}

// G(i, j) += scale * sum_m X[m, i] * U[m, j]      one thread per long index i, all ranks j
template <typename T, int R>
__global__ __launch_bounds__(256) void lora_outer_kernel(const T* __restrict__ X, size_t ldx,
                                                         const float* __restrict__ U, float* __restrict__ G,
                                                         size_t g_i, size_t g_j, int n, int n_long, int r,
                                                         float scale) {
  __shared__ float us[64][R];
  const int i = blockIdx.x * 256 + threadIdx.x;
  float acc[R];
#pragma unroll
  for (int j = 0; j < R; ++j) acc[j] = 0.f;
  for (int m0 = 0; m0 < n; m0 += 64) {
    __syncthreads();
    for (int idx = threadIdx.x; idx < 64 * R; idx += 256) {
      const int mm = idx / R, j = idx % R;
      us[mm][j] = (m0 + mm < n && j < r) ? U[(size_t)(m0 + mm) * r + j] : 0.f;
    }
    __syncthreads();
    if (i < n_long) {
      const int mend = min(64, n - m0);
      for (int mm = 0; mm < mend; ++mm) {
        const float xv = ld(X + (size_t)(m0 + mm) * ldx + i);
#pragma unroll
        for (int j = 0; j < R; ++j) acc[j] += xv * us[mm][j];
      }
    }
  }
  if (i < n_long) {
#pragma unroll
    for (int j = 0; j < R; ++j)
      if (j < r) G[(size_t)i * g_i + (size_t)j * g_j] += scale * acc[j];
  }
}

// --------------------------------------------------------------------------------------
// type-generic dense projection (fallback and the fp32 configuration)
//   TRANS_W = false: C[m, n] = sum_k A[m, k] W[n, k]      TRANS_W = true: ... W[k, n]
// 64 x 64 tile, BK = 16, 256 threads, 4 x 4 outputs per thread, fp32 accumulation.
// --------------------------------------------------------------------------------------
template <typename T, bool TRANS_W>
__global__ __launch_bounds__(256) void gemm_generic_kernel(const T* __restrict__ A, const T* __restrict__ W,
                                                           T* __restrict__ C, const T* __restrict__ bias,
                                                           const T* __restrict__ residual, int M, int N, int K,
                                                           size_t lda, size_t ldw, size_t ldc, size_t ldr) {
  __shared__ float As[16][64 + 1];
  __shared__ float Ws[16][64 + 1];
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
    for (int idx = threadIdx.x; idx < 64 * 16; idx += 256) {
      const int mm = idx / 16, kk = idx % 16;
      As[kk][mm] = (m0 + mm < M && k0 + kk < K) ? ld(A + (size_t)(m0 + mm) * lda + k0 + kk) : 0.f;
      if (!TRANS_W) {
        Ws[kk][mm] = (n0 + mm < N && k0 + kk < K) ? ld(W + (size_t)(n0 + mm) * ldw + k0 + kk) : 0.f;
      }
    }
    if (TRANS_W) {
      for (int idx = threadIdx.x; idx < 64 * 16; idx += 256) {
        const int kk = idx / 64, nn = idx % 64;
        Ws[kk][nn] = (n0 + nn < N && k0 + kk < K) ? ld(W + (size_t)(k0 + kk) * ldw + n0 + nn) : 0.f;
      }
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; b[i] = Ws[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      float v = acc[i][j];
      if (bias) v += ld(bias + n);
      if (residual) v += ld(residual + (size_t)m * ldr + n);
      st(C + (size_t)m * ldc + n, v);
    }
  }
}

// --------------------------------------------------------------------------------------
// host launchers
// --------------------------------------------------------------------------------------
#define DISPATCH_T(dtype, ...)                                   \
  do {                                                           \
    if ((dtype) == FLEXCO_BF16) { using T = bf16_t; __VA_ARGS__; } \
    else { using T = float; __VA_ARGS__; }                       \
  } while (0)

static int32_t post_launch(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(FLEXCO_EHIP, "launch of %s failed: %s", what, hipGetErrorString(e));
  return FLEXCO_OK;
}

int32_t launch_gemm_generic(const void* A, const void* W, void* C, const void* bias, const void* residual, int M,
                            int N, int K, size_t lda, size_t ldw, size_t ldc, size_t ldr, bool trans_w, int dtype,
                            hipStream_t s) {
  dim3 grid((N + 63) / 64, (M + 63) / 64);
  DISPATCH_T(dtype, {
    if (trans_w)
      hipLaunchKernelGGL((gemm_generic_kernel<T, true>), grid, dim3(256), 0, s, (const T*)A, (const T*)W, (T*)C,
                         (const T*)bias, (const T*)residual, M, N, K, lda, ldw, ldc, ldr);
    else
      hipLaunchKernelGGL((gemm_generic_kernel<T, false>), grid, dim3(256), 0, s, (const T*)A, (const T*)W, (T*)C,
                         (const T*)bias, (const T*)residual, M, N, K, lda, ldw, ldc, ldr);
  });
  return post_launch("gemm_generic");
}

// 16-byte row accesses are possible when the width is a multiple of 16 bytes and everything is aligned
static bool vec_ok(int dtype, int width, std::initializer_list<const void*> ptrs) {
  const int nvec = dtype == FLEXCO_BF16 ? 8 : 4;
  if (width % nvec != 0) return false;
  for (const void* p : ptrs)
    if (p && !aligned16(p)) return false;
  return true;
}
#define DISPATCH_TV(dtype, vec, ...)                                  \
  do {                                                               \
    if (vec) { constexpr bool VEC = true; DISPATCH_T(dtype, __VA_ARGS__); }  \
    else { constexpr bool VEC = false; DISPATCH_T(dtype, __VA_ARGS__); }     \
  } while (0)

int32_t launch_rmsnorm(const void* x, const void* g, void* h, int T_, int H, float eps, int dtype, hipStream_t s,
                       void* save, int save_row0, int save_rows) {
  if (T_ == 0) return FLEXCO_OK;
  const bool vec = vec_ok(dtype, H, {x, g, h, save});
  DISPATCH_TV(dtype, vec, hipLaunchKernelGGL((rmsnorm_kernel<T, VEC>), dim3(T_), dim3(256), 0, s, (const T*)x,
                                             (const T*)g, (T*)h, H, eps, (T*)save, save_row0, save ? save_rows : 0));
  return post_launch("rmsnorm");
}

int32_t launch_rmsnorm_bwd(const void* x, const void* g, const void* dh, const void* add, void* dx, int T_, int H,
                           float eps, int dtype, hipStream_t s, void* hn, const float* dh_part, int splits,
                           const RowLoraT* lt_in) {
  if (T_ == 0) return FLEXCO_OK;
  const bool vec = vec_ok(dtype, H, {x, g, dh, add, dx, hn, dh_part});
  const size_t shm = dh_part ? sizeof(float) * (size_t)H : 0;
  RowLoraT lt = {};
  // bf16 rows of up to 8192 elements: sixteen wavefronts per row
  if (dtype == FLEXCO_BF16 && vec && H <= 8192 && (!lt_in || lt_in->n == 0 || (lt_in->n == 1 && row_lora_ok(dtype, lt_in->r)))) {
    if (lt_in && lt_in->n > 0) lt = *lt_in;
    const int R = lt_in && lt_in->n > 0 ? lt.r : 0;
    const size_t stride = (size_t)T_ * H;
#define FLEXCO_NORM_BWD_WIDE(R_, IT_)                                                                              \
    hipLaunchKernelGGL((rmsnorm_bwd_wide_kernel<R_, IT_>), dim3(T_), dim3(1024), 0, s, (const bf16_t*)x,            \
                       (const bf16_t*)g, (const bf16_t*)dh, (const bf16_t*)add, (bf16_t*)dx, (bf16_t*)hn, H, eps,   \
                       dh_part, splits, stride, lt)
    if (H <= 4096) {
      if (R == 0) FLEXCO_NORM_BWD_WIDE(0, 1); else if (R == 16) FLEXCO_NORM_BWD_WIDE(16, 1); else FLEXCO_NORM_BWD_WIDE(32, 1);
    } else {
      if (R == 0) FLEXCO_NORM_BWD_WIDE(0, 2); else if (R == 16) FLEXCO_NORM_BWD_WIDE(16, 2); else FLEXCO_NORM_BWD_WIDE(32, 2);
    }
#undef FLEXCO_NORM_BWD_WIDE
    return post_launch("rmsnorm_bwd");
  }
  if (lt_in && lt_in->n > 0) {
    if (!vec || !row_lora_ok(dtype, lt_in->r) || lt_in->n != 1) return fail(FLEXCO_EUNSUPPORTED, "rmsnorm_bwd: row product not covered");
    lt = *lt_in;
    const size_t stride = (size_t)T_ * H;
#define FLEXCO_NORM_BWD_LT(R_)                                                                                     \
    hipLaunchKernelGGL((rmsnorm_bwd_kernel<bf16_t, true, R_>), dim3(T_), dim3(256), shm, s, (const bf16_t*)x,       \
                       (const bf16_t*)g, (const bf16_t*)dh, (const bf16_t*)add, (bf16_t*)dx, (bf16_t*)hn, H, eps,   \
                       dh_part, splits, stride, lt)
    if (lt.r == 16) FLEXCO_NORM_BWD_LT(16); else FLEXCO_NORM_BWD_LT(32);
#undef FLEXCO_NORM_BWD_LT
    return post_launch("rmsnorm_bwd");
  }
  DISPATCH_TV(dtype, vec, hipLaunchKernelGGL((rmsnorm_bwd_kernel<T, VEC>), dim3(T_), dim3(256), shm, s, (const T*)x,
                                             (const T*)g, (const T*)dh, (const T*)add, (T*)dx, (T*)hn, H, eps, dh_part,
                                             splits, (size_t)T_ * H, lt));
  return post_launch("rmsnorm_bwd");
}

// The frequencies of a (theta, head_dim) pair, computed once (a model has one pair; a lock guards the few cached ones).
static int32_t rope_freq(const flexco_layer_cfg& c, RopeFreq* out) {
  const int half = c.head_dim / 2;
  if (half > ROPE_MAX_HALF) return fail(FLEXCO_EUNSUPPORTED, "rotary embedding: head_dim %d above %d", c.head_dim, 2 * ROPE_MAX_HALF);
  struct Entry { float theta; int d; RopeFreq f; };
  static std::mutex mu;
  static std::vector<Entry> cache;
  std::lock_guard<std::mutex> lock(mu);
  for (const Entry& e : cache)
    if (e.theta == c.rope_theta && e.d == c.head_dim) { *out = e.f; return FLEXCO_OK; }
  Entry e;
  e.theta = c.rope_theta; e.d = c.head_dim;
  for (int i = 0; i < ROPE_MAX_HALF; ++i)
    e.f.rev[i] = i < half ? std::pow((double)c.rope_theta, -2.0 * (double)i / (double)c.head_dim) / 6.283185307179586476925 : 0.0;
  if (cache.size() >= 16) cache.clear();
  cache.push_back(e);
  *out = e.f;
  return FLEXCO_OK;
}

int32_t launch_rope_append(const flexco_layer_cfg& c, void* qkv, const int32_t* tok_pos, const int32_t* slot,
                           const flexco_kv_pool& pool, int T_, int ft_tok0, int n_ft, int ft_pos0, void* q_cache,
                           hipStream_t s) {
  if (T_ == 0) return FLEXCO_OK;
  const size_t shm = sizeof(float) * c.head_dim;
  RopeFreq freq;
  FLEXCO_TRY(rope_freq(c, &freq));
  const bool vec = c.head_dim % 2 == 0 && vec_ok(c.dtype, c.head_dim / 2, {qkv, pool.k_pages, pool.v_pages, q_cache});
  DISPATCH_TV(c.dtype, vec, hipLaunchKernelGGL((rope_append_kernel<T, VEC>), dim3(T_), dim3(256), shm, s, (T*)qkv, tok_pos,
                                               slot, (T*)pool.k_pages, (T*)pool.v_pages, c.n_q_heads, c.n_kv_heads,
                                               c.head_dim, c.page_size, freq, ft_tok0, n_ft, ft_pos0,
                                               (T*)q_cache));
  return post_launch("rope_append");
}

int32_t launch_rope_bwd_pack(const flexco_layer_cfg& c, const void* dq, const float* dk_rows, const float* dv_rows,
                             void* dqkv, int win_start, int n, hipStream_t s, const RowLoraT* lt_in) {
  const size_t shm = sizeof(float) * c.head_dim;
  if (n == 0) return FLEXCO_OK;
  RopeFreq freq;
  FLEXCO_TRY(rope_freq(c, &freq));
  const dim3 grid(n, n <= 512 ? 2 : 1);   // few rows: two blocks per row
  // 16-byte accesses: also the float rows of dk / dv (their row pitch nkv d floats is a multiple of 16 bytes then)
  const bool vec = c.head_dim % 2 == 0 && vec_ok(c.dtype, c.head_dim / 2, {dq, dk_rows, dv_rows, dqkv});
  RowLoraT lt = {};
  if (lt_in && lt_in->n > 0) {
    if (!row_lora_ok(c.dtype, lt_in->r)) return fail(FLEXCO_EUNSUPPORTED, "rope_bwd_pack: row product not covered");
    lt = *lt_in;
#define FLEXCO_ROPE_BWD_LT(R_, V_)                                                                                      \
  hipLaunchKernelGGL((rope_bwd_pack_kernel<bf16_t, R_, V_>), grid, dim3(256), shm, s, (const bf16_t*)dq, dk_rows, dv_rows, \
                     (bf16_t*)dqkv, c.n_q_heads, c.n_kv_heads, c.head_dim, freq, win_start, lt)
    if (lt.r == 16) { if (vec) FLEXCO_ROPE_BWD_LT(16, true); else FLEXCO_ROPE_BWD_LT(16, false); }
    else { if (vec) FLEXCO_ROPE_BWD_LT(32, true); else FLEXCO_ROPE_BWD_LT(32, false); }
#undef FLEXCO_ROPE_BWD_LT
    return post_launch("rope_bwd_pack");
  }
  DISPATCH_TV(c.dtype, vec, hipLaunchKernelGGL((rope_bwd_pack_kernel<T, 0, VEC>), grid, dim3(256), shm, s, (const T*)dq,
                                               dk_rows, dv_rows, (T*)dqkv, c.n_q_heads, c.n_kv_heads, c.head_dim,
                                               freq, win_start, lt));
  return post_launch("rope_bwd_pack");
}

int32_t launch_lora_row_t(const void* dy, size_t lddy, int n, int width, const RowLoraT& lt, hipStream_t s) {
  if (n == 0) return FLEXCO_OK;
  if (!row_lora_ok(FLEXCO_BF16, lt.r) || width % 8 != 0 || lddy % 8 != 0 || !aligned16(dy) || !aligned16(lt.B[0]))
    return fail(FLEXCO_EUNSUPPORTED, "lora_row_t: shape not covered");
  // (sixteen wavefronts per row were measured slower here: the sixteen sums per wavefront at the end grow with them)
  if (lt.r == 16) hipLaunchKernelGGL((lora_row_t_kernel<16, 4>), dim3(n), dim3(256), 0, s, (const bf16_t*)dy, lddy, width, lt);
  else hipLaunchKernelGGL((lora_row_t_kernel<32, 4>), dim3(n), dim3(256), 0, s, (const bf16_t*)dy, lddy, width, lt);
  return post_launch("lora_row_t");
}

int32_t launch_ia3_scale_rows(void* buf, size_t ld, const int32_t* tok, int n_tok, const Ia3ScaleArgs& a, int dtype,
                              hipStream_t s) {
  if (n_tok == 0 || a.n_seg == 0) return FLEXCO_OK;
  const int vn = dtype == FLEXCO_BF16 ? 8 : 4;
  bool vec = ld % vn == 0 && aligned16(buf);
  for (int sg = 0; sg < a.n_seg; ++sg)
    vec = vec && a.col0[sg] % vn == 0 && a.width[sg] % vn == 0 && aligned16(a.l[sg]) && aligned16(a.save[sg]) &&
          a.ld_save[sg] % vn == 0;
  DISPATCH_TV(dtype, vec, hipLaunchKernelGGL((ia3_scale_rows_kernel<T, VEC>), dim3(n_tok), dim3(256), 0, s, (T*)buf, ld,
                                             tok, a));
  return post_launch("ia3_scale_rows");
}

int32_t launch_ia3_colgrad(void* G, size_t ldg, const void* X, size_t ldx, const void* l, float* part, float* dl, int n,
                           int C, int dtype, hipStream_t s) {
  if (n == 0 || C == 0) return FLEXCO_OK;
  const int chunks = (n + IA3_CHUNK - 1) / IA3_CHUNK;
  const int vn = dtype == FLEXCO_BF16 ? 8 : 4;
  const bool vec = C % vn == 0 && ldg % vn == 0 && ldx % vn == 0 && aligned16(G) && aligned16(X) && aligned16(l);
  const int per = 256 * (vec ? vn : 1);
  DISPATCH_TV(dtype, vec, hipLaunchKernelGGL((ia3_colgrad_kernel<T, VEC>), dim3((C + per - 1) / per, chunks), dim3(256), 0,
                                             s, (T*)G, ldg, (const T*)X, ldx, (const T*)l, part, n, C));
  hipLaunchKernelGGL(ia3_colgrad_finalize_kernel, dim3((C + 255) / 256), dim3(256), 0, s, part, chunks, C, dl);
  return post_launch("ia3_colgrad");
}

int32_t launch_swiglu(const void* gu, void* act, int T_, int F, int dtype, hipStream_t s) {
  if (T_ == 0) return FLEXCO_OK;
  const bool vec = vec_ok(dtype, F, {gu, act});
  const int per = 256 * (vec ? (dtype == FLEXCO_BF16 ? 8 : 4) : 1);
  DISPATCH_TV(dtype, vec, hipLaunchKernelGGL((swiglu_kernel<T, VEC>), dim3((F + per - 1) / per, T_), dim3(256), 0, s,
                                             (const T*)gu, (T*)act, F));
  return post_launch("swiglu");
}

int32_t launch_swiglu_bwd(const void* gate, const void* up, const void* dact, void* dgu, int n, int F, int dtype,
                          hipStream_t s, void* act, const float* dact_part, int splits) {
  if (n == 0) return FLEXCO_OK;
  const bool vec = vec_ok(dtype, F, {gate, up, dact, dgu, act, dact_part});
  const int per = 256 * (vec ? (dtype == FLEXCO_BF16 ? 8 : 4) : 1);
  DISPATCH_TV(dtype, vec, hipLaunchKernelGGL((swiglu_bwd_kernel<T, VEC>), dim3((F + per - 1) / per, n), dim3(256), 0,
                                             s, (const T*)gate, (const T*)up, (const T*)dact, (T*)dgu, (T*)act, F, dact_part,
                                             splits, (size_t)n * F));
  return post_launch("swiglu_bwd");
}

int32_t launch_swiglu_remat(const void* gate, const void* up, void* act, int n, int F, int dtype, hipStream_t s) {
  if (n == 0) return FLEXCO_OK;
  const bool vec = vec_ok(dtype, F, {gate, up, act});
  const int per = 256 * (vec ? (dtype == FLEXCO_BF16 ? 8 : 4) : 1);
  DISPATCH_TV(dtype, vec, hipLaunchKernelGGL((swiglu_remat_kernel<T, VEC>), dim3((F + per - 1) / per, n), dim3(256), 0,
                                             s, (const T*)gate, (const T*)up, (T*)act, F));
  return post_launch("swiglu_remat");
}

// Several row copies with the same row count in one launch; falls back to one launch per copy when
// a copy is not made of aligned 16-byte pieces.
int32_t launch_copy_rows_batch(const CopyRowsBatch& b, int n_rows, size_t const* width_bytes, hipStream_t s) {
  if (n_rows == 0 || b.count == 0) return FLEXCO_OK;
  bool v16 = true;
  int wmax = 0;
  for (int e = 0; e < b.count; ++e) {
    v16 = v16 && width_bytes[e] % 16 == 0 && b.ld_src[e] % 16 == 0 && b.ld_dst[e] % 16 == 0 && aligned16(b.src[e]) &&
          aligned16(b.dst[e]);
    wmax = b.width16[e] > wmax ? b.width16[e] : wmax;
  }
  if (!v16) {
    for (int e = 0; e < b.count; ++e)
      FLEXCO_TRY(launch_copy_rows(b.src[e], b.ld_src[e], b.dst[e], b.ld_dst[e], n_rows, width_bytes[e], s));
    return FLEXCO_OK;
  }
  hipLaunchKernelGGL(copy_rows_batch_kernel, dim3((wmax + 255) / 256, n_rows, b.count), dim3(256), 0, s, b);
  return post_launch("copy_rows_batch");
}

int32_t launch_copy_rows(const void* src, size_t ld_src_bytes, void* dst, size_t ld_dst_bytes, int n_rows,
                         size_t width_bytes, hipStream_t s) {
  if (n_rows == 0 || width_bytes == 0) return FLEXCO_OK;
  if (width_bytes % 4) return fail(FLEXCO_ESHAPE, "row copy of %zu bytes is not a multiple of 4", width_bytes);
  const bool v16 = width_bytes % 16 == 0 && ld_src_bytes % 16 == 0 && ld_dst_bytes % 16 == 0 && aligned16(src) &&
                   aligned16(dst);
  if (v16) {
    const int w = (int)(width_bytes / 16);
    hipLaunchKernelGGL((copy_rows_kernel<uint4>), dim3((w + 255) / 256, n_rows), dim3(256), 0, s, (const char*)src,
                       ld_src_bytes, (char*)dst, ld_dst_bytes, w);
  } else {
    const int w = (int)(width_bytes / 4);
    hipLaunchKernelGGL((copy_rows_kernel<uint32_t>), dim3((w + 255) / 256, n_rows), dim3(256), 0, s, (const char*)src,
                       ld_src_bytes, (char*)dst, ld_dst_bytes, w);
  }
  return post_launch("copy_rows");
}

template <int R>
static int32_t lora_ops(int op, const void* X, size_t ldx, const void* S, size_t s_i, size_t s_j, float* U,
                        void* Y, size_t ldy, float* G, size_t g_i, size_t g_j, int n, int n_long, int r,
                        float scale, int dtype, const int32_t* row_idx, hipStream_t s) {
  DISPATCH_T(dtype, {
    if (op == 0)
      hipLaunchKernelGGL((lora_reduce_long_kernel<T, R>), dim3(n), dim3(256), 0, s, (const T*)X, ldx, (const T*)S,
                         s_i, s_j, U, n_long, r, row_idx);
    else if (op == 1)
      hipLaunchKernelGGL((lora_expand_kernel<T, R>), dim3((n_long + 255) / 256, (n + 15) / 16), dim3(256), 0, s, U,
                         (const T*)S, s_i, s_j, (T*)Y, ldy, n, n_long, r, scale, row_idx);
    else
      hipLaunchKernelGGL((lora_outer_kernel<T, R>), dim3((n_long + 255) / 256), dim3(256), 0, s, (const T*)X, ldx,
                         U, G, g_i, g_j, n, n_long, r, scale);
  });
  return post_launch("lora kernel");
}

static int32_t lora_dispatch(int op, const void* X, size_t ldx, const void* S, size_t s_i, size_t s_j, float* U,
                             void* Y, size_t ldy, float* G, size_t g_i, size_t g_j, int n, int n_long, int r,
                             float scale, int dtype, hipStream_t s, const int32_t* row_idx = nullptr) {
  if (n == 0) return FLEXCO_OK;
  if (r <= 8) return lora_ops<8>(op, X, ldx, S, s_i, s_j, U, Y, ldy, G, g_i, g_j, n, n_long, r, scale, dtype, row_idx, s);
  if (r <= 16) return lora_ops<16>(op, X, ldx, S, s_i, s_j, U, Y, ldy, G, g_i, g_j, n, n_long, r, scale, dtype, row_idx, s);
  if (r <= 32) return lora_ops<32>(op, X, ldx, S, s_i, s_j, U, Y, ldy, G, g_i, g_j, n, n_long, r, scale, dtype, row_idx, s);
  return lora_ops<64>(op, X, ldx, S, s_i, s_j, U, Y, ldy, G, g_i, g_j, n, n_long, r, scale, dtype, row_idx, s);
}

// u <- relu(u); where u <= 0 the matching element of t (if given) is zeroed: the ReLU's backward mask
__global__ __launch_bounds__(256) void relu_mask_kernel(float* __restrict__ u, float* __restrict__ t, size_t count) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= count) return;
  if (!(u[i] > 0.f)) {
    u[i] = 0.f;
    if (t) t[i] = 0.f;
  }
}

int32_t launch_relu_mask(float* u, float* t, size_t count, hipStream_t s) {
  if (count == 0) return FLEXCO_OK;
  hipLaunchKernelGGL(relu_mask_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, s, u, t, count);
  return post_launch("relu_mask");
}

// u[n, r] = x[rows, in] A^T,  A [r, in]; rows = row_idx[0..n) or 0..n
int32_t launch_lora_shrink(const void* x, size_t ldx, const void* A, float* u, int n, int in, int r, int dtype,
                           const int32_t* row_idx, hipStream_t s) {
  return lora_dispatch(0, x, ldx, A, 1, (size_t)in, u, nullptr, 0, nullptr, 0, 0, n, in, r, 0.f, dtype, s, row_idx);
}
// y[rows, out] += scale * u B^T,  B [out, r]
int32_t launch_lora_expand(const float* u, const void* B, void* y, size_t ldy, int n, int out, int r, float scale,
                           int dtype, const int32_t* row_idx, hipStream_t s) {
  return lora_dispatch(1, nullptr, 0, B, (size_t)r, 1, const_cast<float*>(u), y, ldy, nullptr, 0, 0, n, out, r,
                       scale, dtype, s, row_idx);
}

// Gradients of one LoRA bypass on n rows (Sec. 4.1 form y = scale (x A^T) B^T):
//   u = x A^T; t = dy B; dB += scale dy^T u; dA += scale t^T x; dx += scale t A
// With relu (a bottleneck adapter: y = relu(x A^T) B^T) u becomes relu(u) and t is zeroed where u <= 0.
int32_t launch_lora_bwd(const void* x, size_t ldx, const void* dy, size_t lddy, const void* A, const void* B,
                        float* dA, float* dB, void* dx, size_t lddx, float* u_ws, float* t_ws, int n, int in,
                        int out, int r, float scale, int dtype, hipStream_t s, bool relu) {
  int32_t rc;
  if ((rc = lora_dispatch(0, x, ldx, A, 1, (size_t)in, u_ws, nullptr, 0, nullptr, 0, 0, n, in, r, 0.f, dtype, s))) return rc;
  if ((rc = lora_dispatch(0, dy, lddy, B, (size_t)r, 1, t_ws, nullptr, 0, nullptr, 0, 0, n, out, r, 0.f, dtype, s))) return rc;
  if (relu && (rc = launch_relu_mask(u_ws, t_ws, (size_t)n * r, s))) return rc;
  if ((rc = lora_dispatch(2, dy, lddy, nullptr, 0, 0, u_ws, nullptr, 0, dB, (size_t)r, 1, n, out, r, scale, dtype, s))) return rc;
  if ((rc = lora_dispatch(2, x, ldx, nullptr, 0, 0, t_ws, nullptr, 0, dA, 1, (size_t)in, n, in, r, scale, dtype, s))) return rc;
  if (dx)
    if ((rc = lora_dispatch(1, nullptr, 0, A, 1, (size_t)in, t_ws, dx, lddx, nullptr, 0, 0, n, in, r, scale, dtype, s))) return rc;
  return FLEXCO_OK;
}

}  // namespace flexco

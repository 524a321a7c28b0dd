// bf16 LoRA kernels around the projection GEMMs.
//
// The bypass network of Sec. 4.1, y = f_B(x) + scale (x A^T) B^T with rank r << in, out, is
// split so that the large dimension is touched once:
//   shrink   u = x A^T  (or t = dy B)   skinny product [n, K] x [K, r] on the matrix cores:
//            one wavefront multiplies 16 rows by up to 64 ranks with v_mfma_f32_16x16x32_bf16,
//            both operands fetched straight from global memory (8 consecutive k per lane),
//            K is cut across the up to 16 wavefronts of a block, whose partial sums are added
//            in wavefront order through LDS, so results do not depend on scheduling; the block
//            writes the fp32 result and/or the scaled bf16 operand of the GEMM extension.
//   expand   is not a kernel: the projection GEMM appends the rank-r product as extra
//            k-steps (gemm_mfma.hip), reading the bf16 matrix the shrink kernel writes.
//   outer    dB += scale dy^T u,  dA += scale t^T x : every output element is a sum over
//            the window's rows only; plain FMA code, 64 consecutive outputs per wavefront,
//            rows interleaved over the block's 4 wavefronts, fixed-order LDS reduction.
#include <cstring>
#include "flexco_internal.h"
#include "device_types.h"

namespace flexco {

namespace {

// One block per 16 rows and matrix; K is cut across the block's wavefronts (blockDim.x / 64, a
// power of two <= 16), whose partial sums are added in wavefront order through LDS.
template <int RT>   // rank tiles of 16
__global__ __launch_bounds__(1024) void lora_shrink_kernel(LoraShrinkArgs a) {
  __shared__ float red[16][RT][64][4];
  const int z = blockIdx.y, tile = blockIdx.x;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nw = blockDim.x >> 6;
  const int m = lane & 15, g = lane >> 4;
  const int row = tile * 16 + m;
  const int want = a.want[z];
  const int row_ad = (row < a.rows && a.row_adapter) ? a.row_adapter[row] : 0;
  const bool row_ok = row < a.rows && row_ad >= 0 && (want < 0 || row_ad == want);
  // every wavefront looks at the same 16 rows, so this is the same for the whole block
  const bool any_row = __ballot(row_ok) != 0;
  if (!any_row) {   // a tile without adapter rows: only its zero rows of the GEMM operand are due
    if (a.out_ext[z] && blockIdx.z == 0)
      for (int idx = threadIdx.x; idx < 16 * a.r; idx += blockDim.x)
        if (tile * 16 + idx / a.r < a.rows) a.out_ext[z][(size_t)tile * 16 * a.r + idx] = (bf16_t)0.f;
    return;
  }
  const bf16_t* X = a.X[z];
  const bf16_t* S = a.S[z];
  const size_t src_row = row_ok ? (size_t)row : 0;   // rows without adapter read row 0; their results are dropped
  const int k_wave = a.K[z] / (nw * a.ksplit);
  const int k0 = (blockIdx.z * nw + wave) * k_wave, k1 = k0 + k_wave;
  const bf16_t* xp = X + src_row * a.ldx[z] + g * 8;
  const bf16_t* sp[RT];
  bool rank_ok[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    rank_ok[rt] = rt * 16 + m < a.r;
    sp[rt] = S + (size_t)(rank_ok[rt] ? rt * 16 + m : 0) * a.lds[z] + g * 8;
  }
  f32x4 acc[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) acc[rt] = f32x4{0.f, 0.f, 0.f, 0.f};
  const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
  // This kernel lives on memory latency: the loads of U steps are issued together, then multiplied.
  // k_wave is a multiple of 128 (4 steps); chunks of 8 steps while they fit (narrow ranks only).
#define FLEXCO_SHRINK_CHUNK(U_)                                                                       \
  {                                                                                                   \
    bf16x8 xa_[U_], sb_[U_][RT];                                                                      \
    _Pragma("unroll") for (int u = 0; u < U_; ++u) {                                                  \
      xa_[u] = *reinterpret_cast<const bf16x8*>(xp + k + 32 * u);                                     \
      _Pragma("unroll") for (int rt = 0; rt < RT; ++rt)                                               \
        sb_[u][rt] = *reinterpret_cast<const bf16x8*>(sp[rt] + k + 32 * u);                           \
    }                                                                                                 \
    _Pragma("unroll") for (int u = 0; u < U_; ++u)                                                    \
      _Pragma("unroll") for (int rt = 0; rt < RT; ++rt)                                               \
        acc[rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa_[u], rank_ok[rt] ? sb_[u][rt] : zero, acc[rt], 0, 0, 0); \
    k += 32 * U_;                                                                                     \
  }
  int k = k0;
  if (RT <= 2)
    while (k + 256 <= k1) FLEXCO_SHRINK_CHUNK(8)
  while (k < k1) FLEXCO_SHRINK_CHUNK(4)
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int q = 0; q < 4; ++q) red[wave][rt][lane][q] = acc[rt][q];
  __syncthreads();
  // D[row = 4 (lane / 16) + e][rank = lane % 16]: the 256 (lane, e) pairs of a rank tile are shared
  // out over the block's threads
  for (int idx = threadIdx.x; idx < 256; idx += blockDim.x) {
    const int ln = idx >> 2, e = idx & 3;
    const int orow = tile * 16 + 4 * (ln >> 4) + e;
    if (orow >= a.rows) continue;
    const int o_ad = a.row_adapter ? a.row_adapter[orow] : 0;
    const bool out_ok = o_ad >= 0 && (want < 0 || o_ad == want);
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      const int rank = rt * 16 + (ln & 15);
      if (rank >= a.r) continue;
      float v = 0.f;
      for (int w = 0; w < nw; ++w) v += red[w][rt][ln][e];
      const size_t o = (size_t)orow * a.r + rank;
      if (a.ksplit > 1) {   // partial product of this block's k range; the finalize kernel adds them up
        a.part[((size_t)(z * a.ksplit + blockIdx.z) * a.rows) * a.r + o] = v;
        continue;
      }
      if (a.out_f32[z] && out_ok && orow >= a.f32_lo && orow < a.f32_hi)
        a.out_f32[z][(size_t)(orow - a.f32_lo) * a.r + rank] = v;
      if (a.out_ext[z]) a.out_ext[z][o] = (bf16_t)(out_ok ? v * a.scale : 0.f);
    }
  }
}

// Second step of a shrink whose contraction was cut over several blocks: out = sum of the partial
// products in block order, written like the one-step kernel writes it.
__global__ __launch_bounds__(256) void lora_shrink_finalize_kernel(LoraShrinkArgs a) {
  const int z = blockIdx.y;
  const size_t o = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (o >= (size_t)a.rows * a.r) return;
  const int orow = (int)(o / a.r), rank = (int)(o % a.r);
  const int o_ad = a.row_adapter ? a.row_adapter[orow] : 0;
  const bool out_ok = o_ad >= 0 && (a.want[z] < 0 || o_ad == a.want[z]);
  float v = 0.f;
  if (out_ok)   // (a tile without any adapter row wrote no partial products)
    for (int ks = 0; ks < a.ksplit; ++ks) v += a.part[((size_t)(z * a.ksplit + ks) * a.rows) * a.r + o];
  if (a.out_f32[z] && out_ok && orow >= a.f32_lo && orow < a.f32_hi)
    a.out_f32[z][(size_t)(orow - a.f32_lo) * a.r + rank] = v;
  if (a.out_ext[z]) a.out_ext[z][o] = (bf16_t)(out_ok ? v * a.scale : 0.f);
}

// Bt[j][o] = B[o][j]
__global__ __launch_bounds__(256) void lora_transpose_kernel(LoraTransposeArgs a) {
  const int z = blockIdx.z;
  const int o = blockIdx.x * 256 + threadIdx.x;
  if (o >= a.out[z]) return;
  for (int j = 0; j < a.r; ++j) a.Bt[z][(size_t)j * a.out[z] + o] = a.B[z][(size_t)o * a.r + j];
}

// G(i, j) += scale * sum_m X[m, i] U[m, j],  G element (i, j) at G[i * g_i + j * g_j]
// Rows are taken in chunks of 256: the chunk's U rows are staged in LDS (broadcast reads), each
// wavefront owns 64 rows of the chunk and issues their 64 loads of X together (a 256-row window is one
// chunk: one wait for U, one for X).
template <int R>
__global__ __launch_bounds__(256) void lora_outer_mfma_path_kernel(LoraOuterArgs a) {
  const int e = blockIdx.y;
  const int n = a.n, r = a.r, n_long = a.n_long[e];
  if ((int)blockIdx.x * 64 >= n_long) return;   // entries of one launch differ in width
  const bf16_t* __restrict__ X = a.X[e];
  const float* __restrict__ U = a.U[e];
  float* __restrict__ G = a.G[e];
  const size_t ldx = a.ldx[e], g_i = a.g_i[e], g_j = a.g_j[e];
  const float scale = a.scale;
  extern __shared__ float smem[];   // us[256][R], later reused as red[3][64][R]
  constexpr int CH = 256, RB = 64;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i = blockIdx.x * 64 + lane;
  const int ic = i < n_long ? i : n_long - 1;
  float acc[R];
#pragma unroll
  for (int j = 0; j < R; ++j) acc[j] = 0.f;
  for (int mb = 0; mb < n; mb += CH) {
    __syncthreads();
    for (int idx = threadIdx.x; idx < CH * R; idx += 256) {
      const int mm = idx / R, j = idx % R;
      smem[idx] = (mb + mm < n && j < r) ? U[(size_t)(mb + mm) * r + j] : 0.f;
    }
    __syncthreads();
    float xv[RB];
#pragma unroll
    for (int q = 0; q < RB; ++q) {
      const int m = mb + wave * RB + q;
      xv[q] = (float)X[(size_t)(m < n ? m : n - 1) * ldx + ic];   // rows past n meet zero U rows
    }
#pragma unroll
    for (int q = 0; q < RB; ++q) {
      const float* u = smem + (wave * RB + q) * R;
#pragma unroll
      for (int j = 0; j < R; ++j) acc[j] += xv[q] * u[j];
    }
  }
  __syncthreads();
  if (wave > 0) {
#pragma unroll
    for (int j = 0; j < R; ++j) smem[((wave - 1) * 64 + lane) * R + j] = acc[j];
  }
  __syncthreads();
  if (wave == 0 && i < n_long) {
    // all loads of the accumulated gradient first, then the stores (one round trip, not R in a row)
    float gv[R];
#pragma unroll
    for (int j = 0; j < R; ++j) gv[j] = j < r ? G[(size_t)i * g_i + (size_t)j * g_j] : 0.f;
#pragma unroll
    for (int j = 0; j < R; ++j) {
      if (j < r) {
        const float v = acc[j] + smem[(0 * 64 + lane) * R + j] + smem[(1 * 64 + lane) * R + j] + smem[(2 * 64 + lane) * R + j];
        G[(size_t)i * g_i + (size_t)j * g_j] = gv[j] + scale * v;
      }
    }
  }
}

int32_t post(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(FLEXCO_EHIP, "launch of %s failed: %s", what, hipGetErrorString(e));
  return FLEXCO_OK;
}

}  // namespace

int32_t launch_lora_shrink_mfma(const LoraShrinkArgs& a_in, int n_mats, hipStream_t s) {
  LoraShrinkArgs a = a_in;
  if (a.rows == 0 || n_mats == 0) return FLEXCO_OK;
  for (int z = 0; z < n_mats; ++z)
    if (a.K[z] % 128 != 0) return fail(FLEXCO_ESHAPE, "LoRA shrink: K = %d is not a multiple of 128", a.K[z]);
  // K is cut into whole groups of 4 MFMA steps (128 columns), first over the wavefronts of a block (a
  // power of two <= 16), and - long contractions with scratch at hand - over several blocks per row tile,
  // so that more than rows / 16 CUs pull the operands in
  int kmin = a.K[0], kmax = a.K[0];
  for (int z = 1; z < n_mats; ++z) { kmin = a.K[z] < kmin ? a.K[z] : kmin; kmax = a.K[z] > kmax ? a.K[z] : kmax; }
  a.ksplit = 1;
  if (a.part && n_mats <= a.part_slots && kmin == kmax && kmax >= 8192)
    for (int sp = LORA_SHRINK_SPLITS; sp > 1; --sp)
      if (kmax % (128 * sp) == 0 && kmax / sp >= 1024) { a.ksplit = sp; break; }
  int nw = a.ksplit > 1 ? 8 : 16;
  for (int z = 0; z < n_mats; ++z)
    while (nw > 1 && a.K[z] % (128 * nw * a.ksplit) != 0) nw >>= 1;
  const dim3 grid((a.rows + 15) / 16, n_mats, a.ksplit), block(64 * nw);
  const int rt = (a.r + 15) / 16;
  switch (rt) {
    case 1: hipLaunchKernelGGL(lora_shrink_kernel<1>, grid, block, 0, s, a); break;
    case 2: hipLaunchKernelGGL(lora_shrink_kernel<2>, grid, block, 0, s, a); break;
    case 3: hipLaunchKernelGGL(lora_shrink_kernel<3>, grid, block, 0, s, a); break;
    default: hipLaunchKernelGGL(lora_shrink_kernel<4>, grid, block, 0, s, a); break;
  }
  if (a.ksplit > 1)
    hipLaunchKernelGGL(lora_shrink_finalize_kernel, dim3((unsigned)(((size_t)a.rows * a.r + 255) / 256), n_mats), dim3(256),
                       0, s, a);
  return post("lora_shrink");
}

int32_t launch_lora_transpose(const LoraTransposeArgs& a, int n_mats, hipStream_t s) {
  int mx = 0;
  for (int z = 0; z < n_mats; ++z) mx = a.out[z] > mx ? a.out[z] : mx;
  if (mx == 0) return FLEXCO_OK;
  hipLaunchKernelGGL(lora_transpose_kernel, dim3((mx + 255) / 256, 1, n_mats), dim3(256), 0, s, a);
  return post("lora_transpose");
}

int32_t launch_lora_outer_batch(const LoraOuterArgs& a, hipStream_t s) {
  if (a.n == 0 || a.count == 0) return FLEXCO_OK;
  int mx = 0;
  for (int e = 0; e < a.count; ++e) mx = a.n_long[e] > mx ? a.n_long[e] : mx;
  const dim3 grid((mx + 63) / 64, a.count);
  if (a.r <= 16)
    hipLaunchKernelGGL(lora_outer_mfma_path_kernel<16>, grid, dim3(256), 256 * 16 * sizeof(float), s, a);
  else if (a.r <= 32)
    hipLaunchKernelGGL(lora_outer_mfma_path_kernel<32>, grid, dim3(256), 256 * 32 * sizeof(float), s, a);
  else
    hipLaunchKernelGGL(lora_outer_mfma_path_kernel<64>, grid, dim3(256), 256 * 64 * sizeof(float), s, a);
  return post("lora_outer");
}

int32_t launch_lora_outer_bf16(const void* X, size_t ldx, const float* U, float* G, size_t g_i, size_t g_j, int n,
                               int n_long, int r, float scale, hipStream_t s) {
  LoraOuterArgs a;
  memset(&a, 0, sizeof(a));
  a.X[0] = (const bf16_t*)X; a.ldx[0] = ldx; a.U[0] = U; a.G[0] = G; a.g_i[0] = g_i; a.g_j[0] = g_j; a.n_long[0] = n_long;
  a.count = 1; a.n = n; a.r = r; a.scale = scale;
  return launch_lora_outer_batch(a, s);
}

}  // namespace flexco

// bf16 projections on the matrix cores (v_mfma_f32_32x32x16_bf16), LDS-staged.
//
//   TRANS = false:  C[M, N] = A[M, K] W[N, K]^T (+ bias[N]) (+ residual[M, N])   forward form
//   TRANS = true :  C[M, N] = A[M, K] W[K, N]                                      input-gradient form
//
// The frozen base projections run over ALL tokens of the mixed batch in one launch, so a
// weight is read from HBM once per iteration whatever the mix of inference and finetuning
// tokens (the paper's fused forward, Sec. 6.2).  The input-gradient form serves the
// token-window backward, where weight gradients are pruned away (Alg. 1) and only
// dX = dY W remains.
//
// Tiling: block tile BM x BN x 64, 256 threads = 4 wavefronts in a 2 x 2 grid, each owning
// (BM/2) x (BN/2) as 32 x 32 MFMA tiles with fp32 accumulators.  Operand tiles are staged
// through LDS in two buffers: the next tile's global loads are issued before the MFMAs of
// the current one and written to the other buffer afterwards (one barrier per k-step).
//   * A tile and the forward W tile are [rows][64] bf16 = 128-byte rows; the eight 16-byte
//     chunks of a row are XOR-swizzled with (row >> 1) & 7, so that both the 16-byte writes
//     and the ds_read_b128 operand fetches of 16 consecutive rows hit 64 distinct banks.
//   * The transposed W tile is [64][BN + 8]: an operand fragment (8 consecutive k for one
//     column) is gathered with 16-bit LDS reads; the 16-byte row padding puts the two
//     k-halves of a wavefront on disjoint banks.
// Work-group ids are remapped so that ids that land on the same XCD (id mod 8) work on
// neighbouring tiles, M fastest: the W tile they share stays in that XCD's L2.
#include "flexco_internal.h"
#include "device_types.h"

namespace flexco {

namespace {

constexpr int BK = 64;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ inline int swz(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

template <int BM, int BN, bool TRANS>
struct Smem {
  static constexpr int A_ELEMS = BM * BK;
  static constexpr int B_LD = TRANS ? (BN + 8) : BK;
  static constexpr int B_ELEMS = TRANS ? BK * (BN + 8) : BN * BK;
  static constexpr size_t BYTES = 2 * (size_t)(A_ELEMS + B_ELEMS) * sizeof(bf16_t);
};

template <int BM, int BN, bool TRANS>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(const bf16_t* __restrict__ A, const bf16_t* __restrict__ W,
                                                        bf16_t* __restrict__ C, const bf16_t* __restrict__ bias,
                                                        const bf16_t* __restrict__ res, int M, int N, int K,
                                                        size_t lda, size_t ldw, size_t ldc, size_t ldr, int tiles_m,
                                                        int tiles_n, GemmExt ext, float* __restrict__ part,
                                                        int k_chunk) {
  constexpr int WM = BM / 2, WN = BN / 2, MT = WM / 32, NT = WN / 32;
  using S = Smem<BM, BN, TRANS>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t* As = reinterpret_cast<bf16_t*>(smem_raw);                 // [2][BM][64] swizzled
  bf16_t* Bs = As + 2 * S::A_ELEMS;                                 // [2][...]

  // ---- work-group id -> tile, XCD-aware ------------------------------------------------
  int lid = blockIdx.x;
  const int nblk = gridDim.x;
  if ((nblk & 7) == 0) lid = (blockIdx.x & 7) * (nblk >> 3) + (blockIdx.x >> 3);
  const int tm = lid % tiles_m, tn = lid / tiles_m;
  const int m0 = tm * BM, n0 = tn * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave >> 1) * WM, wn0 = (wave & 1) * WN;

  // ---- global -> register staging --------------------------------------------------------
  constexpr int A_PASSES = BM / 32;                                  // 8 chunks per row, 32 rows per pass
  constexpr int B_PASSES = TRANS ? (BK * (BN / 8)) / 256 : BN / 32;
  u32x4 sa0[A_PASSES], sb0[B_PASSES], sa1[A_PASSES], sb1[B_PASSES];   // two sets of staging registers
  const int a_c = tid & 7, a_r = tid >> 3;
  constexpr int BCH = BN / 8;                                        // chunks per row of the transposed W tile
  const int bt_c = tid % BCH, bt_r = tid / BCH;

  // (kept as macros on purpose: staging arrays captured by lambdas were left in scratch memory)
#define FLEXCO_LOAD_TILES(k0_, ra, rb)                                                                      \
  {                                                                                                   \
    _Pragma("unroll") for (int p = 0; p < A_PASSES; ++p) {                                            \
      const int r_ = min(m0 + a_r + 32 * p, M - 1);                                                   \
      ra[p] = *reinterpret_cast<const u32x4*>(A + (size_t)r_ * lda + (k0_) + a_c * 8);                \
    }                                                                                                 \
    if (!TRANS) {                                                                                     \
      _Pragma("unroll") for (int p = 0; p < B_PASSES; ++p) {                                          \
        const int r_ = min(n0 + a_r + 32 * p, N - 1);                                                 \
        rb[p] = *reinterpret_cast<const u32x4*>(W + (size_t)r_ * ldw + (k0_) + a_c * 8);              \
      }                                                                                               \
    } else {                                                                                          \
      _Pragma("unroll") for (int p = 0; p < B_PASSES; ++p) {                                          \
        const int kr_ = bt_r + (256 / BCH) * p;                                                       \
        int col_ = n0 + bt_c * 8;                                                                     \
        if (col_ >= N) col_ = 0; /* masked at the store */                                            \
        rb[p] = *reinterpret_cast<const u32x4*>(W + (size_t)((k0_) + kr_) * ldw + col_);              \
      }                                                                                               \
    }                                                                                                 \
  }
#define FLEXCO_STORE_TILES(buf_, ra, rb)                                                                    \
  {                                                                                                   \
    bf16_t* as_ = As + (buf_) * S::A_ELEMS;                                                           \
    bf16_t* bs_ = Bs + (buf_) * S::B_ELEMS;                                                           \
    _Pragma("unroll") for (int p = 0; p < A_PASSES; ++p) {                                            \
      const int r_ = a_r + 32 * p;                                                                    \
      *reinterpret_cast<u32x4*>(as_ + r_ * BK + swz(r_, a_c) * 8) = ra[p];                            \
    }                                                                                                 \
    if (!TRANS) {                                                                                     \
      _Pragma("unroll") for (int p = 0; p < B_PASSES; ++p) {                                          \
        const int r_ = a_r + 32 * p;                                                                  \
        *reinterpret_cast<u32x4*>(bs_ + r_ * BK + swz(r_, a_c) * 8) = rb[p];                          \
      }                                                                                               \
    } else {                                                                                          \
      _Pragma("unroll") for (int p = 0; p < B_PASSES; ++p) {                                          \
        const int kr_ = bt_r + (256 / BCH) * p;                                                       \
        *reinterpret_cast<u32x4*>(bs_ + kr_ * S::B_LD + bt_c * 8) = rb[p];                            \
      }                                                                                               \
    }                                                                                                 \
  }

  f32x16 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // split-K: blockIdx.y owns k in [kbeg, kbeg + k_chunk) and writes fp32 partial sums to `part`
  const int kbeg = blockIdx.y * k_chunk;
  const int nk = k_chunk / BK;
  const int l32 = lane & 31, kg = lane >> 5;

#define FLEXCO_LOAD_FRAGS(kk_, af_, bf_)                                                              \
  {                                                                                                   \
    _Pragma("unroll") for (int i = 0; i < MT; ++i) {                                                  \
      const int r_ = wm0 + i * 32 + l32;                                                              \
      af_[i] = *reinterpret_cast<const bf16x8*>(as + r_ * BK + swz(r_, (kk_) * 2 + kg) * 8);          \
    }                                                                                                 \
    _Pragma("unroll") for (int j = 0; j < NT; ++j) {                                                  \
      if (!TRANS) {                                                                                   \
        const int r_ = wn0 + j * 32 + l32;                                                            \
        bf_[j] = *reinterpret_cast<const bf16x8*>(bs + r_ * BK + swz(r_, (kk_) * 2 + kg) * 8);        \
      } else {                                                                                        \
        const bf16_t* col_ = bs + ((kk_) * 16 + kg * 8) * S::B_LD + wn0 + j * 32 + l32;               \
        _Pragma("unroll") for (int e = 0; e < 8; ++e) bf_[j][e] = col_[e * S::B_LD];                  \
      }                                                                                               \
    }                                                                                                 \
  }
#define FLEXCO_MFMAS(af_, bf_)                                                                        \
  {                                                                                                   \
    _Pragma("unroll") for (int i = 0; i < MT; ++i)                                                    \
      _Pragma("unroll") for (int j = 0; j < NT; ++j)                                                  \
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af_[i], bf_[j], acc[i][j], 0, 0, 0);      \
  }

  // Software pipeline over k-steps of 64 with two LDS buffers and two sets of staging registers,
  // so that a tile's global loads have two whole steps to arrive:
  //   step kt, first half : MFMAs of k-slices 0, 1 of tile kt (LDS buffer kt & 1)
  //   step kt, middle     : the staging set that holds tile kt + 1 (loaded in the middle of step
  //                         kt - 2) is written to the other LDS buffer and reloaded with tile kt + 3
  //   step kt, second half: MFMAs of k-slices 2, 3 - they run while the LDS writes drain
  //   one barrier at the end of the step: the other buffer is complete, this one is free.
  // The other buffer was last read in step kt - 1, which every wavefront left through that
  // step's barrier, so the mid-step writes race with nothing.  Past the last tile the indices are
  // clamped: the extra loads and writes repeat tile nk - 1 and are never read.
#define FLEXCO_STEP(kt_, ra_, rb_)                                                                    \
  {                                                                                                   \
    const int buf = (kt_) & 1;                                                                        \
    const bf16_t* as = As + buf * S::A_ELEMS;                                                         \
    const bf16_t* bs = Bs + buf * S::B_ELEMS;                                                         \
    bf16x8 af[MT], bfr[NT], af2[MT], bfr2[NT];                                                        \
    FLEXCO_LOAD_FRAGS(0, af, bfr)                                                                     \
    FLEXCO_MFMAS(af, bfr)                                                                             \
    FLEXCO_LOAD_FRAGS(1, af, bfr)                                                                     \
    FLEXCO_MFMAS(af, bfr)                                                                             \
    __builtin_amdgcn_sched_barrier(0);                                                                \
    FLEXCO_LOAD_FRAGS(2, af2, bfr2)                                                                   \
    FLEXCO_STORE_TILES(buf ^ 1, ra_, rb_)                                                             \
    FLEXCO_LOAD_TILES(kbeg + min((kt_) + 3, nk - 1) * BK, ra_, rb_)                                   \
    __builtin_amdgcn_sched_barrier(0);                                                                \
    FLEXCO_MFMAS(af2, bfr2)                                                                           \
    FLEXCO_LOAD_FRAGS(3, af, bfr)                                                                     \
    FLEXCO_MFMAS(af, bfr)                                                                             \
    __builtin_amdgcn_sched_barrier(0);                                                                \
    __syncthreads();                                                                                  \
  }
  FLEXCO_LOAD_TILES(kbeg, sa0, sb0)
  FLEXCO_STORE_TILES(0, sa0, sb0)
  __syncthreads();
  FLEXCO_LOAD_TILES(kbeg + min(1, nk - 1) * BK, sa0, sb0)
  FLEXCO_LOAD_TILES(kbeg + min(2, nk - 1) * BK, sa1, sb1)
  int kt = 0;
  for (; kt + 1 < nk; kt += 2) {
    FLEXCO_STEP(kt, sa0, sb0)
    FLEXCO_STEP(kt + 1, sa1, sb1)
  }
  if (kt < nk) FLEXCO_STEP(kt, sa0, sb0)

  // ---- rank-r extension: C += A2 W2^T (forward form; the entry whose column range holds this
  // block) or C += sum_e A2_e W2_e (input-gradient form; every entry).  This is the LoRA bypass
  // network (Sec. 4.1) folded into the base projection as extra k-steps of 16, operands read
  // straight from global memory (they are [rows, r] / [r, cols] matrices of a few KB per tile).
  for (int e = 0; e < (blockIdx.y == 0 ? ext.n : 0); ++e) {
    if (!TRANS && !(n0 >= ext.col0[e] && n0 < ext.col1[e])) continue;
    const bf16_t* A2 = ext.A2[e];
    const bf16_t* W2 = ext.W2[e];
    for (int k2 = 0; k2 < ext.r; k2 += 16) {
      bf16x8 af[MT], bfr[NT];
#pragma unroll
      for (int i = 0; i < MT; ++i) {
        const int r = min(m0 + wm0 + i * 32 + l32, M - 1);
        af[i] = *reinterpret_cast<const bf16x8*>(A2 + (size_t)r * ext.r + k2 + kg * 8);
      }
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        if (!TRANS) {
          const int c = min(n0 + wn0 + j * 32 + l32, ext.col1[e] - 1) - ext.col0[e];
          bfr[j] = *reinterpret_cast<const bf16x8*>(W2 + (size_t)c * ext.ldw2[e] + k2 + kg * 8);
        } else {
          const int c = min(n0 + wn0 + j * 32 + l32, N - 1);
#pragma unroll
          for (int q = 0; q < 8; ++q) bfr[j][q] = W2[(size_t)(k2 + kg * 8 + q) * ext.ldw2[e] + c];
        }
      }
#pragma unroll
      for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
  }

  // ---- epilogue: D[i][j], j = lane % 32, i = 8 (r / 4) + 4 (lane / 32) + r % 4 ---------------
  if (part) {
    float* P = part + (size_t)blockIdx.y * M * N;
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const int col = n0 + wn0 + j * 32 + l32;
        if (col >= N) continue;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = m0 + wm0 + i * 32 + 8 * (r >> 2) + 4 * kg + (r & 3);
          if (row < M) P[(size_t)row * N + col] = acc[i][j][r];
        }
      }
    return;
  }
#pragma unroll
  for (int i = 0; i < MT; ++i) {
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int col = n0 + wn0 + j * 32 + l32;
      if (col >= N) continue;
      const float bv = bias ? (float)bias[col] : 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm0 + i * 32 + 8 * (r >> 2) + 4 * kg + (r & 3);
        if (row >= M) continue;
        float v = acc[i][j][r] + bv;
        if (res) v += (float)res[(size_t)row * ldr + col];
        C[(size_t)row * ldc + col] = (bf16_t)v;
      }
    }
  }
}

// C[row, col] = sum over splits of part[split][row][col] (+ bias) (+ residual), fixed order
__global__ __launch_bounds__(256) void gemm_splitk_reduce_kernel(const float* __restrict__ part, int splits,
                                                                 bf16_t* __restrict__ C, const bf16_t* __restrict__ bias,
                                                                 const bf16_t* __restrict__ res, int M, int N,
                                                                 size_t ldc, size_t ldr) {
  const size_t idx = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (idx >= (size_t)M * N) return;
  const int row = (int)(idx / N), col = (int)(idx % N);     // N % 8 == 0: the 4 elements share a row
  f32x4 v = *reinterpret_cast<const f32x4*>(part + idx);
  for (int sp = 1; sp < splits; ++sp) {
    const f32x4 w = *reinterpret_cast<const f32x4*>(part + (size_t)sp * M * N + idx);
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] += w[j];
  }
  bf16x4 o;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    float x = v[j];
    if (bias) x += (float)bias[col + j];
    if (res) x += (float)res[(size_t)row * ldr + col + j];
    o[j] = (bf16_t)x;
  }
  *reinterpret_cast<bf16x4*>(C + (size_t)row * ldc + col) = o;
}

template <int BM, int BN, bool TRANS>
int32_t launch_cfg(const void* A, const void* W, void* C, const void* bias, const void* res, int M, int N, int K,
                   size_t lda, size_t ldw, size_t ldc, size_t ldr, const GemmExt& ext, hipStream_t s,
                   float* part = nullptr, int splits = 1) {
  using S = Smem<BM, BN, TRANS>;
  auto kern = gemm_bf16_kernel<BM, BN, TRANS>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)S::BYTES);
    if (e != hipSuccess) return fail(FLEXCO_EHIP, "hipFuncSetAttribute(gemm): %s", hipGetErrorString(e));
    attr_set = true;
  }
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n, splits), dim3(256), S::BYTES, s, (const bf16_t*)A, (const bf16_t*)W,
                     (bf16_t*)C, (const bf16_t*)bias, (const bf16_t*)res, M, N, K, lda, ldw, ldc, ldr, tiles_m, tiles_n,
                     ext, splits > 1 ? part : nullptr, K / splits);
  if (splits > 1) {
    const size_t quads = ((size_t)M * N + 3) / 4;
    hipLaunchKernelGGL(gemm_splitk_reduce_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, s, part, splits,
                       (bf16_t*)C, (const bf16_t*)bias, (const bf16_t*)res, M, N, ldc, ldr);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(FLEXCO_EHIP, "launch of gemm_bf16 failed: %s", hipGetErrorString(e));
  return FLEXCO_OK;
}

}  // namespace

static bool ext_fits(const GemmExt& ext, bool trans_w, int BN) {
  if (ext.n == 0) return true;
  if (ext.r % 16 != 0) return false;
  if (trans_w) return true;
  for (int e = 0; e < ext.n; ++e)
    if (ext.col0[e] % BN != 0 || ext.col1[e] % BN != 0) return false;   // one entry per block
  return true;
}

// Largest split count <= want that cuts K into whole 64-wide steps and fits the partial buffer.
static int pick_splits(int M, int N, int K, int tiles, size_t part_elems) {
  if (part_elems == 0 || tiles >= 384) return 1;
  int best = 1;
  for (int sp = 2; sp <= 16; ++sp) {
    if (K % (sp * BK) != 0 || K / sp < 4 * BK) continue;
    if ((size_t)sp * M * N > part_elems) break;
    best = sp;
    if (tiles * sp >= 512) break;
  }
  return best;
}

int32_t launch_gemm_mfma(const void* A, const void* W, void* C, const void* bias, const void* residual, int M, int N,
                         int K, size_t lda, size_t ldw, size_t ldc, size_t ldr, bool trans_w, const GemmExt* ext_in,
                         hipStream_t s, float* part, size_t part_elems) {
  // shapes the tiled kernel covers: K in whole 64-wide steps, 16-byte aligned rows
  if (K % BK != 0 || lda % 8 != 0 || ldw % 8 != 0 || N % 8 != 0) return FLEXCO_EUNSUPPORTED;
  GemmExt ext;
  if (ext_in) ext = *ext_in; else ext.n = 0;
  if (trans_w) {
    if (!ext_fits(ext, true, 128)) return FLEXCO_EUNSUPPORTED;
    // few row tiles (a finetune window) and a long contraction: cut K across blocks so that the
    // weight stream is spread over the whole chip; partial sums are reduced in split order
    const int tiles = ((M + 127) / 128) * ((N + 127) / 128);
    const int sp = part ? pick_splits(M, N, K, tiles, part_elems) : 1;
    return launch_cfg<128, 128, true>(A, W, C, bias, residual, M, N, K, lda, ldw, ldc, ldr, ext, s, part, sp);
  }
  const long big_tiles = (long)((M + 255) / 256) * ((N + 255) / 256);
  if (big_tiles >= 192 && ext_fits(ext, false, 256))
    return launch_cfg<256, 256, false>(A, W, C, bias, residual, M, N, K, lda, ldw, ldc, ldr, ext, s);
  if (!ext_fits(ext, false, 128)) return FLEXCO_EUNSUPPORTED;
  return launch_cfg<128, 128, false>(A, W, C, bias, residual, M, N, K, lda, ldw, ldc, ldr, ext, s);
}

}  // namespace flexco

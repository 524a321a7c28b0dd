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
//            the window's rows only; on the matrix cores (u, t as bf16, the rows of x / dy through
//            transposing LDS reads), 64 output columns per block, rows shared out over its 4
//            wavefronts, fixed-order LDS reduction; a plain FMA kernel covers unaligned shapes.
#include <cstring>
#include "flexco_internal.h"
#include "device_types.h"

namespace flexco {

namespace {

// One block per 16 rows and matrix; K is cut across the block's wavefronts (blockDim.x / 64, at most 16),
// whose partial sums are added in wavefront order through LDS.
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
      if (a.relu >> z & 1) v = fmaxf(v, 0.f);
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
  if (a.relu >> z & 1) v = fmaxf(v, 0.f);
  if (a.out_f32[z] && out_ok && orow >= a.f32_lo && orow < a.f32_hi)
    a.out_f32[z][(size_t)(orow - a.f32_lo) * a.r + rank] = v;
  if (a.out_ext[z]) a.out_ext[z][o] = (bf16_t)(out_ok ? v * a.scale : 0.f);
}

__global__ __launch_bounds__(256) void relu_bwd_mask_kernel(const float* __restrict__ u, float* __restrict__ t,
                                                            bf16_t* __restrict__ t_ext, size_t count) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= count) return;
  const float v = u[i] > 0.f ? t[i] : 0.f;
  t[i] = v;
  if (t_ext) t_ext[i] = (bf16_t)v;
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

// The same products on the matrix cores: G^T[j, i] += scale sum_m U[m, j] X[m, i] with
// v_mfma_f32_16x16x32_bf16, D rows = 16 ranks, D columns = 16 of the block's 64 columns i, k = 32 rows m.
//   * U^T (bf16, row pitch padded) is staged in LDS once per 256-row chunk; a lane reads its 8
//     consecutive m of one rank with one ds_read_b128.
//   * X: wavefront w owns rows 64 w .. + 64 of the chunk, two [32 rows][64 columns] tiles that go from
//     global memory straight into its own LDS buffers; the operand (8 consecutive rows of one column)
//     comes from two transposing reads (ds_read_b64_tr_b16).  32-byte column pairs are XOR-swizzled
//     with row % 4 so that the four rows of a read sit on different banks.
//   * the four wavefronts' sums are added in wavefront order through LDS.
typedef short s16x4 __attribute__((ext_vector_type(4)));
#define FLEXCO_GP(p) ((const __attribute__((address_space(1))) void*)(p))
#define FLEXCO_LP(p) ((__attribute__((address_space(3))) void*)(p))
#define FLEXCO_LDS __attribute__((address_space(3)))
__device__ inline bf16x8 tr_pair(const bf16_t* a, const bf16_t* b) {
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((FLEXCO_LDS s16x4*)a);
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((FLEXCO_LDS s16x4*)b);
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

template <int RT>   // rank tiles of 16
__global__ __launch_bounds__(256) void lora_outer_mfma_kernel(LoraOuterArgs a) {
  constexpr int UP = 264;                                                   // row pitch of U^T in elements
  __shared__ __attribute__((aligned(1024))) bf16_t xt[4][2][32 * 64];       // per wavefront: two X tiles
  __shared__ __attribute__((aligned(16))) bf16_t ut[RT * 16 * UP];          // U^T of the chunk, [rank][row]
  __shared__ __attribute__((aligned(16))) float red[3][RT][4][64][4];       // sums of wavefronts 1..3
  const int e = blockIdx.y;
  const int n = a.n, r = a.r, n_long = a.n_long[e];
  const int i0 = blockIdx.x * 64;
  if (i0 >= n_long) return;   // entries of one launch differ in width
  const bf16_t* __restrict__ X = a.X[e];
  const float* __restrict__ U = a.U[e];
  float* __restrict__ G = a.G[e];
  const size_t ldx = a.ldx[e], g_i = a.g_i[e], g_j = a.g_j[e];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int c = lane & 15, g = lane >> 4;

  f32x4 acc[RT][4];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int cg = 0; cg < 4; ++cg) acc[rt][cg] = f32x4{0.f, 0.f, 0.f, 0.f};

  // tile loads: instruction q fills rows 8 q .. + 8 of a tile; lane -> row 8 q + lane / 8, physical chunk
  // lane % 8; it fetches the logical chunk that belongs there (pair = physical pair ^ row % 4)
  const int d_row = lane >> 3, d_pc = lane & 7;
  const int d_lch = ((((d_pc >> 1) ^ (d_row & 3)) << 1) | (d_pc & 1));
  const int d_col = min(i0 + d_lch * 8, n_long - 8);
  // transposing reads: source lane c of group g -> row 8 g + c / 4 (+ 4), columns 16 cg + 4 (c % 4) ..
  const int t_row = 8 * g + (c >> 2);
  const int t_k = (c >> 2) & 3;

  // a wavefront's two tiles of the chunk that starts at row mb0 (its own LDS buffers: nobody else reads them)
  auto load_tiles = [&](int mb0) {
    const int mw0 = mb0 + 64 * wave;
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int row = min(mw0 + 32 * st + 8 * q + d_row, n - 1);   // rows past n meet zero U
        __builtin_amdgcn_global_load_lds(FLEXCO_GP(X + (size_t)row * ldx + d_col), FLEXCO_LP(&xt[wave][st][q * 512]), 16, 0, 0);
      }
  };
  load_tiles(0);
  for (int mb = 0; mb < n; mb += 256) {
    __syncthreads();   // the previous chunk's reads of ut are done
    if (r == RT * 16) {
      // full rank tiles: the chunk of U is one contiguous run of floats; 4 RT 16-byte loads per thread,
      // all in flight before the first is converted
      f32x4 uv[4 * RT];
#pragma unroll
      for (int k = 0; k < 4 * RT; ++k) {
        const int idx4 = tid + 256 * k, m = idx4 / (4 * RT);
        uv[k] = mb + m < n ? *reinterpret_cast<const f32x4*>(U + ((size_t)mb * r + (size_t)idx4 * 4)) : f32x4{0.f, 0.f, 0.f, 0.f};
      }
#pragma unroll
      for (int k = 0; k < 4 * RT; ++k) {
        const int idx4 = tid + 256 * k, m = idx4 / (4 * RT), j = 4 * (idx4 % (4 * RT));
#pragma unroll
        for (int q = 0; q < 4; ++q) ut[(j + q) * UP + m] = (bf16_t)uv[k][q];
      }
    } else {
      for (int idx = tid; idx < 256 * RT * 16; idx += 256) {
        const int m = idx / (RT * 16), j = idx % (RT * 16);
        ut[j * UP + m] = (bf16_t)((mb + m < n && j < r) ? U[(size_t)(mb + m) * r + j] : 0.f);
      }
    }
    const int mw = mb + 64 * wave;
    __syncthreads();   // ut is complete; the barrier's wait also covers this wavefront's tile loads
    if (mw < n) {
#pragma unroll
      for (int st = 0; st < 2; ++st) {
        bf16x8 af[RT];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
          af[rt] = *reinterpret_cast<const bf16x8*>(&ut[(rt * 16 + c) * UP + 64 * wave + 32 * st + 8 * g]);
#pragma unroll
        for (int cg = 0; cg < 4; ++cg) {
          const bf16_t* p = &xt[wave][st][t_row * 64 + ((cg ^ t_k) << 4) + 4 * (c & 3)];
          const bf16x8 xf = tr_pair(p, p + 4 * 64);
#pragma unroll
          for (int rt = 0; rt < RT; ++rt) acc[rt][cg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[rt], xf, acc[rt][cg], 0, 0, 0);
        }
      }
    }
    // the next chunk's tiles travel while the other wavefronts finish and U is staged: this wavefront's reads
    // of its buffers have returned (the products above consumed them)
    if (mb + 256 < n) {
      asm volatile("" ::: "memory");
      load_tiles(mb + 256);
    }
  }
  // lane (column c of group cg, g) holds ranks 16 rt + 4 g .. + 4
  if (wave > 0) {
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
      for (int cg = 0; cg < 4; ++cg) *reinterpret_cast<f32x4*>(red[wave - 1][rt][cg][lane]) = acc[rt][cg];
  }
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
      for (int cg = 0; cg < 4; ++cg) {
        const int i = i0 + 16 * cg + c;
        if (i >= n_long) continue;
        f32x4 v = acc[rt][cg];
#pragma unroll
        for (int w = 0; w < 3; ++w) {
          const f32x4 o = *reinterpret_cast<const f32x4*>(red[w][rt][cg][lane]);
#pragma unroll
          for (int q = 0; q < 4; ++q) v[q] += o[q];
        }
        float gv[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int j = rt * 16 + 4 * g + q;
          gv[q] = j < r ? G[(size_t)i * g_i + (size_t)j * g_j] : 0.f;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int j = rt * 16 + 4 * g + q;
          if (j < r) G[(size_t)i * g_i + (size_t)j * g_j] = gv[q] + a.scale * v[q];
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
  // K is cut into whole groups of 4 MFMA steps (128 columns), first over the wavefronts of a block (at
  // most 16), and - long contractions with scratch at hand - over several blocks per row tile,
  // so that more than rows / 16 CUs pull the operands in
  int kmin = a.K[0], kmax = a.K[0];
  for (int z = 1; z < n_mats; ++z) { kmin = a.K[z] < kmin ? a.K[z] : kmin; kmax = a.K[z] > kmax ? a.K[z] : kmax; }
  a.ksplit = 1;
  if (a.part && n_mats <= a.part_slots && kmin == kmax && kmax >= 8192)
    for (int sp = LORA_SHRINK_SPLITS; sp > 1; --sp)
      if (kmax % (128 * sp) == 0 && kmax / sp >= 1024) { a.ksplit = sp; break; }
  // wavefronts of a block: a count (not only powers of two) that cuts every K into whole groups, taken for the fewest
  // load rounds of the longest contraction (a round is up to 256 columns per wavefront), the smallest such count
  int nw = 1, best_rounds = (kmax / a.ksplit + 255) / 256;
  for (int c = 2; c <= 16; ++c) {
    bool fits = true;
    for (int z = 0; z < n_mats; ++z) fits = fits && a.K[z] % (128 * c * a.ksplit) == 0;
    const int rounds = (kmax / (c * a.ksplit) + 255) / 256;
    if (fits && rounds < best_rounds) { nw = c; best_rounds = rounds; }
  }
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

int32_t launch_relu_bwd_mask(const float* u, float* t, void* t_ext, size_t count, hipStream_t s) {
  if (count == 0) return FLEXCO_OK;
  hipLaunchKernelGGL(relu_bwd_mask_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, s, u, t, (bf16_t*)t_ext, count);
  return post("relu_bwd_mask");
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
  bool tiles_ok = a.r <= 64;     // whole 16-byte column chunks, rows and base pointers 16-byte aligned
  for (int e = 0; e < a.count; ++e) {
    mx = a.n_long[e] > mx ? a.n_long[e] : mx;
    tiles_ok = tiles_ok && a.n_long[e] % 8 == 0 && a.n_long[e] >= 8 && a.ldx[e] % 8 == 0 && aligned16(a.X[e]) && aligned16(a.U[e]);
  }
  const dim3 grid((mx + 63) / 64, a.count);
  if (tiles_ok) {
    switch ((a.r + 15) / 16) {
      case 1: hipLaunchKernelGGL(lora_outer_mfma_kernel<1>, grid, dim3(256), 0, s, a); break;
      case 2: hipLaunchKernelGGL(lora_outer_mfma_kernel<2>, grid, dim3(256), 0, s, a); break;
      case 3: hipLaunchKernelGGL(lora_outer_mfma_kernel<3>, grid, dim3(256), 0, s, a); break;
      default: hipLaunchKernelGGL(lora_outer_mfma_kernel<4>, grid, dim3(256), 0, s, a); break;
    }
    return post("lora_outer");
  }
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

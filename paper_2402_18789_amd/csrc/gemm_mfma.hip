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
// Tiling: block tile BM x BN, 256 threads = 4 wavefronts in a 2 x 2 grid, each owning
// (BM/2) x (BN/2) as 32 x 32 MFMA tiles with fp32 accumulators.
//   * Forward form: operand tiles go from global memory straight into LDS
//     (global_load_lds_dwordx4: one wavefront instruction fills 1 KB; lane l lands at
//     base + 16 l), no staging registers and no LDS write instructions.  LDS is a ring of stages
//     (four of 32 KB for the 128 tile, two of 64 KB for the 256 tile) whose loads are in flight
//     while another stage is multiplied; the per-stage barrier carries no memory fence, the wait
//     in front of it names exactly the loads that must have landed.  Rows are XOR-swizzled in 16-byte chunks (applied to the
//     global address a lane fetches) so that the ds_read_b128 operand fetches of 16 consecutive
//     rows hit 64 distinct banks.
//   * Input-gradient form: the same ring; the W tile is [64][BN] (k-major as in memory), loaded
//     the same way, and an MFMA operand (8 consecutive k of one column) comes from two
//     transposing LDS reads (ds_read_b64_tr_b16).
// Work-group ids are remapped so that ids that land on the same XCD (id mod 8) work on
// neighbouring tiles, M fastest: the W tile they share stays in that XCD's L2.
#include <algorithm>
#include <cstring>
#include "flexco_internal.h"
#include "device_types.h"

namespace flexco {

namespace {

constexpr int BK = 64;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
#define FLEXCO_LDS __attribute__((address_space(3)))

#define FLEXCO_GP(p) ((const __attribute__((address_space(1))) void*)(p))
#define FLEXCO_LP(p) ((__attribute__((address_space(3))) void*)(p))

__device__ inline int swz(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

template <int BM, int BN, bool TRANS, bool GLU = false, int NSTAGES = 0>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(const bf16_t* __restrict__ A, const bf16_t* __restrict__ W,
                                                        bf16_t* __restrict__ C, const bf16_t* __restrict__ bias,
                                                        const bf16_t* __restrict__ res, int M, int N, int K,
                                                        size_t lda, size_t ldw, size_t ldc, size_t ldr, int tiles_m,
                                                        int tiles_n, GemmExt ext, float* __restrict__ part,
                                                        int k_chunk, GemmGlu glu) {
  constexpr int WM = BM / 2, WN = BN / 2, MT = WM / 32, NT = WN / 32;

  // ---- work-group id -> tile, XCD-aware ------------------------------------------------
  int lid = blockIdx.x;
  const int nblk = gridDim.x;
  if ((nblk & 7) == 0) lid = (blockIdx.x & 7) * (nblk >> 3) + (blockIdx.x >> 3);
  const int tm = lid % tiles_m, tn = lid / tiles_m;
  const int m0 = tm * BM, n0 = tn * BN;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wavefront-uniform: LDS bases of the tile loads stay scalar
  const int wm0 = (wave >> 1) * WM, wn0 = (wave & 1) * WN;

  f32x16 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // split-K: blockIdx.y owns k in [kbeg, kbeg + k_chunk) and writes fp32 partial sums to `part`
  const int kbeg = blockIdx.y * k_chunk;
  const int l32 = lane & 31, kg = lane >> 5;

  // The W fragment is the MFMA's first operand: a lane then holds, for ONE output row (lane % 32), runs
  // of 4 consecutive output columns, so the epilogue moves 8 bytes per lane and instruction.
  // (the pipelines are macros on purpose: register arrays captured by lambdas were left in
  // scratch memory)
#define FLEXCO_MFMAS(af_, bf_)                                                                        \
  {                                                                                                   \
    _Pragma("unroll") for (int i = 0; i < MT; ++i)                                                    \
      _Pragma("unroll") for (int j = 0; j < NT; ++j)                                                  \
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf_[j], af_[i], acc[i][j], 0, 0, 0);      \
  }

  // ===================== operand tiles: global memory -> LDS directly ==========================
  // A ring of stages of 64 k-columns; a stage holds the A tile [BM][64] and the W tile ([BN][64]
  // in the forward form, [64][BN] in the input-gradient form), A first.  The 128-row forward
  // tiles use four stages (32 KB each at 128 columns, 40 KB - all of the LDS - at 192): up to
  // three in flight or waiting while one is multiplied.
  // The 256-row tiles use two stages (64 KB at 256 columns, 56 KB at 192): half as many barriers, and a stage's buffer is
  // handed to the loads of the stage after next as soon as its last fragments are in registers
  // (measured equal at T = 1024 and 4-7 % faster than four 32 KB stages at T >= 2048).  The
  // input-gradient form uses two stages of 32 KB, so that two blocks share a CU (its grids are
  // K-split into more blocks than CUs).  The stages are separate arrays, not one indexed
  // buffer: the compiler then sees that loads in flight target an array no ds_read of that
  // moment touches, and inserts no wait of its own.
  // NSTAGES = 2 for a 128-row forward tile: two such blocks share a CU.  With more tiles than CUs that is 15-30 %
  // faster than one four-stage block per CU in two rounds (one block's waits are the other's products); with one
  // tile per CU the four stages win.
  constexpr int NST = NSTAGES ? NSTAGES : (TRANS ? 2 : ((BM + BN) * BK * 2 * 4 <= 160 * 1024 ? 4 : 2));   // stages in the ring
  constexpr int SL = BK / 16;                                       // MFMA k-slices per stage
  constexpr int PA = BM / 32, PB = BN / 32;                         // 1 KB load instructions per wavefront and stage
  constexpr int ST_ELEMS = (BM + BN) * BK;
  static_assert(!TRANS || BN == 128 || BN == 256, "the input-gradient form's W tile swizzle assumes 256- or 512-byte rows");
  __shared__ __attribute__((aligned(1024))) bf16_t ring0[ST_ELEMS];
  __shared__ __attribute__((aligned(1024))) bf16_t ring1[ST_ELEMS];
  __shared__ __attribute__((aligned(1024))) bf16_t ring2[NST == 4 ? ST_ELEMS : 8];
  __shared__ __attribute__((aligned(1024))) bf16_t ring3[NST == 4 ? ST_ELEMS : 8];
  // [rows][64] tiles (128-byte rows): chunk c of row r is stored at chunk c ^ ((r >> 1) & 7) (the
  // variant measured fastest for the ds_read_b128 operand fetches: 85 % of the LDS peak).
  // [64][BN] W tile of the input-gradient form (256- or 512-byte rows, read by transposing LDS reads of
  // 4 consecutive rows x 64 bytes per pass): chunk c of row r is stored at chunk c ^ (4 (r & 3)),
  // which puts the four rows of a pass on the four 64-byte quarters of the banks (the exchange stays
  // inside a 256-byte half of a 512-byte row).
#define FLEXCO_KEY(r_) (((r_) >> 1) & 7)
  // Load instruction p of wavefront w fills 1 KB = rows 8 (4 p + w) .. + 8 of a [rows][64] tile (rows
  // TR (4 p + w) .. + TR of the [64][BN] tile, TR = 512 / BN); lane l lands at base + 16 l, so it fetches from
  // global memory the logical chunk that belongs at its physical chunk.  The keys do not depend on p.
  const int d_row = lane >> 3;
  const int d_c = (lane & 7) ^ FLEXCO_KEY(wave * 8 + d_row);
  constexpr int TCH = BN / 8, TR = 64 / TCH;      // 16-byte chunks of a W-tile row, rows per load instruction
  const int t_row = lane / TCH;
  const int t_c = (lane % TCH) ^ (((wave * TR + t_row) & 3) << 2);
  const bf16_t* ga[PA];
  const bf16_t* gw[PB];
#pragma unroll
  for (int p = 0; p < PA; ++p)
    ga[p] = A + (size_t)min(m0 + (p * 4 + wave) * 8 + d_row, M - 1) * lda + kbeg + d_c * 8;
#pragma unroll
  for (int p = 0; p < PB; ++p) {
    if (GLU) {
      // W-tile rows alternate between the two halves of W in runs of 16: rows 32 f .. + 16 are gate rows
      // (act columns tile + 16 f .. + 16), rows 32 f + 16 .. + 16 the up rows of the same columns, so that
      // a lane's accumulators of one fragment hold gate and up of the same 4 + 4 act columns
      const int rr = (p * 4 + wave) * 8 + d_row;
      const int ac = glu.col0 + tn * (BN / 2) + (rr >> 5) * 16 + (rr & 15);
      gw[p] = W + ((size_t)((rr >> 4) & 1) * glu.F + min(ac, glu.F - 1)) * ldw + kbeg + d_c * 8;
    } else if (!TRANS) {
      gw[p] = W + (size_t)min(n0 + (p * 4 + wave) * 8 + d_row, N - 1) * ldw + kbeg + d_c * 8;
    } else {
      int col = n0 + t_c * 8;
      if (col >= N) col = 0;   // masked at the store
      gw[p] = W + (size_t)(kbeg + (p * 4 + wave) * TR + t_row) * ldw + col;
    }
  }
  const int ns = k_chunk / BK;                   // stages of this block

  // stage index past the end: clamped, the loads repeat the last stage into a free buffer
#define FLEXCO_DMA(ring_, s_)                                                                         \
  {                                                                                                   \
    const int koff_ = min((s_), ns - 1) * BK;                                                         \
    _Pragma("unroll") for (int p = 0; p < PA; ++p)                                                    \
      __builtin_amdgcn_global_load_lds(FLEXCO_GP(ga[p] + koff_),                                      \
                                       FLEXCO_LP(ring_ + (p * 4 + wave) * 512), 16, 0, 0);            \
    _Pragma("unroll") for (int p = 0; p < PB; ++p)                                                    \
      __builtin_amdgcn_global_load_lds(FLEXCO_GP(gw[p] + (TRANS ? (size_t)koff_ * ldw : (size_t)koff_)), \
                                       FLEXCO_LP(ring_ + BM * BK + (p * 4 + wave) * 512), 16, 0, 0);  \
  }
  // Operand fragments of W in the input-gradient form come from transposing LDS reads
  // (ds_read_b64_tr_b16): within a group of 16 lanes, lane s hands in the address of 4 consecutive
  // columns, 4 (s % 4) .., of row s / 4, and lane i receives column i of those 4 rows - i.e. 4
  // consecutive k for one column, the MFMA operand order.  Group g of the wavefront covers columns
  // 16 (g % 2) .. + 16 and the k-half g / 2; two reads (rows 0..3 and 4..7) make the 8 k of a fragment.
  const int tr_k = 8 * (lane >> 5) + ((lane & 15) >> 2);
  const int tr_n = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  const int tr_sw = ((lane & 15) >> 2) << 2;     // 4 (row & 3): the fragment's rows are tr_k + multiples of 4
#define FLEXCO_FRAGS(ring_, kk_, af_, bf_)                                                            \
  {                                                                                                   \
    _Pragma("unroll") for (int i = 0; i < MT; ++i) {                                                  \
      const int r_ = wm0 + i * 32 + l32;                                                              \
      af_[i] = *reinterpret_cast<const bf16x8*>(ring_ + r_ * BK + (((kk_) * 2 + kg) ^ FLEXCO_KEY(r_)) * 8); \
    }                                                                                                 \
    _Pragma("unroll") for (int j = 0; j < NT; ++j) {                                                  \
      if (!TRANS) {                                                                                   \
        const int r_ = wn0 + j * 32 + l32;                                                            \
        bf_[j] = *reinterpret_cast<const bf16x8*>(ring_ + (BM + r_) * BK + (((kk_) * 2 + kg) ^ FLEXCO_KEY(r_)) * 8); \
      } else {                                                                                        \
        const int col_ = wn0 + j * 32 + tr_n;                                                         \
        const bf16_t* blk_ = ring_ + BM * BK + ((kk_) * 16 + tr_k) * BN + (((col_ >> 3) ^ tr_sw) * 8) + (col_ & 7); \
        const s16x4 lo_ = __builtin_amdgcn_ds_read_tr16_b64_v4i16((FLEXCO_LDS s16x4*)blk_);           \
        const s16x4 hi_ = __builtin_amdgcn_ds_read_tr16_b64_v4i16((FLEXCO_LDS s16x4*)(blk_ + 4 * BN)); \
        bf_[j] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo_, hi_, 0, 1, 2, 3, 4, 5, 6, 7)); \
      }                                                                                               \
    }                                                                                                 \
  }
  // Barrier without the memory fences of __syncthreads (those would drain every load in
  // flight): the wait before it covers exactly the stage that has to be complete, and the
  // empty asm statements keep the compiler from moving LDS accesses across it.
#define FLEXCO_WAIT_BARRIER(imm_)                                                                     \
  {                                                                                                   \
    __builtin_amdgcn_sched_barrier(0);                                                                \
    __builtin_amdgcn_s_waitcnt(imm_);                                                                 \
    asm volatile("" ::: "memory");                                                                    \
    __builtin_amdgcn_s_barrier();                                                                     \
    asm volatile("" ::: "memory");                                                                    \
    __builtin_amdgcn_sched_barrier(0);                                                                \
  }
  // Stage s (ring buffer cur_) enters with its slice-0 fragments in set 0.  Slices alternate
  // between the two fragment sets, each fetched one slice ahead.  In the last slice:
  //   wait until this wavefront's loads of stage s + 1 have landed (with four stages those of
  //   stage s + 2 may stay in flight), barrier -> stage s + 1 is complete for everyone, and
  //   everyone has the last fragments of stage s in registers; start the loads of the stage
  //   that takes over the freed buffer; fetch slice 0 of stage s + 1; then the last slice's
  //   MFMAs cover those latencies.
#define FLEXCO_STAGE(cur_, nxt_, free_, s_)                                                           \
  {                                                                                                   \
    _Pragma("unroll") for (int kk = 0; kk < SL; kk += 2) {                                            \
      FLEXCO_FRAGS(cur_, kk + 1, af1, bf1)                                                            \
      FLEXCO_MFMAS(af0, bf0)                                                                          \
      FLEXCO_ORDER_READS_FIRST                                                                        \
      __builtin_amdgcn_sched_barrier(0);                                                              \
      if (kk + 2 < SL) {                                                                              \
        FLEXCO_FRAGS(cur_, kk + 2, af0, bf0)                                                          \
        FLEXCO_MFMAS(af1, bf1)                                                                        \
        FLEXCO_ORDER_READS_FIRST                                                                      \
      } else {                                                                                        \
        FLEXCO_WAIT_BARRIER(WAIT_NEXT_STAGE)                                                          \
        FLEXCO_DMA(free_, (s_) + AHEAD)                                                               \
        FLEXCO_FRAGS(nxt_, 0, af0, bf0)                                                               \
        FLEXCO_MFMAS(af1, bf1)                                                                        \
        FLEXCO_ORDER_LOADS_READS_FIRST                                                                \
      }                                                                                               \
      __builtin_amdgcn_sched_barrier(0);                                                              \
    }                                                                                                 \
  }
  // Instruction order inside a slice, imposed on the scheduler (it otherwise sinks the fragment
  // reads behind the MFMAs, right in front of their first use): LDS reads - or global loads and
  // LDS reads - ahead of each MFMA until they are used up, the remaining MFMAs after.
  // Masks: 0x008 MFMA, 0x020 VMEM read, 0x100 DS read.
  constexpr int NRD = MT + (TRANS ? 2 * NT : NT);                  // LDS reads of one slice
  constexpr int NMF = MT * NT;                                     // its MFMAs
  constexpr int NLD = PA + PB;                                     // loads of one stage
#define FLEXCO_ORDER_READS_FIRST                                                                      \
  {                                                                                                   \
    _Pragma("unroll") for (int q = 0; q < NMF; ++q) {                                                 \
      __builtin_amdgcn_sched_group_barrier(0x100, (NRD + NMF - 1) / NMF, 0);                          \
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                              \
    }                                                                                                 \
  }
#define FLEXCO_ORDER_LOADS_READS_FIRST                                                                \
  {                                                                                                   \
    _Pragma("unroll") for (int q = 0; q < NMF; ++q) {                                                 \
      __builtin_amdgcn_sched_group_barrier(0x020, (NLD + NMF - 1) / NMF, 0);                          \
      __builtin_amdgcn_sched_group_barrier(0x100, (NRD + NMF - 1) / NMF, 0);                          \
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                              \
    }                                                                                                 \
  }
  // s_waitcnt immediates: vmcnt in bits 3:0 and 15:14, expcnt 6:4 and lgkmcnt 11:8 left at
  // their maxima (no wait)
#define FLEXCO_VMCNT(n_) (0x0F70 | ((n_) & 15) | (((n_) >> 4) << 14))
  // before a stage's barrier: the next stage has landed; with four stages one more may stay in flight
  constexpr int WAIT_NEXT_STAGE = NST == 4 ? FLEXCO_VMCNT(NLD) : FLEXCO_VMCNT(0);
  // the buffer freed at stage s's barrier held stage s - 1 (four stages) or stage s itself (two)
  constexpr int AHEAD = NST == 4 ? 3 : 2;
  // ---- operands of the rank-r extension's first step and the residual / bias of the epilogue, fetched ahead of the
  // main loop (128-row tiles: the registers are there; their round trips - one or two per block, all blocks
  // ending together - otherwise lie open at the end of the launch) --------------------------------------------
  // forward form: an entry covers a column range whose ends are multiples of 32, so each 32-column
  // fragment of the tile belongs to at most one entry; fragments outside this entry multiply zeros
#define FLEXCO_EXT_SKIPS(e_) (!TRANS && !GLU && (n0 + BN <= ext.col0[e_] || n0 >= ext.col1[e_]))
#define FLEXCO_EXT_LOAD(e_, k2_, af_, bfr_)                                                           \
  {                                                                                                   \
    const bf16_t* A2_ = ext.A2[e_];                                                                   \
    const bf16_t* W2_ = ext.W2[e_];                                                                   \
    _Pragma("unroll") for (int i = 0; i < MT; ++i) {                                                  \
      const int r_ = min(m0 + wm0 + i * 32 + l32, M - 1);                                             \
      af_[i] = *reinterpret_cast<const bf16x8*>(A2_ + (size_t)r_ * ext.r + (k2_) + kg * 8);           \
    }                                                                                                 \
    _Pragma("unroll") for (int j = 0; j < NT; ++j) {                                                  \
      if (GLU) {                                                                                      \
        /* this lane's W-tile row is a gate or an up row: column of the [gate | up] range the entries address */ \
        const int ac_ = glu.col0 + tn * (BN / 2) + ((wn0 + j * 32) >> 1) + (l32 & 15);                \
        const int lc_ = (l32 >> 4) * glu.F + ac_;                                                     \
        if (ac_ < glu.F && lc_ >= ext.col0[e_] && lc_ < ext.col1[e_]) {                               \
          bfr_[j] = *reinterpret_cast<const bf16x8*>(W2_ + (size_t)(lc_ - ext.col0[e_]) * ext.ldw2[e_] + (k2_) + kg * 8); \
        } else {                                                                                      \
          _Pragma("unroll") for (int q = 0; q < 8; ++q) bfr_[j][q] = (bf16_t)0.f;                     \
        }                                                                                             \
      } else if (!TRANS) {                                                                            \
        const int cj_ = n0 + wn0 + j * 32;                                                            \
        if (cj_ >= ext.col0[e_] && cj_ < ext.col1[e_]) {                                              \
          const int c_ = min(cj_ + l32, ext.col1[e_] - 1) - ext.col0[e_];                             \
          bfr_[j] = *reinterpret_cast<const bf16x8*>(W2_ + (size_t)c_ * ext.ldw2[e_] + (k2_) + kg * 8); \
        } else {                                                                                      \
          _Pragma("unroll") for (int q = 0; q < 8; ++q) bfr_[j][q] = (bf16_t)0.f;                     \
        }                                                                                             \
      } else {                                                                                        \
        const int c_ = min(n0 + wn0 + j * 32 + l32, N - 1);                                           \
        _Pragma("unroll") for (int q = 0; q < 8; ++q) bfr_[j][q] = W2_[(size_t)((k2_) + kg * 8 + q) * ext.ldw2[e_] + c_]; \
      }                                                                                               \
    }                                                                                                 \
  }
  constexpr bool PF = MT * NT <= 4;
  int e_first = -1;
  bf16x8 paf[PF ? MT : 1], pbf[PF ? NT : 1];
  if constexpr (PF) {
    if (blockIdx.y == 0) {
      for (int e = 0; e < ext.n; ++e)
        if (!FLEXCO_EXT_SKIPS(e)) { e_first = e; break; }
      if (e_first >= 0) FLEXCO_EXT_LOAD(e_first, 0, paf, pbf)
    }
  }
  // residual and bias in the layout the epilogue stores in: 8 lanes x 8 columns per row, 8 rows per instruction,
  // 32 rows x 64 columns per group of two fragments
  constexpr int NG = (NT + 1) / 2;
  constexpr bool PF_RES = !GLU && MT * NT <= 6;
  bf16x8 rpre[PF_RES ? MT : 1][PF_RES ? NG : 1][4];
  bf16x8 bpre[PF_RES ? NG : 1];
  if constexpr (PF_RES) if (!part) {
#pragma unroll
    for (int j0 = 0; j0 < NT; j0 += 2) {
      const int col = n0 + wn0 + j0 * 32 + (lane & 7) * 8;
      const bool col_ok = (lane & 7) * 8 < ((j0 + 1 < NT) ? 64 : 32) && col < N;
      if (bias && col_ok) bpre[j0 / 2] = *reinterpret_cast<const bf16x8*>(bias + col);
      if (res) {
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
          for (int p = 0; p < 4; ++p) {
            const int row = m0 + wm0 + i * 32 + p * 8 + (lane >> 3);
            if (col_ok && row < M) rpre[i][j0 / 2][p] = *reinterpret_cast<const bf16x8*>(res + (size_t)row * ldr + col);
          }
      }
    }
  }
  bf16x8 af0[MT], bf0[NT], af1[MT], bf1[NT];
  if constexpr (NST == 4) {
    FLEXCO_DMA(ring0, 0)
    FLEXCO_DMA(ring1, 1)
    FLEXCO_DMA(ring2, 2)
    FLEXCO_WAIT_BARRIER(FLEXCO_VMCNT(2 * NLD))
    FLEXCO_FRAGS(ring0, 0, af0, bf0)
    int st = 0;
    for (; st + 3 < ns; st += 4) {
      FLEXCO_STAGE(ring0, ring1, ring3, st)
      FLEXCO_STAGE(ring1, ring2, ring0, st + 1)
      FLEXCO_STAGE(ring2, ring3, ring1, st + 2)
      FLEXCO_STAGE(ring3, ring0, ring2, st + 3)
    }
    if (st < ns) FLEXCO_STAGE(ring0, ring1, ring3, st)
    if (st + 1 < ns) FLEXCO_STAGE(ring1, ring2, ring0, st + 1)
    if (st + 2 < ns) FLEXCO_STAGE(ring2, ring3, ring1, st + 2)
  } else {
    FLEXCO_DMA(ring0, 0)
    FLEXCO_DMA(ring1, 1)
    FLEXCO_WAIT_BARRIER(FLEXCO_VMCNT(NLD))
    FLEXCO_FRAGS(ring0, 0, af0, bf0)
    int st = 0;
    for (; st + 1 < ns; st += 2) {
      FLEXCO_STAGE(ring0, ring1, ring0, st)
      FLEXCO_STAGE(ring1, ring0, ring1, st + 1)
    }
    if (st < ns) FLEXCO_STAGE(ring0, ring1, ring0, st)
  }
  __builtin_amdgcn_s_waitcnt(FLEXCO_VMCNT(0));   // nothing may land in LDS after the block ends

  // ---- rank-r extension: C += A2 W2^T (forward form; the entry whose column range holds this
  // block) or C += sum_e A2_e W2_e (input-gradient form; every entry).  This is the LoRA bypass
  // network (Sec. 4.1) folded into the base projection as extra k-steps of 16, operands read
  // straight from global memory (they are [rows, r] / [r, cols] matrices of a few KB per tile).
  // The first step's operands were fetched before the main loop where the tile leaves registers for them.
  for (int e = 0; e < (blockIdx.y == 0 ? ext.n : 0); ++e) {
    if (FLEXCO_EXT_SKIPS(e)) continue;
    for (int k2 = 0; k2 < ext.r; k2 += 16) {
      bf16x8 af[MT], bfr[NT];
      bool have = false;
      if constexpr (PF) {
        if (e == e_first && k2 == 0) {
#pragma unroll
          for (int i = 0; i < MT; ++i) af[i] = paf[i];
#pragma unroll
          for (int j = 0; j < NT; ++j) bfr[j] = pbf[j];
          have = true;
        }
      }
      if (!have) FLEXCO_EXT_LOAD(e, k2, af, bfr)
#pragma unroll
      for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
    }
  }
  // ---- epilogue: register 4 q + e of acc[i][j] is row lane % 32, column 8 q + 4 (lane / 32) + e of
  // the 32 x 32 block.  Stored as they lie, an instruction would touch 32 rows with 16 (bf16) or 32 (fp32)
  // bytes each; measured, such stores run at about 1 TB/s where whole 128-byte lines reach 3.5.  So every
  // wavefront turns its rows through a piece of the (now free) ring that only it touches: accumulators in,
  // 16 bytes per lane along a row out, 128 contiguous bytes or more per row and instruction. ------------
  __syncthreads();   // every wavefront is done with the ring, and (after its own wait above) its loads have landed
  if (GLU) {
    // registers 4 qq + e (gate) and 8 + 4 qq + e (up) of acc[i][j] belong to act column 8 qq + 4 (lane / 32) + e
    // of the fragment's 16
    constexpr int AW = WN / 2;                       // act columns of a wavefront's tile
    constexpr int PITCH = AW + 8;                    // staged row in elements (16 bytes of padding)
    constexpr int LPR = AW / 8;                      // lanes that cover a row, 16 bytes each
    constexpr int LPRP = LPR <= 4 ? 4 : 8;           // ... rounded up to a power of two (the others idle)
    constexpr int RPI = 64 / LPRP;                   // rows per instruction
    static_assert(4 * 32 * PITCH <= ST_ELEMS, "the staged act rows of four wavefronts fit a stage");
    bf16_t* stg = ring0 + wave * 32 * PITCH;
    const int ac_end = min(glu.col0 + N / 2, glu.F);
    const int ac_w = glu.col0 + tn * (BN / 2) + (wn0 >> 1);      // first act column of this wavefront
    const int rl = lane / LPRP, cl = (lane % LPRP) * 8;
    const bool lane_on = (lane % LPRP) < LPR && ac_w + cl < ac_end;   // F % 8 == 0: a run of 8 is in or out as a whole
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      const int rb = m0 + wm0 + i * 32;
      const bool band_saves = glu.save_gate && rb + 32 > glu.save_row0 && rb < glu.save_row0 + glu.save_rows;   // uniform
#pragma unroll
      for (int what = 0; what < 3; ++what) {         // 0: act, 1: gate, 2: up (the last two for finetune rows only)
        if (what > 0 && !band_saves) break;
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
          for (int qq = 0; qq < 2; ++qq) {
            bf16x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              // gate and up pass through the storage type first (they are what the backward pass reads back)
              const bf16_t gs = (bf16_t)acc[i][j][4 * qq + e], us = (bf16_t)acc[i][j][8 + 4 * qq + e];
              const float gv = (float)gs, uv = (float)us;
              // (reciprocal instruction, 1 ulp, instead of the ten-instruction IEEE division: the tile's 64 K sigmoids are on
              // the critical path of a launch whose blocks all end together)
              o[e] = what == 0 ? (bf16_t)(gv * __builtin_amdgcn_rcpf(1.0f + __expf(-gv)) * uv) : (what == 1 ? gs : us);
            }
            *reinterpret_cast<bf16x4*>(stg + l32 * PITCH + j * 16 + 8 * qq + 4 * kg) = o;
          }
        bf16_t* dst = what == 0 ? C : (what == 1 ? glu.save_gate : glu.save_up);
        const size_t ldd = what == 0 ? ldc : glu.ld_save;
#pragma unroll
        for (int p = 0; p < 32 / RPI; ++p) {
          const int r = p * RPI + rl, row = rb + r;
          const int drow = what == 0 ? row : row - glu.save_row0;
          const bool ok = lane_on && row < M && (what == 0 || (drow >= 0 && drow < glu.save_rows));
          if (ok) *reinterpret_cast<bf16x8*>(dst + (size_t)drow * ldd + ac_w + cl) = *reinterpret_cast<const bf16x8*>(stg + r * PITCH + cl);
        }
        if (MT * NT > 4) __builtin_amdgcn_sched_barrier(0);
      }
    }
    return;
  }
  // fp32 staging (what is added to the accumulators - bias, residual - is added in fp32 before the one rounding):
  // 32 rows x 64 columns at a time (two fragments; one if the wavefront's tile has an odd one left), rows 272 bytes apart
  constexpr int PITCH32 = 64 + 4;
  static_assert(2 * 32 * PITCH32 * 4 <= ST_ELEMS * 2, "the staged rows of two wavefronts fit a stage");
  float* stg = reinterpret_cast<float*>(wave < 2 ? ring0 : ring1) + (wave & 1) * 32 * PITCH32;
  float* P = part ? part + (size_t)blockIdx.y * M * N : nullptr;
#pragma unroll
  for (int i = 0; i < MT; ++i) {
    const int rb = m0 + wm0 + i * 32;
#pragma unroll
    for (int j0 = 0; j0 < NT; j0 += 2) {
      const int nj = (j0 + 1 < NT) ? 2 : 1;          // fragments in this group (compile-time after unrolling)
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        if (jj >= nj) break;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          f32x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = acc[i][j0 + jj][4 * q + e];
          *reinterpret_cast<f32x4*>(stg + l32 * PITCH32 + jj * 32 + 8 * q + 4 * kg) = v;
        }
      }
      const int cb = n0 + wn0 + j0 * 32;             // first column of the group
      if (part) {
        // 16 lanes x 4 columns per row, 4 rows per instruction
        const int rl = lane >> 4, cl = (lane & 15) * 4;
#pragma unroll
        for (int p = 0; p < 8; ++p) {
          const int r = p * 4 + rl, row = rb + r, col = cb + cl;
          if (cl < nj * 32 && row < M && col < N)    // N % 8 == 0: a run of 4 is inside or outside as a whole
            *reinterpret_cast<f32x4*>(P + (size_t)row * N + col) = *reinterpret_cast<const f32x4*>(stg + r * PITCH32 + cl);
        }
      } else {
        // 8 lanes x 8 columns per row, 8 rows per instruction
        const int rl = lane >> 3, cl = (lane & 7) * 8;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          const int r = p * 8 + rl, row = rb + r, col = cb + cl;
          if (cl < nj * 32 && row < M && col < N) {  // N % 8 == 0: a run of 8 is inside or outside as a whole
            const f32x4 lo = *reinterpret_cast<const f32x4*>(stg + r * PITCH32 + cl);
            const f32x4 hi = *reinterpret_cast<const f32x4*>(stg + r * PITCH32 + cl + 4);
            float v[8];
#pragma unroll
            for (int e = 0; e < 4; ++e) { v[e] = lo[e]; v[4 + e] = hi[e]; }
            if (bias) {
              bf16x8 b8;
              if constexpr (PF_RES) b8 = bpre[j0 / 2]; else b8 = *reinterpret_cast<const bf16x8*>(bias + col);
#pragma unroll
              for (int e = 0; e < 8; ++e) v[e] += (float)b8[e];
            }
            if (res) {
              bf16x8 r8;
              if constexpr (PF_RES) r8 = rpre[i][j0 / 2][p]; else r8 = *reinterpret_cast<const bf16x8*>(res + (size_t)row * ldr + col);
#pragma unroll
              for (int e = 0; e < 8; ++e) v[e] += (float)r8[e];
            }
            bf16x8 o;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (bf16_t)v[e];
            *reinterpret_cast<bf16x8*>(C + (size_t)row * ldc + col) = o;
          }
        }
      }
      // (keeps the scheduler from gathering the stores of the whole tile up front, which costs more
      // registers than the large tile has left)
      if (MT * NT > 4) __builtin_amdgcn_sched_barrier(0);
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

template <int BM, int BN, bool TRANS, bool GLU = false, int NSTAGES = 0>
int32_t launch_cfg(const void* A, const void* W, void* C, const void* bias, const void* res, int M, int N, int K,
                   size_t lda, size_t ldw, size_t ldc, size_t ldr, const GemmExt& ext, hipStream_t s,
                   int timer_id, float* part = nullptr, int splits = 1, bool first_of_call = true,
                   const GemmGlu* glu_in = nullptr, bool skip_reduce = false) {
  auto kern = gemm_bf16_kernel<BM, BN, TRANS, GLU, NSTAGES>;   // all LDS is static
  GemmGlu glu;
  if (glu_in) glu = *glu_in; else memset(&glu, 0, sizeof(glu));
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  // while the class's timer runs, the kernels carry an event pair of their own (start and end stamps of
  // the dispatch itself)
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (timer_id >= 0) (void)kernel_timer_pair(timer_id, &e0, &e1, first_of_call);
  // (the plain launch when no pair is due: it is the form a stream capture records)
#define FLEXCO_LAUNCH_TIMED(kern_, grid_, ...)                                                        \
  {                                                                                                   \
    if (e0) hipExtLaunchKernelGGL(kern_, grid_, dim3(256), 0, s, e0, e1, 0, __VA_ARGS__);             \
    else hipLaunchKernelGGL(kern_, grid_, dim3(256), 0, s, __VA_ARGS__);                              \
  }
  FLEXCO_LAUNCH_TIMED(kern, dim3(tiles_m * tiles_n, splits), (const bf16_t*)A, (const bf16_t*)W, (bf16_t*)C,
                      (const bf16_t*)bias, (const bf16_t*)res, M, N, K, lda, ldw, ldc, ldr, tiles_m, tiles_n, ext,
                      splits > 1 ? part : nullptr, K / splits, glu)
  if (splits > 1 && !skip_reduce) {
    const size_t quads = ((size_t)M * N + 3) / 4;
    e0 = e1 = nullptr;
    if (timer_id >= 0) (void)kernel_timer_pair(timer_id, &e0, &e1, false);
    FLEXCO_LAUNCH_TIMED(gemm_splitk_reduce_kernel, dim3((unsigned)((quads + 255) / 256)), part, splits, (bf16_t*)C,
                        (const bf16_t*)bias, (const bf16_t*)res, M, N, ldc, ldr)
  }
#undef FLEXCO_LAUNCH_TIMED
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(FLEXCO_EHIP, "launch of gemm_bf16 failed: %s", hipGetErrorString(e));
  return FLEXCO_OK;
}

}  // namespace

static bool ext_fits(const GemmExt& ext, bool trans_w, int N) {
  if (ext.n == 0) return true;
  if (ext.r % 16 != 0) return false;
  if (trans_w) return true;
  for (int e = 0; e < ext.n; ++e)      // whole 32-column fragments per entry
    if (ext.col0[e] % 32 != 0 || (ext.col1[e] % 32 != 0 && ext.col1[e] != N)) return false;
  return true;
}

// The entries of `ext` restricted to output columns [c0, c1), in the coordinates of a GEMM over those
// columns only.
static GemmExt sub_ext(const GemmExt& ext, int c0, int c1) {
  GemmExt o;
  o.n = 0;
  o.r = ext.r;
  for (int e = 0; e < ext.n; ++e) {
    const int lo = std::max(ext.col0[e], c0), hi = std::min(ext.col1[e], c1);
    if (lo >= hi) continue;
    o.col0[o.n] = lo - c0;
    o.col1[o.n] = hi - c0;
    o.A2[o.n] = ext.A2[e];
    o.W2[o.n] = ext.W2[e] + (size_t)(lo - ext.col0[e]) * ext.ldw2[e];
    o.ldw2[o.n] = ext.ldw2[e];
    ++o.n;
  }
  return o;
}

// Largest split count <= want that cuts K into whole 64-wide steps and fits the partial buffer.
// Split count for a grid of `tiles` output tiles: the one with the least estimated time,
// rounds of `want` resident blocks (resident blocks per CU x 256) times the k-range of a block, plus a
// small charge per split for the partial sums it writes and the reduction reads back.  Splits cut K
// into whole 64-wide stages, at least four per block, and must fit the partial buffer.
static int pick_splits(int M, int N, int K, int tiles, size_t part_elems, int want) {
  if (part_elems == 0) return 1;
  int best = 1;
  double best_cost = 1e30;
  for (int sp = 1; sp <= 16; ++sp) {
    if (K % (sp * BK) != 0 || (sp > 1 && K / sp < 4 * BK)) continue;
    if (sp > 1 && (size_t)sp * M * N > part_elems) break;
    const int rounds = (tiles * sp + want - 1) / want;
    const double cost = (double)rounds / sp + 0.015 * (sp - 1);   // (0.02 took 7 splits where 8 fill the last CU slots: 3 % slower)
    if (cost < best_cost - 1e-12) { best_cost = cost; best = sp; }
  }
  return best;
}

// Rates of the input-gradient form's two tile shapes with every block slot taken, PFLOP/s (fitted to twelve products of
// 512 to 1536 rows at the 8B, 14B and 32B shapes; with them the estimate picks the faster shape in each).
constexpr double TRANS_RATE_128 = 0.94, TRANS_RATE_256 = 1.05;

// Tile shapes of a forward-form product by estimated time.  A launch runs in rounds of one block per CU; a
// round costs the tile's area over the rate its kernel sustains with the chip full (measured, relative:
// 256 x 256 tiles 1.24, 256 x 192 1.09, 128 x 192 1.0, 128 x 128 0.875).  Candidates: columns [0, 256 a) in
// 256-wide tiles and the rest in ONE of the three narrower shapes, as two launches (a partial last round of
// wide tiles is what the narrower ones avoid); a = 0 is a single shape for the whole matrix.
struct GemmPlan {
  int a256;    // number of 256-wide column tiles
  int rest;    // shape of the remaining columns: 0 = 128 x 128, 1 = 128 x 192, 2 = 256 x 192
};
static GemmPlan plan_forward(int M, int N) {
  const int CU = 256;
  auto rounds = [&](long tiles) { return (double)((tiles + CU - 1) / CU); };
  const long tm256 = (M + 255) / 256, tm128 = (M + 127) / 128;
  const double c256 = 256.0 * 256 / 1.24;
  const long tm_rest[3] = {tm128, tm128, tm256};
  const int bn_rest[3] = {128, 192, 192};
  const double c_rest[3] = {128.0 * 128 / 0.875, 128.0 * 192 / 1.0, 256.0 * 192 / 1.09};
  GemmPlan best{0, 0};
  double best_t = 1e300;
  const int n256 = (N + 255) / 256;
  for (int a = n256; a >= 0; --a) {
    const int rest = N - 256 * a;                   // columns left for the narrower tiles
    if (rest < 0 && a != n256) continue;
    const double t_a = a ? rounds(tm256 * a) * c256 : 0.0;
    if (rest <= 0) {
      if (t_a < best_t - 1e-9) { best_t = t_a; best = GemmPlan{a, 0}; }
      continue;
    }
    for (int sh = 2; sh >= 0; --sh) {
      const double t = t_a + rounds(tm_rest[sh] * ((rest + bn_rest[sh] - 1) / bn_rest[sh])) * c_rest[sh];
      if (t < best_t - 1e-9) { best_t = t; best = GemmPlan{a, sh}; }
    }
  }
  return best;
}

// What launch_gemm_mfma does for a shape: one or two launches, each a tile shape over a range of output columns,
// possibly with K cut across blocks.  A pure function of the arguments (host arithmetic only).
GemmLaunchPlan plan_gemm_mfma(int M, int N, int K, bool trans_w, size_t part_elems) {
  GemmLaunchPlan pl;
  pl.n = 0;
  auto add = [&](int bm, int bn, int cols, int splits, int stages) {
    pl.step[pl.n++] = GemmLaunchStep{bm, bn, cols, splits, stages};
  };
  if (trans_w) {
    // few row tiles (a finetune window) and a long contraction: cut K across blocks so that the
    // weight stream is spread over the whole chip; partial sums are reduced in split order
    // (256 x 128 tiles, one block per CU, were measured slower than two co-resident 128 x 128 blocks)
    const int tiles = ((M + 127) / 128) * ((N + 127) / 128);
    const int sp = part_elems ? pick_splits(M, N, K, tiles, part_elems, 512) : 1;
    // A window of 512 rows or more has the rows for 256 x 256 tiles, one block per CU, which sustain more per CU
    // than two 128 x 128 blocks; few of them cover the output, so the choice goes by estimated time: whole rounds of
    // the grid over the block slots x the k-range of a block x the area a CU holds at a time over the rate of the
    // shape, plus the partial sums' way out and back in (1 us per million of them).
    int sp256 = 0;
    if (M >= 512) {
      auto est_us = [&](long blocks, int slots, int splits, double area, double pflops) {
        const double rounds = (double)((blocks * splits + slots - 1) / slots);
        return rounds * (K / splits) * area * 2.0 * 256 / (pflops * 1e9) + (splits > 1 ? (double)splits * M * N * 1e-6 : 0.0);
      };
      double best = 0.97 * est_us(tiles, 512, sp, 2.0 * 128 * 128, TRANS_RATE_128);   // (the large tile has to win clearly)
      const long tiles256 = (long)((M + 255) / 256) * ((N + 255) / 256);
      for (int c = 1; c <= 16; ++c) {
        if (K % (c * BK) != 0 || (c > 1 && (K / c < 8 * BK || (size_t)c * M * N > part_elems))) continue;
        const double t = est_us(tiles256, 256, c, 256.0 * 256, TRANS_RATE_256);
        if (t < best - 1e-9) { best = t; sp256 = c; }
      }
    }
    if (sp256) add(256, 256, N, sp256, 2);
    else add(128, 128, N, sp, 2);
    return pl;
  }
  // A batch of few tokens (decode-only iterations) has one or two row tiles and far fewer output tiles
  // than CUs, and its time is the weight stream's: cut K across blocks so that the whole chip pulls on it.
  if (part_elems && M <= 256) {
    const int tiles = ((M + 127) / 128) * ((N + 127) / 128);
    const int sp = tiles < 192 ? pick_splits(M, N, K, tiles, part_elems, 256) : 1;
    if (sp > 1) {
      add(128, 128, N, sp, 4);
      return pl;
    }
  }
  const GemmPlan fp = plan_forward(M, N);
  const int n1 = std::min(N, 256 * fp.a256);
  if (n1 > 0) add(256, 256, n1, 1, 2);
  if (n1 < N) {
    // more 128 x 128 tiles than CUs: two-stage blocks, two per CU (the planner takes 128 x 192 tiles for single
    // rounds only)
    const long t128 = (long)((M + 127) / 128) * ((N - n1 + 127) / 128);
    if (fp.rest == 0) add(128, 128, N - n1, 1, t128 > 256 ? 2 : 4);
    else if (fp.rest == 1) add(128, 192, N - n1, 1, 4);
    else add(256, 192, N - n1, 1, 2);
  }
  return pl;
}

int32_t launch_gemm_mfma(const void* A, const void* W, void* C, const void* bias, const void* residual, int M, int N,
                         int K, size_t lda, size_t ldw, size_t ldc, size_t ldr, bool trans_w, const GemmExt* ext_in,
                         hipStream_t s, float* part, size_t part_elems, int timer_id, int* splits_out) {
  if (splits_out) *splits_out = 1;
  // shapes the tiled kernel covers: K in whole 64-wide steps, 16-byte aligned rows
  // (and 8-byte aligned runs of 4 output columns in C, bias and residual)
  if (K % BK != 0 || lda % 8 != 0 || ldw % 8 != 0 || N % 8 != 0 || ldc % 4 != 0 || (residual && ldr % 4 != 0) ||
      ((uintptr_t)C & 7) || ((uintptr_t)bias & 7) || ((uintptr_t)residual & 7))
    return FLEXCO_EUNSUPPORTED;
  GemmExt ext;
  if (ext_in) ext = *ext_in; else ext.n = 0;
  if (!ext_fits(ext, trans_w, N)) return FLEXCO_EUNSUPPORTED;
  const GemmLaunchPlan pl = plan_gemm_mfma(M, N, K, trans_w, part ? part_elems : 0);
  if (trans_w) {
    const GemmLaunchStep& st = pl.step[0];
    // splits_out: the caller's next kernel adds the partial sums itself (part[split][M][N], in split order) and
    // the reduction launch is left out; bias and residual are then not applied
    const bool leave = splits_out && st.splits > 1 && !bias && !residual;
    if (leave) *splits_out = st.splits;
    if (st.bm == 256)
      return launch_cfg<256, 256, true>(A, W, C, bias, residual, M, N, K, lda, ldw, ldc, ldr, ext, s, timer_id, part, st.splits,
                                        true, nullptr, leave);
    return launch_cfg<128, 128, true>(A, W, C, bias, residual, M, N, K, lda, ldw, ldc, ldr, ext, s, timer_id, part, st.splits, true,
                                      nullptr, leave);
  }
  if (pl.step[0].splits > 1)
    return launch_cfg<128, 128, false>(A, W, C, bias, residual, M, N, K, lda, ldw, ldc, ldr, ext, s, timer_id, part,
                                       pl.step[0].splits);
  int c0 = 0;
  for (int i = 0; i < pl.n; ++i) {
    const GemmLaunchStep& st = pl.step[i];
    const bf16_t* W1 = (const bf16_t*)W + (size_t)c0 * ldw;
    bf16_t* C1 = (bf16_t*)C + c0;
    const bf16_t* b1 = bias ? (const bf16_t*)bias + c0 : nullptr;
    const bf16_t* r1 = residual ? (const bf16_t*)residual + c0 : nullptr;
    const GemmExt e1 = sub_ext(ext, c0, c0 + st.cols);
    const bool first = i == 0;
    int32_t rc;
    if (st.bm == 256 && st.bn == 256)
      rc = launch_cfg<256, 256, false>(A, W1, C1, b1, r1, M, st.cols, K, lda, ldw, ldc, ldr, e1, s, timer_id, nullptr, 1, first);
    else if (st.bm == 256)
      rc = launch_cfg<256, 192, false>(A, W1, C1, b1, r1, M, st.cols, K, lda, ldw, ldc, ldr, e1, s, timer_id, nullptr, 1, first);
    else if (st.bn == 192)
      rc = launch_cfg<128, 192, false>(A, W1, C1, b1, r1, M, st.cols, K, lda, ldw, ldc, ldr, e1, s, timer_id, nullptr, 1, first);
    else if (st.stages == 2)
      rc = launch_cfg<128, 128, false, false, 2>(A, W1, C1, b1, r1, M, st.cols, K, lda, ldw, ldc, ldr, e1, s, timer_id, nullptr, 1, first);
    else
      rc = launch_cfg<128, 128, false>(A, W1, C1, b1, r1, M, st.cols, K, lda, ldw, ldc, ldr, e1, s, timer_id, nullptr, 1, first);
    if (rc) return rc;
    c0 += st.cols;
  }
  return FLEXCO_OK;
}

// Gated form: the planner of the forward form over the 2F interleaved columns; a tile of BN W-rows covers
// BN / 2 act columns.
int32_t launch_gemm_glu_mfma(const void* A, const void* W, void* act, int M, int F, int K, size_t lda, size_t ldw,
                             size_t ld_act, const GemmExt* ext_in, void* save_gate, void* save_up, int save_row0,
                             int save_rows, size_t ld_save, hipStream_t s, int timer_id) {
  if (K % BK != 0 || lda % 8 != 0 || ldw % 8 != 0 || F % 8 != 0 || ld_act % 4 != 0 || ld_save % 4 != 0 ||
      ((uintptr_t)act & 7) || ((uintptr_t)save_gate & 7) || ((uintptr_t)save_up & 7))
    return FLEXCO_EUNSUPPORTED;
  GemmExt ext;
  if (ext_in) ext = *ext_in; else ext.n = 0;
  if (ext.n > 0 && ext.r % 16 != 0) return FLEXCO_EUNSUPPORTED;
  GemmGlu glu;
  glu.F = F; glu.col0 = 0; glu.save_gate = (bf16_t*)save_gate; glu.save_up = (bf16_t*)save_up;
  glu.save_row0 = save_row0; glu.save_rows = save_gate ? save_rows : 0; glu.ld_save = ld_save;
  const int N = 2 * F;
  const GemmLaunchPlan pl = plan_gemm_mfma(M, N, K, false, 0);
  int c0 = 0;                                       // interleaved columns done = 2 x the act columns done
  for (int i = 0; i < pl.n; ++i) {
    const GemmLaunchStep& st = pl.step[i];
    glu.col0 = c0 / 2;
    const bool first = i == 0;
    int32_t rc;
    if (st.bm == 256 && st.bn == 256)
      rc = launch_cfg<256, 256, false, true>(A, W, act, nullptr, nullptr, M, st.cols, K, lda, ldw, ld_act, 0, ext, s, timer_id,
                                             nullptr, 1, first, &glu);
    else if (st.bm == 256)
      rc = launch_cfg<256, 192, false, true>(A, W, act, nullptr, nullptr, M, st.cols, K, lda, ldw, ld_act, 0, ext, s, timer_id,
                                             nullptr, 1, first, &glu);
    else if (st.bn == 192)
      rc = launch_cfg<128, 192, false, true>(A, W, act, nullptr, nullptr, M, st.cols, K, lda, ldw, ld_act, 0, ext, s, timer_id,
                                             nullptr, 1, first, &glu);
    else if (st.stages == 2)
      rc = launch_cfg<128, 128, false, true, 2>(A, W, act, nullptr, nullptr, M, st.cols, K, lda, ldw, ld_act, 0, ext, s, timer_id,
                                                nullptr, 1, first, &glu);
    else
      rc = launch_cfg<128, 128, false, true>(A, W, act, nullptr, nullptr, M, st.cols, K, lda, ldw, ld_act, 0, ext, s, timer_id,
                                             nullptr, 1, first, &glu);
    if (rc) return rc;
    c0 += st.cols;
  }
  return FLEXCO_OK;
}

}  // namespace flexco

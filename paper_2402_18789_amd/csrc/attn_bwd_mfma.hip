// Attention backward of one token window on the matrix cores (Sec. 6.1, Alg. 2 Backward).
//
// Queries are the window's rows i at positions win_start + i; keys/values are the cached rows
// [0, l), l = win_start + win_len, read through the sequence's page list.  The softmax
// probabilities are recomputed from Q, K and the stored log-sum-exp (graph pruning keeps Q, K, V
// and rematerialises P).  With delta_i = sum_d dO_id O_id:
//     P_ij = exp(q_i . k_j / sqrt(d) - lse_i)           (j <= position of i)
//     dP_ij = dO_i . v_j ,   dS_ij = P_ij (dP_ij - delta_i)
//     dQ_i = sum_j dS_ij k_j / sqrt(d)                   -> kernel A, one block per 32 rows x head
//     dK_j = sum_i dS_ij q_i / sqrt(d),  dV_j = sum_i P_ij dO_i   summed over the window's rows
//            and over the query heads of the kv group     -> kernel B, one block per 64 keys x kv head
// Two kernels, each owning its outputs: no atomics, results do not depend on scheduling.  dK/dV are
// added into the KV-gradient accumulator rows [0, l) (Sec. 7).
//
// bf16, head_dim 128, page_size 16.  All products are v_mfma_f32_16x16x32_bf16.
//   * The tiles a block walks over (K and V pages in kernel A; Q and dO rows in kernel B) go from
//     global memory straight into LDS (global_load_lds_dwordx4, lane l lands at base + 16 l) in two
//     buffer sets: the loads of step i + 1 are in flight while step i is multiplied, one barrier
//     per step.
//   * Operands whose contracted index is contiguous in memory are fetched with ds_read_b128;
//     operands that must be read "across" rows (V and K^T in kernel A; Q^T, dO^T in kernel B) come
//     from transposing LDS reads (ds_read_b64_tr_b16: in a group of 16 lanes, lane s hands in the
//     address of 4 consecutive elements, 4 (s % 4) .., of row s / 4, and lane i receives element i
//     of each of those 4 rows).
//   * No padding: 16-byte chunks are XOR-swizzled (applied to the global address a lane fetches)
//     so that both access patterns are free of bank conflicts.
#include "flexco_internal.h"
#include "device_types.h"

namespace flexco {

namespace {

constexpr int D = 128, PS = 16;
constexpr int TILE16 = 16 * D;          // elements of 16 rows of 128
constexpr int VPAGE = D * PS;           // elements of one V page, [128 d][16 keys]
constexpr float LOG2E = 1.4426950408889634f;
typedef short s16x4 __attribute__((ext_vector_type(4)));
#define FLEXCO_GP(p) ((const __attribute__((address_space(1))) void*)(p))
#define FLEXCO_LP(p) ((__attribute__((address_space(3))) void*)(p))
#define FLEXCO_LDS __attribute__((address_space(3)))

struct BwdArgs {
  const bf16_t *q, *dout, *out;
  const float* lse;
  float* delta;       // [s, nq]: written by kernel A (row sums of dO (.) O), read by kernel B
  const bf16_t *kp, *vp;
  const int32_t* pages;
  bf16_t* dq;
  float *dk_accum, *dv_accum;
  int w0, s, l, nq, nkv;
  float scale, scale_log2;
};

// [rows][128] bf16 tiles (256-byte rows = sixteen 16-byte chunks): chunk cc of row r is stored at
// chunk cc ^ rsw(r), rsw(r) = 2 p(r) + r / 8 with the chunk pair p(r) = r for rows 0..7 and (r + 4) % 8 for
// rows 8..15.  What that serves (LDS: 64 banks of 4 bytes; measured on this chip):
//   * a transposing read (ds_read_b64_tr_b16, like ds_read_b64) is served 32 lanes per cycle, lanes 0..31 and
//     32..63: its 8 rows (0..7 or 8..15, 32 bytes = one chunk pair each) get 8 different chunk pairs;
//   * a ds_read_b128 is served 16 lanes per cycle, and not consecutive ones: lanes {0-3, 12-15, 20-23, 24-27},
//     {4-7, 8-11, 16-19, 28-31}, and the same plus 32.  With lane = 16 g + row reading logical chunk 4 dc + g,
//     a cycle holds rows {0-3, 12-15} at chunk X and rows {4-11} at chunk X ^ 1 (or the other way round): rows
//     0-3 and 12-15 own the same four chunk pairs, one chunk of each, so the 16 lanes cover 16 different chunks.
__device__ inline int rsw(int r) { return (((r + ((r >> 3) << 2)) & 7) << 1) | ((r >> 3) & 1); }

// wait for this wavefront's loads, then a barrier without memory fences (those would also drain
// loads issued after the wait); the empty asm statements keep LDS accesses on their side of it
#define FLEXCO_WAIT_ALL_BARRIER                  \
  {                                              \
    __builtin_amdgcn_s_waitcnt(0x0F70);          \
    asm volatile("" ::: "memory");               \
    __builtin_amdgcn_s_barrier();                \
    asm volatile("" ::: "memory");               \
  }

// 8 consecutive "row" values of one column as an MFMA operand: 4 rows at a and the next 4 at b
// (a, b already hold the lane's row, chunk and half-chunk)
__device__ inline bf16x8 tr_pair(const bf16_t* a, const bf16_t* b) {
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((FLEXCO_LDS s16x4*)a);
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((FLEXCO_LDS s16x4*)b);
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

// ---------------------------------------------------------------------------------------------
// kernel A: dQ.  grid (ceil(s / 32), nq), SP = 8 (or 4) wavefronts.  Wavefront w: rows [32 b + 16 (w % 2), + 16), and
// of the SP pages a step stages, pages 2 (w / 2) and 2 (w / 2) + 1; the SP / 2 key groups are added
// in a fixed order at the end.  (The grid has one block per CU or fewer and a step is a chain of
// dependent LDS reads and MFMAs: eight wavefronts halve the number of steps.)
// ---------------------------------------------------------------------------------------------
template <int SP>                                                // pages a step stages, one per wavefront
__global__ __launch_bounds__(64 * SP) void attn_bwd_dq_mfma_kernel(BwdArgs a) {
  __shared__ __attribute__((aligned(1024))) bf16_t kb0[SP * TILE16];
  __shared__ __attribute__((aligned(1024))) bf16_t kb1[SP * TILE16];
  __shared__ __attribute__((aligned(1024))) bf16_t vb0[SP * VPAGE];
  __shared__ __attribute__((aligned(1024))) bf16_t vb1[SP * VPAGE];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wavefront-uniform: LDS bases of the loads stay scalar
  const int c = lane & 15, g = lane >> 4;
  const int rt = wave & 1, kh = wave >> 1;
  // Work-group ids go round the 8 XCDs; the kv head is the id's fastest digit, so that (with 8 kv heads) every
  // block that reads a kv head's K / V pages runs on the same XCD and finds them in that XCD's L2 (the cached
  // rows of one kv head of a 4096-token sequence are 2 MB; all kv heads together would not fit one L2)
  const int group = a.nq / a.nkv;
  const int lid = blockIdx.y * gridDim.x + blockIdx.x;
  const int kvh = lid % a.nkv;
  const int h = kvh * group + (lid / a.nkv) % group;
  const int bx = lid / a.nq;                                     // row block
  const int i0 = bx * 32 + rt * 16;
  const int row_c = i0 + c;
  const bool row_ok = row_c < a.s;
  const int rcl = row_ok ? row_c : a.s - 1;
  const int pos_c = row_ok ? a.w0 + row_c : -1;
  const int wave_last_pos = a.w0 + min(i0 + 15, a.s - 1);      // may be < first key if the tile is empty
  const int blk_last_row = min(bx * 32 + 31, a.s - 1);
  const int np = (a.w0 + blk_last_row) / PS + 1;                 // pages visible to the block
  const int nit = (np + SP - 1) / SP;
  const int last_page = (a.l - 1) / PS, last_key = (a.l - 1) % PS;

  bf16x8 qf[4], dof[4];
  {
    const bf16_t* qr = a.q + ((size_t)rcl * a.nq + h) * D + g * 8;
    const bf16_t* dr = a.dout + ((size_t)rcl * a.nq + h) * D + g * 8;
#pragma unroll
    for (int dc = 0; dc < 4; ++dc) {
      qf[dc] = *reinterpret_cast<const bf16x8*>(qr + dc * 32);
      dof[dc] = *reinterpret_cast<const bf16x8*>(dr + dc * 32);
    }
  }
  const float lse2 = a.lse[(size_t)rcl * a.nq + h] * LOG2E;
  // delta_i = sum_d dO_id O_id of the wavefront's rows: the four lanes of a row hold 32 of its 128 d each
  float delta = 0.f;
  {
    const bf16_t* orow = a.out + ((size_t)rcl * a.nq + h) * D + g * 8;
#pragma unroll
    for (int dc = 0; dc < 4; ++dc) {
      const bf16x8 of = *reinterpret_cast<const bf16x8*>(orow + dc * 32);
#pragma unroll
      for (int q = 0; q < 8; ++q) delta += (float)dof[dc][q] * (float)of[q];
    }
    delta = sum_xor16(delta);
    delta = sum_xor32(delta);
    if (kh == 0 && g == 0 && row_ok) a.delta[(size_t)row_c * a.nq + h] = delta;   // for kernel B
  }

  f32x4 dq[8];
#pragma unroll
  for (int mt = 0; mt < 8; ++mt) dq[mt] = f32x4{0.f, 0.f, 0.f, 0.f};

  // ---- loads: wavefront w brings in page slot w of a step, K rows and V ---------------------
  // K: instruction q fills rows 4 q .. + 4 of the slot; lane -> row 4 q + lane / 16, physical chunk
  //    lane % 16.  Rows at or past l were never written: their address is moved to row l - 1, so
  //    that what lands is finite (those keys are masked, but 0 x NaN would still poison dQ).
  // V: a page is [128 d][16 keys] = 256 chunks; instruction q fills physical chunks 64 q .. + 64;
  //    physical chunk P holds logical chunk P ^ (8 if bit 4 of P): rows d and d + 8 of a
  //    transposing read then sit 128 bytes apart (mod 256).
  const int k_rin = lane >> 4, k_pc = lane & 15;
  const int v_lc = lane ^ (((lane >> 4) & 1) << 3);
  int page_nxt;
#define FLEXCO_ISSUE(kb_, vb_, it_, page_)                                                            \
  {                                                                                                   \
    const int slot_ = SP * (it_) + wave;                                                              \
    const size_t pb_ = ((size_t)(page_) * a.nkv + kvh);                                               \
    _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                                   \
      const int key_ = 4 * q + k_rin;                                                                 \
      const int keff_ = slot_ * PS + key_ < a.l ? key_ : last_key;                                    \
      const bf16_t* src_ = a.kp + (pb_ * PS + keff_) * (size_t)D + ((k_pc ^ rsw(key_)) * 8);          \
      __builtin_amdgcn_global_load_lds(FLEXCO_GP(src_), FLEXCO_LP(kb_ + wave * TILE16 + q * 4 * D), 16, 0, 0); \
    }                                                                                                 \
    _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                                   \
      const bf16_t* src_ = a.vp + pb_ * (size_t)VPAGE + (64 * q + v_lc) * 8;                          \
      __builtin_amdgcn_global_load_lds(FLEXCO_GP(src_), FLEXCO_LP(vb_ + wave * VPAGE + q * 512), 16, 0, 0); \
    }                                                                                                 \
  }

  // ---- per-lane offsets of the LDS reads -------------------------------------------------------
  // K rows as A operand of S^T = K Q^T: lane (key c, g) reads chunk 4 dc + g of row c
  const int krow_off = c * D;
  const int krow_sw = rsw(c);
  // transposing reads: source lane s = lane % 16 of group g
  const int s4 = c >> 2, sc = c & 3;
  // K^T as A operand of dQ^T += K^T dS^T: rows (keys) 4 g + s / 4 of a slot, columns 16 mt + 4 (s % 4)
  const int kt_row = 4 * g + s4;
  const int kt_base = kt_row * D + (sc & 1) * 4;
  const int kt_sw = rsw(kt_row), kt_hi = sc >> 1;
  // V as A operand of dP^T = V dO^T: rows d = 32 dc + 8 g + 4 hh + s / 4, keys 4 (s % 4) ..;
  // logical chunk 2 d + (s % 4) / 2, physical = logical ^ (8 if bit 3 of d, i.e. g odd)
  const int v_base = (((2 * (8 * g + s4) + (sc >> 1)) ^ ((g & 1) << 3)) * 8) + (sc & 1) * 4;

  // MASKED_ = false: the step's keys lie before every row's own position (the leading steps of a window on a long
  // prefix): no comparisons, no per-element branches
#define FLEXCO_DQ_COMPUTE(kb_, vb_, it_, MASKED_)                                                     \
  if (!(MASKED_) || (SP * (it_) + 2 * kh) * PS <= wave_last_pos) { /* else: nothing visible to these rows (uniform) */ \
    float ds[8];                                                                                      \
    _Pragma("unroll") for (int xx = 0; xx < 2; ++xx) {                                                \
      const bf16_t* kt_ = kb_ + (2 * kh + xx) * TILE16;                                               \
      const bf16_t* vt_ = vb_ + (2 * kh + xx) * VPAGE;                                                \
      f32x4 sacc = {0.f, 0.f, 0.f, 0.f}, pacc = {0.f, 0.f, 0.f, 0.f};                                 \
      _Pragma("unroll") for (int dc = 0; dc < 4; ++dc) {                                              \
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(kt_ + krow_off + (((dc * 4 + g) ^ krow_sw) * 8)); \
        sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qf[dc], sacc, 0, 0, 0);                    \
        /* rows d + 4: 8 logical chunks on = bit 3 of the chunk index = bit 6 of the element offset */ \
        const bf16x8 vf = tr_pair(vt_ + dc * 512 + v_base, vt_ + dc * 512 + (v_base ^ 64));           \
        pacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, dof[dc], pacc, 0, 0, 0);                   \
      }                                                                                               \
      _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                                 \
        const int kpos = (SP * (it_) + 2 * kh + xx) * PS + 4 * g + j;                                 \
        const bool ok = !(MASKED_) || kpos <= pos_c;                                                  \
        /* (the mask goes into the exponent: 2^-inf = 0 without a branch around the exponential) */   \
        const float e_ = sacc[j] * a.scale_log2 - lse2;                                               \
        const float p = __builtin_amdgcn_exp2f(ok ? e_ : -INFINITY);                                  \
        ds[xx * 4 + j] = p * (pacc[j] - delta);                                                       \
      }                                                                                               \
    }                                                                                                 \
    bf16x8 dsf;                                                                                       \
    _Pragma("unroll") for (int j = 0; j < 8; ++j) dsf[j] = (bf16_t)ds[j];                             \
    /* dQ^T[d, row] += K^T[d, keys] dS^T[keys, row]; lane (d, g): keys 4g..4g+3 of both pages */       \
    _Pragma("unroll") for (int mt = 0; mt < 8; ++mt) {                                                \
      const int off_ = kt_base + (((mt * 2 + kt_hi) ^ kt_sw) * 8);                                    \
      const bf16x8 kt = tr_pair(kb_ + (2 * kh) * TILE16 + off_, kb_ + (2 * kh + 1) * TILE16 + off_);  \
      dq[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kt, dsf, dq[mt], 0, 0, 0);                     \
    }                                                                                                 \
  }

  // step it: my loads of step it have landed -> barrier -> everyone's have, and everyone is done
  // with the other buffer set -> start the loads of step it + 1 into it -> multiply step it
#define FLEXCO_DQ_STEP(kb_, vb_, kn_, vn_, it_, MASKED_)                                              \
  {                                                                                                   \
    FLEXCO_WAIT_ALL_BARRIER                                                                           \
    if ((it_) + 1 < nit) {                                                                            \
      FLEXCO_ISSUE(kn_, vn_, (it_) + 1, page_nxt)                                                     \
      page_nxt = a.pages[min(SP * ((it_) + 2) + wave, last_page)];                                    \
    }                                                                                                 \
    FLEXCO_DQ_COMPUTE(kb_, vb_, it_, MASKED_)                                                         \
  }

  {
    const int page0 = a.pages[min(wave, last_page)];
    FLEXCO_ISSUE(kb0, vb0, 0, page0)
    page_nxt = a.pages[min(SP + wave, last_page)];
  }
  // leading steps whose two pages of this wavefront (2 kh, 2 kh + 1 of the step's SP) end at or before the position
  // of the wavefront's first row, in pairs (the two buffer sets); every form of a step has the one barrier, so the
  // wavefronts of a block may be in different loops
  const int vis_pages = (a.w0 + i0 + 1) / PS - 2 * kh - 2;           // step it is wholly visible iff SP it <= this
  const int n_vis = i0 < a.s && vis_pages >= 0 ? min(vis_pages / SP + 1, nit) & ~1 : 0;
  int it = 0;
  for (; it < n_vis; it += 2) {
    FLEXCO_DQ_STEP(kb0, vb0, kb1, vb1, it, false)
    FLEXCO_DQ_STEP(kb1, vb1, kb0, vb0, it + 1, false)
  }
  for (; it + 1 < nit; it += 2) {
    FLEXCO_DQ_STEP(kb0, vb0, kb1, vb1, it, true)
    FLEXCO_DQ_STEP(kb1, vb1, kb0, vb0, it + 1, true)
  }
  if (it < nit) FLEXCO_DQ_STEP(kb0, vb0, kb1, vb1, it, true)

  // ---- add the four key quarters (kh = 0, 1, 2, 3 in this order), scale, store -------------------
  float* red = reinterpret_cast<float*>(kb0);                    // [2 rt][32][64 lanes] floats = 16 KB
#pragma unroll 1
  for (int src = 1; src < SP / 2; ++src) {
    __syncthreads();
    if (kh == src) {
#pragma unroll
      for (int mt = 0; mt < 8; ++mt)
#pragma unroll
        for (int j = 0; j < 4; ++j) red[((rt * 8 + mt) * 4 + j) * 64 + lane] = dq[mt][j];
    }
    __syncthreads();
    if (kh == 0) {
#pragma unroll
      for (int mt = 0; mt < 8; ++mt)
#pragma unroll
        for (int j = 0; j < 4; ++j) dq[mt][j] += red[((rt * 8 + mt) * 4 + j) * 64 + lane];
    }
  }
  if (kh == 0 && row_ok) {
    bf16_t* out = a.dq + ((size_t)row_c * a.nq + h) * D + 4 * g;
#pragma unroll
    for (int mt = 0; mt < 8; ++mt) {
      bf16x4 v;
#pragma unroll
      for (int j = 0; j < 4; ++j) v[j] = (bf16_t)(dq[mt][j] * a.scale);
      *reinterpret_cast<bf16x4*>(out + mt * 16) = v;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// kernel B: dK, dV.  grid (ceil(l / 64), nkv), 8 wavefronts (NH = 2).  Wavefront w owns the page (16 keys)
// 4 b + w % 4 and walks over the window's rows, 32 rows per step, for every second query head of the
// kv group (w / 4 = 0: heads 0, 2, ..; 1: heads 1, 3, ..): the two halves of a block multiply different
// heads at the same time and their sums are added in a fixed order at the end.  NH = 1: four wavefronts
// that walk every head of the group, nothing to add at the end.  (The grid has one
// block per CU or fewer, and a step is a chain of dependent LDS reads and MFMAs: the second half's
// chains fill the first half's waits.)
// ---------------------------------------------------------------------------------------------
template <int NH>   // head halves that work side by side: 2 (eight wavefronts) or 1 (four)
__global__ __launch_bounds__(256 * NH, NH == 1 ? 2 : 1) void attn_bwd_dkv_mfma_kernel(BwdArgs a) {
  __shared__ __attribute__((aligned(1024))) bf16_t qb0[NH][2 * TILE16];
  __shared__ __attribute__((aligned(1024))) bf16_t qb1[NH][2 * TILE16];
  __shared__ __attribute__((aligned(1024))) bf16_t ob0[NH][2 * TILE16];
  __shared__ __attribute__((aligned(1024))) bf16_t ob1[NH][2 * TILE16];
  __shared__ __attribute__((aligned(256))) float ld0[NH][64];   // lse[32] | delta[32] of the step's rows
  __shared__ __attribute__((aligned(256))) float ld1[NH][64];
  __shared__ float red[NH == 2 ? 4 : 1][NH == 2 ? 8 * 4 * 64 : 1];   // sums of the second half, one output at a time
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wavefront-uniform: LDS bases of the loads stay scalar
  const int pw = wave & 3, hg = wave >> 2;
  const int c = lane & 15, g = lane >> 4;
  // (kv head = fastest digit of the work-group id: see kernel A; here it is the group's Q / dO rows that the
  // blocks of one kv head share)
  const int group = a.nq / a.nkv;
  const int lid = blockIdx.y * gridDim.x + blockIdx.x;
  const int kvh = lid % a.nkv;
  const int bx = lid / a.nkv;                                    // block of 64 keys
  const int pg = bx * 4 + pw;
  const int key0 = pg * PS;
  const bool page_ok = key0 < a.l;
  const size_t page = (size_t)a.pages[page_ok ? pg : (a.l - 1) / PS];
  const int kpos = key0 + c;
  const bool key_ok = kpos < a.l;

  // K rows of this page as B operand (k = d): lane (key c, g) holds d = 32 dc + 8 g .. + 8
  // V of this page as B operand (k = d): the same elements of V, gathered from the position-minor page
  bf16x8 kf[4], vf[4];
  {
    const bf16_t* kr = a.kp + ((page * a.nkv + kvh) * PS + c) * (size_t)D + g * 8;
    const bf16_t* vr = a.vp + (page * a.nkv + kvh) * (size_t)D * PS + c;
#pragma unroll
    for (int dc = 0; dc < 4; ++dc) {
      kf[dc] = *reinterpret_cast<const bf16x8*>(kr + dc * 32);
#pragma unroll
      for (int j = 0; j < 8; ++j) vf[dc][j] = vr[(size_t)(dc * 32 + g * 8 + j) * PS];
    }
  }
  f32x4 dk[8], dv[8];
#pragma unroll
  for (int mt = 0; mt < 8; ++mt) { dk[mt] = f32x4{0.f, 0.f, 0.f, 0.f}; dv[mt] = f32x4{0.f, 0.f, 0.f, 0.f}; }

  const int blk_key0 = bx * 64;
  const int first_row = max(0, blk_key0 - a.w0) & ~31;       // first window row that sees the block's keys
  const int nrb = (a.s - first_row + 31) / 32;               // row blocks per head
  const int nit = ((group + NH - 1) / NH) * nrb;             // steps: heads NH (it / nrb) + hg

  // ---- loads: 8 instructions per 32-row tile (4 rows each); wavefront (pw, hg) issues 2 pw, 2 pw + 1
  // of its half's Q tile and dO tile; wavefront pw = 0 also brings in the rows' lse (lanes 0..31) and
  // delta (lanes 32..63), 4 bytes per lane.  Rows past the window repeat its last row, a head past the
  // group repeats the group's last head (both masked later).
  const int t_rin = lane >> 4, t_pc = lane & 15;
#define FLEXCO_ISSUE_QO(qb_, ob_, ld_, it_)                                                           \
  {                                                                                                   \
    const int h_ = kvh * group + min(NH * ((it_) / nrb) + hg, group - 1);                              \
    const int r0_ = first_row + 32 * ((it_) % nrb);                                                   \
    _Pragma("unroll") for (int e = 0; e < 2; ++e) {                                                   \
      const int row_ = 4 * (2 * pw + e) + t_rin;                                                      \
      const size_t src_ = ((size_t)min(r0_ + row_, a.s - 1) * a.nq + h_) * D + ((t_pc ^ rsw(row_)) * 8); \
      __builtin_amdgcn_global_load_lds(FLEXCO_GP(a.q + src_), FLEXCO_LP(qb_[hg] + (2 * pw + e) * 4 * D), 16, 0, 0); \
      __builtin_amdgcn_global_load_lds(FLEXCO_GP(a.dout + src_), FLEXCO_LP(ob_[hg] + (2 * pw + e) * 4 * D), 16, 0, 0); \
    }                                                                                                 \
    if (pw == 0) {                                                                                    \
      const size_t idx_ = (size_t)min(r0_ + (lane & 31), a.s - 1) * a.nq + h_;                        \
      const float* src_ = (lane < 32 ? a.lse : a.delta) + idx_;                                       \
      __builtin_amdgcn_global_load_lds(FLEXCO_GP(src_), FLEXCO_LP(ld_[hg]), 4, 0, 0);                 \
    }                                                                                                 \
  }

  const int row_off = c * D, row_sw = rsw(c);
  const int s4 = c >> 2, sc = c & 3;
  const int tr_row = 4 * g + s4;
  const int tr_base = tr_row * D + (sc & 1) * 4;
  const int tr_sw = rsw(tr_row), tr_hi = sc >> 1;

  // (an unmasked form of the step for row blocks wholly after the page, chosen per step, cost more in register copies
  // where the two forms join than the masks do: 200 moves per step; the dQ kernel's steps split into two loops instead)
#define FLEXCO_DKV_COMPUTE(qb_, ob_, ld_, it_)                                                        \
  {                                                                                                   \
    const int r0 = first_row + 32 * ((it_) % nrb);                                                    \
    const bool head_ok = NH * ((it_) / nrb) + hg < group;                                             \
    /* (a step with nothing to add - a head past the group, a page past the sequence, rows before the page - is not */ \
    /* skipped: its elements are all masked and add zeros; a branch around the products cost a copy of all 64      */ \
    /* accumulator registers every second step)                                                                   */ \
    {                                                                                                 \
      const bf16_t* qt_ = qb_[hg];                                                                    \
      const bf16_t* ot_ = ob_[hg];                                                                    \
      const float* lt_ = ld_[hg];                                                                     \
      float p[8], ds[8];                                                                              \
      _Pragma("unroll") for (int x = 0; x < 2; ++x) {                                                 \
        f32x4 sacc = {0.f, 0.f, 0.f, 0.f}, pacc = {0.f, 0.f, 0.f, 0.f};                               \
        _Pragma("unroll") for (int dc = 0; dc < 4; ++dc) {                                            \
          const int off_ = x * TILE16 + row_off + (((dc * 4 + g) ^ row_sw) * 8);                      \
          const bf16x8 qa = *reinterpret_cast<const bf16x8*>(qt_ + off_);                             \
          const bf16x8 oa = *reinterpret_cast<const bf16x8*>(ot_ + off_);                             \
          sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qa, kf[dc], sacc, 0, 0, 0);   /* S[row, key] */  \
          pacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(oa, vf[dc], pacc, 0, 0, 0);   /* dP[row, key] */ \
        }                                                                                             \
        _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                               \
          const int rl = x * 16 + 4 * g + j;            /* lane (key c, g) holds rows 4g..4g+3 of tile x */ \
          const int row = r0 + rl;                                                                    \
          const bool ok = head_ok && key_ok && row < a.s && kpos <= a.w0 + row;                       \
          /* (the mask goes into the exponent: 2^-inf = 0 without a branch around the exponential) */ \
          const float e_ = sacc[j] * a.scale_log2 - lt_[rl] * LOG2E;   /* (read before the choice: no branch) */ \
          const float pv = __builtin_amdgcn_exp2f(ok ? e_ : -INFINITY);                               \
          p[x * 4 + j] = pv;                                                                          \
          ds[x * 4 + j] = pv * (pacc[j] - lt_[32 + rl]);                                              \
        }                                                                                             \
      }                                                                                               \
      bf16x8 pf, dsf;                                                                                 \
      _Pragma("unroll") for (int j = 0; j < 8; ++j) { pf[j] = (bf16_t)p[j]; dsf[j] = (bf16_t)ds[j]; } \
      /* dV^T[d, key] += dO^T[d, rows] P[rows, key];  dK^T[d, key] += Q^T[d, rows] dS[rows, key] */    \
      /* lane (d, g): rows 4g..4g+3 of both row tiles at column d */                                   \
      _Pragma("unroll") for (int mt = 0; mt < 8; ++mt) {                                              \
        const int off_ = tr_base + (((mt * 2 + tr_hi) ^ tr_sw) * 8);                                  \
        const bf16x8 ot = tr_pair(ot_ + off_, ot_ + TILE16 + off_);                                   \
        const bf16x8 qt = tr_pair(qt_ + off_, qt_ + TILE16 + off_);                                   \
        dv[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ot, pf, dv[mt], 0, 0, 0);                    \
        dk[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qt, dsf, dk[mt], 0, 0, 0);                   \
      }                                                                                               \
    }                                                                                                 \
  }
#define FLEXCO_DKV_STEP(qb_, ob_, ld_, qn_, on_, ln_, it_)                                            \
  {                                                                                                   \
    FLEXCO_WAIT_ALL_BARRIER                                                                           \
    if ((it_) + 1 < nit) FLEXCO_ISSUE_QO(qn_, on_, ln_, (it_) + 1)                                    \
    FLEXCO_DKV_COMPUTE(qb_, ob_, ld_, it_)                                                            \
  }

  FLEXCO_ISSUE_QO(qb0, ob0, ld0, 0)
  int it = 0;
  for (; it + 1 < nit; it += 2) {
    FLEXCO_DKV_STEP(qb0, ob0, ld0, qb1, ob1, ld1, it)
    FLEXCO_DKV_STEP(qb1, ob1, ld1, qb0, ob0, ld0, it + 1)
  }
  if (it < nit) FLEXCO_DKV_STEP(qb0, ob0, ld0, qb1, ob1, ld1, it)
  __builtin_amdgcn_s_waitcnt(0x0F70);   // nothing may land in LDS after the block ends

  // ---- the second half's sums join the first half's (dK, then dV), which adds them to the accumulator ----
#pragma unroll
  for (int which = 0; which < (NH == 2 ? 2 : 0); ++which) {
    __syncthreads();
    if (hg == 1) {
#pragma unroll
      for (int mt = 0; mt < 8; ++mt)
#pragma unroll
        for (int j = 0; j < 4; ++j) red[pw][(mt * 4 + j) * 64 + lane] = which == 0 ? dk[mt][j] : dv[mt][j];
    }
    __syncthreads();
    if (hg == 0) {
#pragma unroll
      for (int mt = 0; mt < 8; ++mt)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float v = red[pw][(mt * 4 + j) * 64 + lane];
          if (which == 0) dk[mt][j] += v; else dv[mt][j] += v;
        }
    }
  }
  if (hg == 0 && key_ok) {
    float* dkp = a.dk_accum + ((size_t)kpos * a.nkv + kvh) * D + 4 * g;
    float* dvp = a.dv_accum + ((size_t)kpos * a.nkv + kvh) * D + 4 * g;
#pragma unroll
    for (int mt = 0; mt < 8; ++mt) {
      f32x4 ok = *reinterpret_cast<f32x4*>(dkp + mt * 16), ov = *reinterpret_cast<f32x4*>(dvp + mt * 16);
#pragma unroll
      for (int j = 0; j < 4; ++j) { ok[j] += dk[mt][j] * a.scale; ov[j] += dv[mt][j]; }
      *reinterpret_cast<f32x4*>(dkp + mt * 16) = ok;
      *reinterpret_cast<f32x4*>(dvp + mt * 16) = ov;
    }
  }
}

}  // namespace

int32_t launch_attention_bwd_mfma(const flexco_layer_cfg& c, const flexco_kv_pool& pool, const int32_t* seq_pages,
                                  int win_start, int win_len, const void* q, const void* out, const float* lse,
                                  float* delta, const void* dout, void* dq, float* dk_accum, float* dv_accum,
                                  hipStream_t s) {
  if (c.dtype != FLEXCO_BF16 || c.head_dim != D || c.page_size != PS) return FLEXCO_EUNSUPPORTED;
  BwdArgs a;
  a.q = (const bf16_t*)q; a.dout = (const bf16_t*)dout; a.out = (const bf16_t*)out; a.lse = lse; a.delta = delta;
  a.kp = (const bf16_t*)pool.k_pages; a.vp = (const bf16_t*)pool.v_pages; a.pages = seq_pages;
  a.dq = (bf16_t*)dq; a.dk_accum = dk_accum; a.dv_accum = dv_accum;
  a.w0 = win_start; a.s = win_len; a.l = win_start + win_len; a.nq = c.n_q_heads; a.nkv = c.n_kv_heads;
  a.scale = 1.0f / sqrtf((float)D);
  a.scale_log2 = a.scale * LOG2E;
  // kernel A: eight wavefronts and eight pages per step while the grid gives a CU one block; with more blocks than
  // CUs, four wavefronts and four pages (64 KB of LDS, two blocks share a CU, each with its own barrier): 3 - 6 %
  // faster there, 13 % slower on the one-block grid of a 256-row window
  const dim3 grid_a((a.s + 31) / 32, a.nq);
  if ((long)grid_a.x * grid_a.y > 256) hipLaunchKernelGGL(attn_bwd_dq_mfma_kernel<4>, grid_a, dim3(256), 0, s, a);
  else hipLaunchKernelGGL(attn_bwd_dq_mfma_kernel<8>, grid_a, dim3(512), 0, s, a);
  // kernel B: the same choice - with more blocks than CUs, four-wavefront blocks that walk all heads of the kv group
  // in turn (33 KB of LDS, two blocks per CU): 7 - 9 % faster on the 4096-key windows
  const dim3 grid_b((a.l + 63) / 64, a.nkv);
  if ((long)grid_b.x * grid_b.y > 256) hipLaunchKernelGGL(attn_bwd_dkv_mfma_kernel<1>, grid_b, dim3(256), 0, s, a);
  else hipLaunchKernelGGL(attn_bwd_dkv_mfma_kernel<2>, grid_b, dim3(512), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(FLEXCO_EHIP, "launch of attn_bwd_mfma failed: %s", hipGetErrorString(e));
  return FLEXCO_OK;
}

}  // namespace flexco

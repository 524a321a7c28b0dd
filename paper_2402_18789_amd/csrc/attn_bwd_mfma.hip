// Attention backward of one token window on the matrix cores (Sec. 6.1, Alg. 2 Backward).
//
// Queries are the window's rows i at positions win_start + i; keys/values are the cached rows
// [0, l), l = win_start + win_len, read through the sequence's page list.  The softmax
// probabilities are recomputed from Q, K and the stored log-sum-exp (graph pruning keeps Q, K, V
// and rematerialises P).  With delta_i = sum_d dO_id O_id:
//     P_ij = exp(q_i . k_j / sqrt(d) - lse_i)           (j <= position of i)
//     dP_ij = dO_i . v_j ,   dS_ij = P_ij (dP_ij - delta_i)
//     dQ_i = sum_j dS_ij k_j / sqrt(d)                   -> kernel A, one block per 64 rows x head
//     dK_j = sum_i dS_ij q_i / sqrt(d),  dV_j = sum_i P_ij dO_i   summed over the window's rows
//            and over the query heads of the kv group     -> kernel B, one block per 64 keys x kv head
// Two kernels, each owning its outputs: no atomics, results do not depend on scheduling.  dK/dV are
// added into the KV-gradient accumulator rows [0, l) (Sec. 7).
//
// bf16, head_dim 128, page_size 16.  All products are v_mfma_f32_16x16x32_bf16.  Operands whose
// contracted index is contiguous in memory (K rows, Q rows, dO rows) are used as they are;
// operands that must be read "across" their rows (V and K^T in kernel A; Q^T, dO^T in kernel B)
// are staged in LDS once per block and gathered with 16-bit reads; row strides are padded so
// that the four k-groups of a wavefront fall on disjoint banks.
#include "flexco_internal.h"
#include "device_types.h"

namespace flexco {

namespace {

constexpr int D = 128, PS = 16;
constexpr int LDR = D + 8;   // padded row of a staged [rows][128] tile (272 bytes)
constexpr float LOG2E = 1.4426950408889634f;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

struct BwdArgs {
  const bf16_t *q, *dout;
  const float *lse, *delta;
  const bf16_t *kp, *vp;
  const int32_t* pages;
  bf16_t* dq;
  float *dk_accum, *dv_accum;
  int w0, s, l, nq, nkv;
  float scale, scale_log2;
};

// byte offset of element (d, key) of a staged V page: [d][16 keys] rows of 32 bytes, every group of
// 8 rows shifted by 64 bytes so that d, d + 8, d + 16, d + 24 land on different banks
__device__ inline int vs_off(int d, int key) { return d * 32 + (d >> 3) * 64 + key * 2; }
constexpr int VS_PAGE_BYTES = D * 32 + (D / 8) * 64;   // 5120

__device__ inline bf16x8 zero8() { return bf16x8{0, 0, 0, 0, 0, 0, 0, 0}; }

// ---------------------------------------------------------------------------------------------
// kernel A: dQ.  grid (ceil(s / 64), nq); wavefront w of a block owns rows [64 b + 16 w, + 16).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void attn_bwd_dq_mfma_kernel(BwdArgs a) {
  __shared__ __attribute__((aligned(16))) bf16_t Ks[32 * LDR];
  __shared__ __attribute__((aligned(16))) unsigned char Vs[2 * VS_PAGE_BYTES];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int c = lane & 15, g = lane >> 4;
  const int h = blockIdx.y, group = a.nq / a.nkv, kvh = h / group;
  const int i0 = blockIdx.x * 64 + wave * 16;
  const int row_c = i0 + c;
  const bool row_ok = row_c < a.s;
  const int rcl = row_ok ? row_c : a.s - 1;
  const int pos_c = row_ok ? a.w0 + row_c : -1;
  const int wave_last_pos = a.w0 + min(i0 + 15, a.s - 1);      // may be < first key if the tile is empty
  const int blk_last_row = min(blockIdx.x * 64 + 63, a.s - 1);
  const int np = (a.w0 + blk_last_row) / PS + 1;                 // pages visible to the block

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
  const float delta = a.delta[(size_t)rcl * a.nq + h];

  f32x4 dq[8];
#pragma unroll
  for (int mt = 0; mt < 8; ++mt) dq[mt] = f32x4{0.f, 0.f, 0.f, 0.f};

  for (int pp = 0; pp < np; pp += 2) {
    __syncthreads();
    // ---- stage the K and V rows of two pages; slots at or beyond l (never written) become zero ----
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const int qid = tid + 256 * e;
      const int x = qid >> 8, rem = qid & 255;
      const bool pg_ok = pp + x < np;
      const size_t page = (size_t)a.pages[pg_ok ? pp + x : pp];
      {   // K chunk: key = rem / 16, 16-byte chunk rem % 16
        const int key = rem >> 4, ch = rem & 15;
        u32x4 v = *reinterpret_cast<const u32x4*>(a.kp + ((page * a.nkv + kvh) * PS + key) * (size_t)D + ch * 8);
        if (!pg_ok || (pp + x) * PS + key >= a.l) v = u32x4{0, 0, 0, 0};
        *reinterpret_cast<u32x4*>(Ks + (x * 16 + key) * LDR + ch * 8) = v;
      }
      {   // V chunk: d = rem / 2, keys 8 (rem % 2) .. + 8
        const int d = rem >> 1, half = rem & 1;
        bf16x8 v = *reinterpret_cast<const bf16x8*>(a.vp + ((page * a.nkv + kvh) * (size_t)D + d) * PS + half * 8);
        const int kbase = (pp + x) * PS + half * 8;
        if (!pg_ok || kbase + 8 > a.l) {
#pragma unroll
          for (int j = 0; j < 8; ++j)
            if (!pg_ok || kbase + j >= a.l) v[j] = (bf16_t)0.f;
        }
        *reinterpret_cast<bf16x8*>(Vs + x * VS_PAGE_BYTES + vs_off(d, half * 8)) = v;
      }
    }
    __syncthreads();
    if (pp * PS > wave_last_pos) continue;     // nothing visible to this wavefront's rows (uniform)

    float ds[8];
#pragma unroll
    for (int x = 0; x < 2; ++x) {
      f32x4 sacc = {0.f, 0.f, 0.f, 0.f}, pacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int dc = 0; dc < 4; ++dc) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(Ks + (x * 16 + c) * LDR + dc * 32 + g * 8);
        sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qf[dc], sacc, 0, 0, 0);
        bf16x8 vf;
#pragma unroll
        for (int j = 0; j < 8; ++j)
          vf[j] = *reinterpret_cast<const bf16_t*>(Vs + x * VS_PAGE_BYTES + vs_off(dc * 32 + g * 8 + j, c));
        pacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, dof[dc], pacc, 0, 0, 0);
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int kpos = (pp + x) * PS + 4 * g + j;
        const bool ok = kpos <= pos_c;
        const float p = __builtin_amdgcn_exp2f(sacc[j] * a.scale_log2 - lse2);
        ds[x * 4 + j] = ok ? p * (pacc[j] - delta) : 0.f;
      }
    }
    bf16x8 dsf;
#pragma unroll
    for (int j = 0; j < 8; ++j) dsf[j] = (bf16_t)ds[j];
    // dQ^T[d, row] += K^T[d, keys] dS^T[keys, row];  lane (d, g) gathers keys {4g..4g+3} of both pages
#pragma unroll
    for (int mt = 0; mt < 8; ++mt) {
      bf16x8 kt;
      const bf16_t* col = Ks + mt * 16 + c;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        kt[j] = col[(4 * g + j) * LDR];
        kt[4 + j] = col[(16 + 4 * g + j) * LDR];
      }
      dq[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kt, dsf, dq[mt], 0, 0, 0);
    }
  }
  if (row_ok) {
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
// kernel B: dK, dV.  grid (ceil(l / 64), nkv); wavefront w owns the page (16 keys) 4 b + w.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void attn_bwd_dkv_mfma_kernel(BwdArgs a) {
  __shared__ __attribute__((aligned(16))) bf16_t Qs[32 * LDR];
  __shared__ __attribute__((aligned(16))) bf16_t Os[32 * LDR];
  __shared__ float lse_s[32], delta_s[32];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int c = lane & 15, g = lane >> 4;
  const int kvh = blockIdx.y, group = a.nq / a.nkv;
  const int pg = blockIdx.x * 4 + wave;
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

  const int blk_key0 = blockIdx.x * 64;
  const int first_row = max(0, blk_key0 - a.w0) & ~31;       // first window row that sees the block's keys
  for (int hg = 0; hg < group; ++hg) {
    const int h = kvh * group + hg;
    for (int r0 = first_row; r0 < a.s; r0 += 32) {
      __syncthreads();
      // ---- stage 32 rows of Q and dO of head h (rows beyond the window repeat the last row; masked) ----
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const int qid = tid + 256 * e;           // 512 chunks: row = qid / 16, chunk qid % 16
        const int row = qid >> 4, ch = qid & 15;
        const int rcl = min(r0 + row, a.s - 1);
        const size_t src = ((size_t)rcl * a.nq + h) * D + ch * 8;
        *reinterpret_cast<u32x4*>(Qs + row * LDR + ch * 8) = *reinterpret_cast<const u32x4*>(a.q + src);
        *reinterpret_cast<u32x4*>(Os + row * LDR + ch * 8) = *reinterpret_cast<const u32x4*>(a.dout + src);
      }
      if (tid < 32) {
        const int rcl = min(r0 + tid, a.s - 1);
        lse_s[tid] = a.lse[(size_t)rcl * a.nq + h] * LOG2E;
        delta_s[tid] = a.delta[(size_t)rcl * a.nq + h];
      }
      __syncthreads();
      if (!page_ok || key0 > a.w0 + min(r0 + 31, a.s - 1)) continue;   // no row of the pair sees this page

      float p[8], ds[8];
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        f32x4 sacc = {0.f, 0.f, 0.f, 0.f}, pacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int dc = 0; dc < 4; ++dc) {
          const bf16x8 qa = *reinterpret_cast<const bf16x8*>(Qs + (x * 16 + c) * LDR + dc * 32 + g * 8);
          const bf16x8 oa = *reinterpret_cast<const bf16x8*>(Os + (x * 16 + c) * LDR + dc * 32 + g * 8);
          sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qa, kf[dc], sacc, 0, 0, 0);   // S[row, key]
          pacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(oa, vf[dc], pacc, 0, 0, 0);   // dP[row, key]
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int rl = x * 16 + 4 * g + j;            // lane (key c, g) holds rows 4g..4g+3 of tile x
          const int row = r0 + rl;
          const bool ok = key_ok && row < a.s && kpos <= a.w0 + row;
          const float pv = __builtin_amdgcn_exp2f(sacc[j] * a.scale_log2 - lse_s[rl]);
          p[x * 4 + j] = ok ? pv : 0.f;
          ds[x * 4 + j] = ok ? pv * (pacc[j] - delta_s[rl]) : 0.f;
        }
      }
      bf16x8 pf, dsf;
#pragma unroll
      for (int j = 0; j < 8; ++j) { pf[j] = (bf16_t)p[j]; dsf[j] = (bf16_t)ds[j]; }
      // dV^T[d, key] += dO^T[d, rows] P[rows, key];  dK^T[d, key] += Q^T[d, rows] dS[rows, key]
      // lane (d, g) gathers rows {4g..4g+3} of both row tiles at column d
#pragma unroll
      for (int mt = 0; mt < 8; ++mt) {
        bf16x8 ot, qt;
        const bf16_t* ocol = Os + mt * 16 + c;
        const bf16_t* qcol = Qs + mt * 16 + c;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          ot[j] = ocol[(4 * g + j) * LDR];
          ot[4 + j] = ocol[(16 + 4 * g + j) * LDR];
          qt[j] = qcol[(4 * g + j) * LDR];
          qt[4 + j] = qcol[(16 + 4 * g + j) * LDR];
        }
        dv[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ot, pf, dv[mt], 0, 0, 0);
        dk[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qt, dsf, dk[mt], 0, 0, 0);
      }
    }
  }
  if (key_ok) {
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
                                  int win_start, int win_len, const void* q, const float* lse, const float* delta,
                                  const void* dout, void* dq, float* dk_accum, float* dv_accum, hipStream_t s) {
  if (c.dtype != FLEXCO_BF16 || c.head_dim != D || c.page_size != PS) return FLEXCO_EUNSUPPORTED;
  BwdArgs a;
  a.q = (const bf16_t*)q; a.dout = (const bf16_t*)dout; a.lse = lse; a.delta = delta;
  a.kp = (const bf16_t*)pool.k_pages; a.vp = (const bf16_t*)pool.v_pages; a.pages = seq_pages;
  a.dq = (bf16_t*)dq; a.dk_accum = dk_accum; a.dv_accum = dv_accum;
  a.w0 = win_start; a.s = win_len; a.l = win_start + win_len; a.nq = c.n_q_heads; a.nkv = c.n_kv_heads;
  a.scale = 1.0f / sqrtf((float)D);
  a.scale_log2 = a.scale * LOG2E;
  hipLaunchKernelGGL(attn_bwd_dq_mfma_kernel, dim3((a.s + 63) / 64, a.nq), dim3(256), 0, s, a);
  hipLaunchKernelGGL(attn_bwd_dkv_mfma_kernel, dim3((a.l + 63) / 64, a.nkv), dim3(256), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(FLEXCO_EHIP, "launch of attn_bwd_mfma failed: %s", hipGetErrorString(e));
  return FLEXCO_OK;
}

}  // namespace flexco

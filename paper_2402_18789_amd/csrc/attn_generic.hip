// Type-generic mixed attention (forward partials + merge) and window backward.
//
// These kernels serve the fp32 configuration and any shape the MFMA kernels do not cover.
// They share the work list and the partial-result format with the MFMA path:
//   work item (tile, split) x kv head  ->  for each column c of the tile (token c / group,
//   query head kvh * group + c % group): running max m, sum l and un-normalised
//   accumulator acc[d] over the keys of the split that the column may see.
//   part_ml [n_parts, nkv, cols_per_tile, 2], part_acc [n_parts, nkv, cols_per_tile, d]
// The merge kernel combines the splits of a tile (log-sum-exp weighting).
#include "flexco_internal.h"
#include "device_types.h"

namespace flexco {

__device__ inline float wsum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ inline float wmax(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

struct AttnArgs {
  const int32_t *tok_pos, *block_table, *tile_req, *tile_tok0, *tile_ntok, *tile_nsplit, *tile_part0, *item_tile,
      *item_split, *item_ntiles;
  int max_pages, nq, nkv, d, ps, split_keys, cols_per_tile;
  float scale;
};

template <typename T>
__global__ __launch_bounds__(256) void attn_fwd_generic_kernel(AttnArgs a, const T* __restrict__ q, size_t ldq,
                                                               const T* __restrict__ kp, const T* __restrict__ vp,
                                                               float* __restrict__ part_ml,
                                                               float* __restrict__ part_acc) {
  extern __shared__ float smem[];   // per wave: q[d] + scores[split_keys]
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  float* qs = smem + wave * (a.d + a.split_keys);
  float* sc = qs + a.d;
  // one block per tile of the work item that has this split (blockIdx.z = tile within the item)
  const int item = blockIdx.x, kvh = blockIdx.y;
  if ((int)blockIdx.z >= a.item_ntiles[item]) return;
  const int tile = a.item_tile[item] + blockIdx.z, split = a.item_split[item];
  if (split >= a.tile_nsplit[tile]) return;
  const int r = a.tile_req[tile], t0 = a.tile_tok0[tile], ntok = a.tile_ntok[tile];
  const int group = a.nq / a.nkv;
  const int part = a.tile_part0[tile] + split;
  const int k0 = split * a.split_keys;
  const int32_t* bt = a.block_table + (size_t)r * a.max_pages;
  for (int c = wave; c < ntok * group; c += 4) {
    const int t = t0 + c / group, h = kvh * group + c % group;
    const int kend = min(k0 + a.split_keys, a.tok_pos[t] + 1);
    const int nk = max(0, kend - k0);
    for (int dd = lane; dd < a.d; dd += 64) qs[dd] = ld(q + (size_t)t * ldq + h * a.d + dd);
    __builtin_amdgcn_wave_barrier();
    float m = -INFINITY;
    for (int jj = lane; jj < nk; jj += 64) {
      const int j = k0 + jj;
      const size_t page = bt[j / a.ps];
      const T* kr = kp + ((page * a.nkv + kvh) * a.ps + j % a.ps) * (size_t)a.d;
      float s = 0.f;
      for (int dd = 0; dd < a.d; ++dd) s += qs[dd] * ld(kr + dd);
      s *= a.scale;
      sc[jj] = s;
      m = fmaxf(m, s);
    }
    m = wmax(m);
    float l = 0.f;
    for (int jj = lane; jj < nk; jj += 64) {
      const float p = __expf(sc[jj] - m);
      sc[jj] = p;
      l += p;
    }
    l = wsum(l);
    __builtin_amdgcn_wave_barrier();
    const size_t idx = ((size_t)part * a.nkv + kvh) * a.cols_per_tile + c;
    for (int dd = lane; dd < a.d; dd += 64) {
      float acc = 0.f;
      for (int jj = 0; jj < nk; ++jj) {
        const int j = k0 + jj;
        const size_t page = bt[j / a.ps];
        acc += sc[jj] * ld(vp + ((page * a.nkv + kvh) * (size_t)a.d + dd) * a.ps + j % a.ps);
      }
      part_acc[idx * a.d + dd] = acc;
    }
    if (lane == 0) { part_ml[idx * 2] = m; part_ml[idx * 2 + 1] = l; }
    __builtin_amdgcn_wave_barrier();
  }
}

// One wave per (token, query head): combine the tile's splits.
template <typename T>
__global__ __launch_bounds__(64) void attn_merge_kernel(const int32_t* __restrict__ tok_tile,
                                                        const int32_t* __restrict__ tile_tok0,
                                                        const int32_t* __restrict__ tile_nsplit,
                                                        const int32_t* __restrict__ tile_part0,
                                                        const float* __restrict__ part_ml,
                                                        const float* __restrict__ part_acc, T* __restrict__ out,
                                                        size_t ldo, float* __restrict__ lse, int nq, int nkv, int d,
                                                        int cols_per_tile, int skip_single_split, AttnKeep keep) {
  const int t = blockIdx.x, h = blockIdx.y;
  const int group = nq / nkv, kvh = h / group;
  const int tile = tok_tile[t];
  const int c = (t - tile_tok0[tile]) * group + h % group;
  const int nsplit = tile_nsplit[tile], part0 = tile_part0[tile];
  if (skip_single_split && nsplit == 1) return;   // the attention kernel has written these rows itself
  float M = -INFINITY;
  for (int s = 0; s < nsplit; ++s) {
    const size_t idx = ((size_t)(part0 + s) * nkv + kvh) * cols_per_tile + c;
    M = fmaxf(M, part_ml[idx * 2]);
  }
  float L = 0.f;
  for (int s = 0; s < nsplit; ++s) {
    const size_t idx = ((size_t)(part0 + s) * nkv + kvh) * cols_per_tile + c;
    const float ms = part_ml[idx * 2];
    if (ms > -INFINITY) L += part_ml[idx * 2 + 1] * __expf(ms - M);
  }
  const float inv = 1.0f / L;
  const bool kept = keep.lse2 && t >= keep.tok0 && t < keep.tok0 + keep.n;
  for (int dd = threadIdx.x; dd < d; dd += 64) {
    float acc = 0.f;
    for (int s = 0; s < nsplit; ++s) {
      const size_t idx = ((size_t)(part0 + s) * nkv + kvh) * cols_per_tile + c;
      const float ms = part_ml[idx * 2];
      if (ms > -INFINITY) acc += part_acc[idx * d + dd] * __expf(ms - M);
    }
    st(out + (size_t)t * ldo + h * d + dd, acc * inv);
    if (kept) st((T*)keep.out2 + ((size_t)(t - keep.tok0) * nq + h) * d + dd, acc * inv);
  }
  if (threadIdx.x == 0) {
    if (lse) lse[(size_t)t * nq + h] = M + __logf(L);
    if (kept) keep.lse2[(size_t)(t - keep.tok0) * nq + h] = M + __logf(L);
  }
}

__device__ inline void store4(float* p, const float (&v)[4]) { *reinterpret_cast<f32x4*>(p) = f32x4{v[0], v[1], v[2], v[3]}; }
__device__ inline void store4(bf16_t* p, const float (&v)[4]) {
  bf16x4 t;
#pragma unroll
  for (int j = 0; j < 4; ++j) t[j] = (bf16_t)v[j];
  *reinterpret_cast<bf16x4*>(p) = t;
}

// The same for head_dim 128 with 16-byte accesses: 32 lanes per (token, query head), eight of them per block (the
// one-wavefront form above is a grid of T x nq blocks of which most leave at once - tiles with a single split - and
// the others read four bytes per lane).
template <typename T>
__global__ __launch_bounds__(256) void attn_merge128_kernel(const int32_t* __restrict__ tok_tile,
                                                            const int32_t* __restrict__ tile_tok0,
                                                            const int32_t* __restrict__ tile_nsplit,
                                                            const int32_t* __restrict__ tile_part0,
                                                            const float* __restrict__ part_ml,
                                                            const float* __restrict__ part_acc, T* __restrict__ out,
                                                            size_t ldo, float* __restrict__ lse, int nq, int nkv,
                                                            int cols_per_tile, int skip_single_split, AttnKeep keep) {
  constexpr int d = 128;
  const int t = blockIdx.x, h = blockIdx.y * 8 + (threadIdx.x >> 5), ln = threadIdx.x & 31;
  if (h >= nq) return;
  const int group = nq / nkv, kvh = h / group;
  const int tile = tok_tile[t];
  const int nsplit = tile_nsplit[tile];
  if (skip_single_split && nsplit == 1) return;   // the attention kernel has written these rows itself
  const int c = (t - tile_tok0[tile]) * group + h % group;
  const size_t idx0 = ((size_t)tile_part0[tile] * nkv + kvh) * cols_per_tile + c;
  const size_t step = (size_t)nkv * cols_per_tile;         // from one split's row to the next
  float M = -INFINITY;
  for (int s = 0; s < nsplit; ++s) M = fmaxf(M, part_ml[(idx0 + s * step) * 2]);
  float L = 0.f;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < nsplit; ++s) {
    const size_t idx = idx0 + s * step;
    const float ms = part_ml[idx * 2];
    if (ms > -INFINITY) {
      const float w = __expf(ms - M);
      L += part_ml[idx * 2 + 1] * w;
      const f32x4 a = *reinterpret_cast<const f32x4*>(part_acc + idx * d + 4 * ln);
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[j] += a[j] * w;
    }
  }
  const float inv = 1.0f / L;
  float v[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) v[j] = acc[j] * inv;
  const bool kept = keep.lse2 && t >= keep.tok0 && t < keep.tok0 + keep.n;
  store4(out + (size_t)t * ldo + h * d + 4 * ln, v);
  if (kept) store4((T*)keep.out2 + ((size_t)(t - keep.tok0) * nq + h) * d + 4 * ln, v);
  if (ln == 0) {
    if (lse) lse[(size_t)t * nq + h] = M + __logf(L);
    if (kept) keep.lse2[(size_t)(t - keep.tok0) * nq + h] = M + __logf(L);
  }
}

// ------------------------------------------------------------------------------------------
// window backward (Sec. 6.1): queries = window rows at positions win_start + i, keys/values
// = cached rows [0, l).  P is recomputed from Q, K and the stored log-sum-exp.
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(64) void attn_delta_kernel(const T* __restrict__ out, const T* __restrict__ dout,
                                                        float* __restrict__ delta, int nq, int d) {
  const size_t i = blockIdx.x;
  const int h = blockIdx.y;
  float s = 0.f;
  for (int dd = threadIdx.x; dd < d; dd += 64)
    s += ld(out + (i * nq + h) * d + dd) * ld(dout + (i * nq + h) * d + dd);
  s = wsum(s);
  if (threadIdx.x == 0) delta[i * nq + h] = s;
}

template <typename T>
__global__ __launch_bounds__(64) void attn_bwd_dq_generic_kernel(const T* __restrict__ q, const T* __restrict__ dout,
                                                                 const float* __restrict__ lse,
                                                                 const float* __restrict__ delta,
                                                                 const T* __restrict__ kp, const T* __restrict__ vp,
                                                                 const int32_t* __restrict__ pages,
                                                                 T* __restrict__ dq, int win_start, int nq, int nkv,
                                                                 int d, int ps, float scale) {
  extern __shared__ float smem[];   // q[d], do[d], ds[64]
  float* qs = smem;
  float* dos = smem + d;
  float* dss = smem + 2 * d;
  const size_t i = blockIdx.x;
  const int h = blockIdx.y, lane = threadIdx.x;
  const int group = nq / nkv, kvh = h / group;
  const int p = win_start + (int)i;
  for (int dd = lane; dd < d; dd += 64) {
    qs[dd] = ld(q + (i * nq + h) * d + dd);
    dos[dd] = ld(dout + (i * nq + h) * d + dd);
  }
  const float row_lse = lse[i * nq + h], row_delta = delta[i * nq + h];
  float acc[4] = {0.f, 0.f, 0.f, 0.f};   // d <= 256
  for (int kc = 0; kc <= p; kc += 64) {
    __builtin_amdgcn_wave_barrier();
    const int j = kc + lane;
    float ds = 0.f;
    if (j <= p) {
      const size_t page = pages[j / ps];
      const T* kr = kp + ((page * nkv + kvh) * ps + j % ps) * (size_t)d;
      const T* vr = vp + ((page * nkv + kvh) * (size_t)d) * ps + j % ps;
      float s = 0.f, dp = 0.f;
      for (int dd = 0; dd < d; ++dd) {
        s += qs[dd] * ld(kr + dd);
        dp += dos[dd] * ld(vr + (size_t)dd * ps);
      }
      const float pj = __expf(s * scale - row_lse);
      ds = pj * (dp - row_delta) * scale;
    }
    dss[lane] = ds;
    __builtin_amdgcn_wave_barrier();
    const int nk = min(64, p + 1 - kc);
    for (int jj = 0; jj < nk; ++jj) {
      const int jk = kc + jj;
      const size_t page = pages[jk / ps];
      const T* kr = kp + ((page * nkv + kvh) * ps + jk % ps) * (size_t)d;
      const float w = dss[jj];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (lane + 64 * u < d) acc[u] += w * ld(kr + lane + 64 * u);
    }
  }
#pragma unroll
  for (int u = 0; u < 4; ++u)
    if (lane + 64 * u < d) st(dq + (i * nq + h) * d + lane + 64 * u, acc[u]);
}

// one wave per (key j, kv head): sums over every window row that sees key j and every
// query head of the group; adds into the KV-gradient accumulator rows (Sec. 7).
template <typename T>
__global__ __launch_bounds__(64) void attn_bwd_dkv_generic_kernel(const T* __restrict__ q, const T* __restrict__ dout,
                                                                  const float* __restrict__ lse,
                                                                  const float* __restrict__ delta,
                                                                  const T* __restrict__ kp, const T* __restrict__ vp,
                                                                  const int32_t* __restrict__ pages,
                                                                  float* __restrict__ dk_accum,
                                                                  float* __restrict__ dv_accum, int win_start,
                                                                  int win_len, int nq, int nkv, int d, int ps,
                                                                  float scale) {
  extern __shared__ float smem[];   // k[d], v[d], p[64], ds[64]
  float* ks = smem;
  float* vs = smem + d;
  float* pss = smem + 2 * d;
  float* dss = pss + 64;
  const int j = blockIdx.x, kvh = blockIdx.y, lane = threadIdx.x;
  const int group = nq / nkv;
  const size_t page = pages[j / ps];
  for (int dd = lane; dd < d; dd += 64) {
    ks[dd] = ld(kp + ((page * nkv + kvh) * ps + j % ps) * (size_t)d + dd);
    vs[dd] = ld(vp + ((page * nkv + kvh) * (size_t)d + dd) * ps + j % ps);
  }
  const int i_first = max(0, j - win_start);          // first window row that sees key j
  const int n_pairs = (win_len - i_first) * group;
  float dk[4] = {0.f, 0.f, 0.f, 0.f}, dv[4] = {0.f, 0.f, 0.f, 0.f};
  for (int pc = 0; pc < n_pairs; pc += 64) {
    __builtin_amdgcn_wave_barrier();
    const int pr = pc + lane;
    float pj = 0.f, ds = 0.f;
    if (pr < n_pairs) {
      const size_t i = i_first + pr / group;
      const int h = kvh * group + pr % group;
      const T* qr = q + (i * nq + h) * d;
      const T* dor = dout + (i * nq + h) * d;
      float s = 0.f, dp = 0.f;
      for (int dd = 0; dd < d; ++dd) {
        s += ld(qr + dd) * ks[dd];
        dp += ld(dor + dd) * vs[dd];
      }
      pj = __expf(s * scale - lse[i * nq + h]);
      ds = pj * (dp - delta[i * nq + h]) * scale;
    }
    pss[lane] = pj;
    dss[lane] = ds;
    __builtin_amdgcn_wave_barrier();
    const int np = min(64, n_pairs - pc);
    for (int pp = 0; pp < np; ++pp) {
      const size_t i = i_first + (pc + pp) / group;
      const int h = kvh * group + (pc + pp) % group;
      const float wp = pss[pp], wd = dss[pp];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int dd = lane + 64 * u;
        if (dd < d) {
          dv[u] += wp * ld(dout + (i * nq + h) * d + dd);
          dk[u] += wd * ld(q + (i * nq + h) * d + dd);
        }
      }
    }
  }
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int dd = lane + 64 * u;
    if (dd < d) {
      dk_accum[((size_t)j * nkv + kvh) * d + dd] += dk[u];
      dv_accum[((size_t)j * nkv + kvh) * d + dd] += dv[u];
    }
  }
}

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

int32_t launch_attention_generic(const flexco_layer_cfg& c, const flexco_maps& m, const void* q, size_t ldq,
                                 const flexco_kv_pool& pool, float* part_ml, float* part_acc, hipStream_t s) {
  AttnArgs a;
  a.tok_pos = m.tok_pos; a.block_table = m.block_table; a.tile_req = m.tile_req; a.tile_tok0 = m.tile_tok0;
  a.tile_ntok = m.tile_ntok; a.tile_nsplit = m.tile_nsplit; a.tile_part0 = m.tile_part0; a.item_tile = m.item_tile;
  a.item_split = m.item_split; a.item_ntiles = m.item_ntiles;
  a.max_pages = m.max_pages; a.nq = c.n_q_heads; a.nkv = c.n_kv_heads; a.d = c.head_dim; a.ps = c.page_size;
  a.split_keys = m.kv_split_pages * c.page_size;
  a.cols_per_tile = m.tile_tokens * (c.n_q_heads / c.n_kv_heads);
  a.scale = 1.0f / sqrtf((float)c.head_dim);
  const size_t shm = 4 * sizeof(float) * (size_t)(a.d + a.split_keys);
  if (shm > 64 * 1024) return fail(FLEXCO_EUNSUPPORTED, "kv_split_pages * page_size = %d keys is too large for the generic attention kernel", a.split_keys);
  DISPATCH_T(c.dtype, hipLaunchKernelGGL((attn_fwd_generic_kernel<T>), dim3(m.n_items, c.n_kv_heads, FLEXCO_ATTN_ITEM_TILES), dim3(256), shm,
                                         s, a, (const T*)q, ldq, (const T*)pool.k_pages, (const T*)pool.v_pages,
                                         part_ml, part_acc));
  return post_launch("attn_fwd_generic");
}

int32_t launch_attention_merge(const flexco_layer_cfg& c, const flexco_maps& m, const float* part_ml,
                               const float* part_acc, void* out, size_t ldo, float* lse, hipStream_t s,
                               bool skip_single_split, const AttnKeep* keep_in) {
  AttnKeep keep{nullptr, nullptr, 0, 0};
  if (keep_in) keep = *keep_in;
  const int cpt = m.tile_tokens * (c.n_q_heads / c.n_kv_heads);
  if (c.head_dim == 128 && ((uintptr_t)part_acc & 15) == 0 && ldo % 4 == 0 && ((uintptr_t)out & 15) == 0 &&
      ((uintptr_t)keep.out2 & 15) == 0) {
    DISPATCH_T(c.dtype, hipLaunchKernelGGL((attn_merge128_kernel<T>), dim3(m.T, (c.n_q_heads + 7) / 8), dim3(256), 0, s,
                                           m.tok_tile, m.tile_tok0, m.tile_nsplit, m.tile_part0, part_ml, part_acc, (T*)out,
                                           ldo, lse, c.n_q_heads, c.n_kv_heads, cpt, skip_single_split ? 1 : 0, keep));
    return post_launch("attn_merge");
  }
  DISPATCH_T(c.dtype, hipLaunchKernelGGL((attn_merge_kernel<T>), dim3(m.T, c.n_q_heads), dim3(64), 0, s, m.tok_tile,
                                         m.tile_tok0, m.tile_nsplit, m.tile_part0, part_ml, part_acc, (T*)out, ldo,
                                         lse, c.n_q_heads, c.n_kv_heads, c.head_dim, cpt, skip_single_split ? 1 : 0, keep));
  return post_launch("attn_merge");
}

int32_t launch_attention_delta(const flexco_layer_cfg& c, const void* out, const void* dout, float* delta, int n,
                               hipStream_t s) {
  DISPATCH_T(c.dtype, hipLaunchKernelGGL((attn_delta_kernel<T>), dim3(n, c.n_q_heads), dim3(64), 0, s, (const T*)out,
                                         (const T*)dout, delta, c.n_q_heads, c.head_dim));
  return post_launch("attn_delta");
}

int32_t launch_attention_bwd_generic(const flexco_layer_cfg& c, const flexco_kv_pool& pool, const int32_t* seq_pages,
                                     int win_start, int win_len, const void* q, const float* lse, const float* delta,
                                     const void* dout, void* dq, float* dk_accum, float* dv_accum, hipStream_t s) {
  const float scale = 1.0f / sqrtf((float)c.head_dim);
  const int l = win_start + win_len;
  const size_t shm = sizeof(float) * (2 * (size_t)c.head_dim + 128);
  DISPATCH_T(c.dtype, {
    hipLaunchKernelGGL((attn_bwd_dq_generic_kernel<T>), dim3(win_len, c.n_q_heads), dim3(64), shm, s, (const T*)q,
                       (const T*)dout, lse, delta, (const T*)pool.k_pages, (const T*)pool.v_pages, seq_pages,
                       (T*)dq, win_start, c.n_q_heads, c.n_kv_heads, c.head_dim, c.page_size, scale);
    hipLaunchKernelGGL((attn_bwd_dkv_generic_kernel<T>), dim3(l, c.n_kv_heads), dim3(64), shm, s, (const T*)q,
                       (const T*)dout, lse, delta, (const T*)pool.k_pages, (const T*)pool.v_pages, seq_pages,
                       dk_accum, dv_accum, win_start, win_len, c.n_q_heads, c.n_kv_heads, c.head_dim, c.page_size,
                       scale);
  });
  return post_launch("attn_bwd_generic");
}

}  // namespace flexco

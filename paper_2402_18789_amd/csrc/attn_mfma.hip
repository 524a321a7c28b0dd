// Mixed paged attention on the matrix cores: decode tokens, prefill chunks and finetune
// windows in one launch (Sec. 6.2: finetuning tokens follow the causal pattern of prefill).
//
// bf16 storage, head_dim 128, page_size 16, at most 16 query heads per kv head.
//
// One wavefront = one work item (tile, key split) x kv head.  A tile has up to 16 columns:
// (token, query head of this kv group) pairs - for a decode request the group's heads of its
// single token, for a chunk request tile_tokens tokens x group heads.  All columns share
// every K/V byte the wavefront loads.
//
// The products are laid out so that NO operand ever moves between lanes or through LDS:
//   S^T[key, col]  = K[key, :] . Q[col, :]      v_mfma_f32_16x16x32_bf16, A = K page rows
//       read straight from the page (16 keys x 128 d, key-major), B = Q (registers, loaded once)
//   result: lane (col = lane % 16, g = lane / 16) holds keys 4g..4g+3 of the page.
//   O^T[d, col]   += V^T[d, keys] . P^T[keys, col]  with a k-dimension of 32 = two pages;
//       lane (col, g) supplies P of keys {4g..4g+3 of page 0, 4g..4g+3 of page 1}: exactly
//       the registers the first product left in that lane.  V is stored position-minor
//       ([d][16 positions] per page), so lane (d, g) fetches the matching 4 + 4 positions
//       with two 8-byte loads.
// Online softmax runs per column in the exp2 domain; the running maximum is reduced over the
// four lanes that share a column with two row swaps (no LDS).  Each work item writes an
// un-normalised partial (m, l, acc[128]) per column; a merge kernel combines the splits.
//
// Key positions beyond a column's own position are masked in the scores; positions beyond
// the tile's last position may be unwritten cache slots, so their V bits are cleared as well.
#include "flexco_internal.h"
#include "device_types.h"

namespace flexco {

namespace {

struct FwdArgs {
  const int32_t *tok_pos, *block_table, *tile_req, *tile_tok0, *tile_ntok, *tile_nsplit, *tile_part0, *item_tile,
      *item_split, *item_ntiles;
  int max_pages, nq, nkv, n_items, split_pages;
  float scale_log2;   // log2(e) / sqrt(d)
  // a tile with a single key split needs no merge: its rows go straight to the output
  bf16_t* out;
  size_t ldo;
  float* lse;         // or NULL
  AttnKeep keep;      // second copy of the finetune window's rows
};

constexpr int D = 128, PS = 16;
constexpr int NC_MAX = FLEXCO_ATTN_ITEM_TILES;   // column tiles one work item may carry
constexpr int MAXSP = 256;                   // pages of a key split at most

// A work item carries 1 .. NC neighbouring column tiles of one request (a decode token: one).  The
// wavefront loads every K/V page of the item's key range once and multiplies it against each tile in
// turn: a chunk of 16 / group * NC tokens re-reads its prefix from the caches NC times less often
// than tile by tile.  Each tile keeps its own running maximum, sum and accumulator and its own partial
// row, so the merge kernel sees tiles as before.
// NC = NC_MAX: every item of the work list; NC = 1: the single decode tokens only (the other items go to the
// four-wavefront kernel of attn_chunk_mfma.hip)
template <int NC>
__global__ __launch_bounds__(256) void attn_fwd_mfma_kernel(FwdArgs a, const bf16_t* __restrict__ q, size_t ldq,
                                                            const bf16_t* __restrict__ kp,
                                                            const bf16_t* __restrict__ vp,
                                                            float* __restrict__ part_ml,
                                                            float* __restrict__ part_acc) {
  __shared__ int page_tab[4][MAXSP];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  // consecutive wavefronts take the kv heads of one item: the K (and V) blocks they read are the
  // consecutive 4 KB pieces of the same pages, fetched at about the same time
  const int unit = blockIdx.x * 4 + wave;
  const int item = unit / a.nkv;
  if (item >= a.n_items) return;
  const int kvh = unit % a.nkv;
  const int tile0 = a.item_tile[item], split = a.item_split[item];
  const int ntl = __builtin_amdgcn_readfirstlane(a.item_ntiles[item]);
  if (NC == 1 && !(ntl == 1 && a.tile_ntok[tile0] == 1)) return;
  const int r = a.tile_req[tile0];
  const int group = a.nq / a.nkv;
  const int c = lane & 15, g = lane >> 4;
  // the item's keys: up to the last position of its last tile
  const int tl = tile0 + ntl - 1;
  const int last_pos = a.tok_pos[a.tile_tok0[tl] + a.tile_ntok[tl] - 1];
  const int vis_pages = last_pos / PS + 1;
  const int first_pos = a.tok_pos[a.tile_tok0[tile0]];   // the item's first column sees the fewest keys
  const int pb = split * a.split_pages;
  const int pe = min(pb + a.split_pages, vis_pages);

  // per tile: Q fragments (lane (col, g) holds d = 32 dc + 8 g .. + 8, dc = 0..3), own position, state
  bf16x8 qf[NC][4];
  int pos_c[NC];
  f32x4 o[NC][8];
  float m[NC], l[NC];
#pragma unroll
  for (int cs = 0; cs < NC; ++cs) {
    pos_c[cs] = -1;
    m[cs] = -INFINITY;
    l[cs] = 0.f;
#pragma unroll
    for (int mt = 0; mt < 8; ++mt) o[cs][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (cs < ntl) {
      const int t0 = a.tile_tok0[tile0 + cs], ntok = a.tile_ntok[tile0 + cs];
      const bool col_ok = c < ntok * group;
      const int t_c = col_ok ? t0 + c / group : t0;
      const int h_c = kvh * group + (col_ok ? c % group : 0);
      pos_c[cs] = col_ok ? a.tok_pos[t_c] : -1;
      const bf16_t* qr = q + (size_t)t_c * ldq + h_c * D + g * 8;
#pragma unroll
      for (int dc = 0; dc < 4; ++dc) qf[cs][dc] = *reinterpret_cast<const bf16x8*>(qr + dc * 32);
    }
  }

  bf16x8 kf[2][4];     // [page of the pair][d chunk]
  bf16x4 vf[2][8];     // [page of the pair][d tile]

  // page ids of the whole split in a table of the wavefront's own in LDS (split_pages <= MAXSP; the kernel has no
  // other use for LDS): no dependent load from global memory per step, no registers held for them.  Written and
  // read by this wavefront only, whose LDS operations execute in order: no barrier.
  const int npg = pe - pb;
  int* ptab = page_tab[wave];
#pragma unroll
  for (int q4 = 0; q4 < MAXSP / 64; ++q4)
    if (q4 == 0 || 64 * q4 < npg)   // wavefront-uniform
      ptab[64 * q4 + lane] = a.block_table[(size_t)r * a.max_pages + (64 * q4 + lane < npg ? pb + 64 * q4 + lane : pb)];

  auto load_pair = [&](int rel, bf16x8 (&kk)[2][4], bf16x4 (&vv)[2][8]) {
#pragma unroll
    for (int x = 0; x < 2; ++x) {
      const int pidx = (rel + x < npg) ? rel + x : rel;
      const size_t page = (size_t)__builtin_amdgcn_readfirstlane(ptab[pidx]);   // pidx is wavefront-uniform
      const bf16_t* kpage = kp + ((page * a.nkv + kvh) * PS + c) * (size_t)D + g * 8;
#pragma unroll
      for (int dc = 0; dc < 4; ++dc) kk[x][dc] = *reinterpret_cast<const bf16x8*>(kpage + dc * 32);
      const bf16_t* vpage = vp + ((page * a.nkv + kvh) * (size_t)D + c) * PS + g * 4;
#pragma unroll
      for (int mt = 0; mt < 8; ++mt) vv[x][mt] = *reinterpret_cast<const bf16x4*>(vpage + mt * 16 * PS);
    }
  };

  // one step = 32 keys (two pages) against the columns of every tile, operands in (kf, vf)
  auto step = [&](int pp, bf16x8 (&kf)[2][4], bf16x4 (&vf)[2][8]) {
    // ---- clear V bits of slots past the item's last position (may be unwritten) ----------
    if ((pp + 2) * PS > last_pos + 1) {
#pragma unroll
      for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const bool ok = (pp + x < pe) && ((pp + x) * PS + 4 * g + j <= last_pos);
          if (!ok) {
#pragma unroll
            for (int mt = 0; mt < 8; ++mt) vf[x][mt][j] = (bf16_t)0.f;
          }
        }
    }
    const bool all_visible = (pp + 2) * PS - 1 <= first_pos && pp + 1 < pe;
#pragma unroll
    for (int cs = 0; cs < NC; ++cs) {
      if (cs >= ntl) break;                    // wavefront-uniform
      // ---- scores of 32 keys x 16 columns -------------------------------------------------
      float s[8];
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int dc = 0; dc < 4; ++dc) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[x][dc], qf[cs][dc], acc, 0, 0, 0);
        if (all_visible) {      // wavefront-uniform: both pages lie before every column's own position
#pragma unroll
          for (int j = 0; j < 4; ++j) s[x * 4 + j] = acc[j] * a.scale_log2;
        } else {
          const bool page_ok = pp + x < pe;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int kpos = (pp + x) * PS + 4 * g + j;
            s[x * 4 + j] = (page_ok && kpos <= pos_c[cs]) ? acc[j] * a.scale_log2 : -INFINITY;
          }
        }
      }
      // ---- online softmax per column -------------------------------------------------------
      float mx = s[0];
#pragma unroll
      for (int j = 1; j < 8; ++j) mx = fmaxf(mx, s[j]);
      mx = max_xor16(mx);
      mx = max_xor32(mx);
      const float m_new = fmaxf(m[cs], mx);
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m[cs] - m_use);
      float p[8], psum = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        p[j] = __builtin_amdgcn_exp2f(s[j] - m_use);
        psum += p[j];
      }
      l[cs] = l[cs] * alpha + psum;        // per-lane share of the column's sum; reduced at the end
      m[cs] = m_new;
      bf16x8 pf;
#pragma unroll
      for (int j = 0; j < 8; ++j) pf[j] = (bf16_t)p[j];
      // ---- O^T = alpha O^T + V^T P^T --------------------------------------------------------
      // (skipping the rescaling while no maximum moves - by a branch with the products inside, or, as the chunk
      // kernel does, by an in-place multiplication in a branch of its own - was tried twice here: with four tiles'
      // accumulators the compiler spills 37 - 45 registers and the decode stream slows down by 10 %)
#pragma unroll
      for (int mt = 0; mt < 8; ++mt) {
        bf16x8 vfull;
#pragma unroll
        for (int j = 0; j < 4; ++j) { vfull[j] = vf[0][mt][j]; vfull[4 + j] = vf[1][mt][j]; }
        f32x4 acc = o[cs][mt];
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] *= alpha;
        o[cs][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vfull, pf, acc, 0, 0, 0);
      }
    }
  };

  // Two register sets used in turn: while one pair of pages is multiplied, the next pair is in
  // flight into the other set.  The prefetch is unconditional (past the end it re-reads the current
  // pair, unused), so the number of loads in flight is the same on every path and the wait before a
  // step's MFMAs covers only loads issued one step earlier.
  bf16x8 k1[2][4];
  bf16x4 v1[2][8];
  if (npg > 0) load_pair(0, kf, vf);
  for (int rel = 0; rel < npg; rel += 4) {
    load_pair(rel + 2 < npg ? rel + 2 : rel, k1, v1);
    step(pb + rel, kf, vf);
    load_pair(rel + 4 < npg ? rel + 4 : rel, kf, vf);
    if (rel + 2 < npg) step(pb + rel + 2, k1, v1);
  }
  // ---- write the partial of every (tile, split, kv head) that has this split -------------
  const int cpt = (16 / group > 1 ? 16 / group : 1) * group;
#pragma unroll
  for (int cs = 0; cs < NC; ++cs) {
    if (cs >= ntl) break;
    const int tile = tile0 + cs;
    if (split >= a.tile_nsplit[tile]) continue;   // the tile's own keys end before this split
    float lsum = l[cs];
    lsum = sum_xor16(lsum);
    lsum = sum_xor32(lsum);
    if (a.tile_nsplit[tile] == 1) {   // the whole key range in one split: normalise and write the output rows
      if (c < a.tile_ntok[tile] * group) {
        const int t = a.tile_tok0[tile] + c / group, h = kvh * group + c % group;
        const float inv = 1.0f / lsum;
        bf16_t* po = a.out + (size_t)t * a.ldo + h * D + 4 * g;
#pragma unroll
        for (int mt = 0; mt < 8; ++mt) {
          bf16x4 v;
#pragma unroll
          for (int q = 0; q < 4; ++q) v[q] = (bf16_t)(o[cs][mt][q] * inv);
          *reinterpret_cast<bf16x4*>(po + mt * 16) = v;
        }
        if (a.lse && g == 0) a.lse[(size_t)t * a.nq + h] = m[cs] * 0.6931471805599453f + __logf(lsum);
        if (a.keep.lse2 && t >= a.keep.tok0 && t < a.keep.tok0 + a.keep.n) {
          bf16_t* p2 = (bf16_t*)a.keep.out2 + ((size_t)(t - a.keep.tok0) * a.nq + h) * D + 4 * g;
#pragma unroll
          for (int mt = 0; mt < 8; ++mt) {
            bf16x4 v;
#pragma unroll
            for (int q = 0; q < 4; ++q) v[q] = (bf16_t)(o[cs][mt][q] * inv);
            *reinterpret_cast<bf16x4*>(p2 + mt * 16) = v;
          }
          if (g == 0) a.keep.lse2[(size_t)(t - a.keep.tok0) * a.nq + h] = m[cs] * 0.6931471805599453f + __logf(lsum);
        }
      }
      continue;
    }
    if (c < a.tile_ntok[tile] * group) {
      const size_t idx = ((size_t)(a.tile_part0[tile] + split) * a.nkv + kvh) * cpt + c;
      if (g == 0) {
        part_ml[idx * 2] = m[cs] * 0.6931471805599453f;     // back to the natural-log domain
        part_ml[idx * 2 + 1] = lsum;
      }
      float* pa = part_acc + idx * D + 4 * g;
#pragma unroll
      for (int mt = 0; mt < 8; ++mt) *reinterpret_cast<f32x4*>(pa + mt * 16) = o[cs][mt];
    }
  }
}

}  // namespace

int32_t launch_attention_mfma(const flexco_layer_cfg& c, const flexco_maps& m, const void* q, size_t ldq,
                              const flexco_kv_pool& pool, float* part_ml, float* part_acc, void* out, size_t ldo,
                              float* lse, hipStream_t s, const AttnKeep* keep, bool skip_chunk, bool nothing_to_do) {
  const int group = c.n_q_heads / c.n_kv_heads;
  if (c.dtype != FLEXCO_BF16 || c.head_dim != D || c.page_size != PS || group > 16 || ldq % 8 != 0 ||
      m.kv_split_pages > MAXSP || ldo % 4 != 0 || ((uintptr_t)out & 7))
    return FLEXCO_EUNSUPPORTED;
  if (nothing_to_do) return FLEXCO_OK;
  FwdArgs a;
  a.tok_pos = m.tok_pos; a.block_table = m.block_table; a.tile_req = m.tile_req; a.tile_tok0 = m.tile_tok0;
  a.tile_ntok = m.tile_ntok; a.tile_nsplit = m.tile_nsplit; a.tile_part0 = m.tile_part0; a.item_tile = m.item_tile;
  a.item_split = m.item_split; a.item_ntiles = m.item_ntiles;
  a.max_pages = m.max_pages; a.nq = c.n_q_heads; a.nkv = c.n_kv_heads; a.n_items = m.n_items;
  a.split_pages = m.kv_split_pages;
  a.scale_log2 = 1.4426950408889634f / sqrtf((float)D);
  a.out = (bf16_t*)out; a.ldo = ldo; a.lse = lse;
  a.keep = keep ? *keep : AttnKeep{nullptr, nullptr, 0, 0};
  if (skip_chunk)
    hipLaunchKernelGGL(attn_fwd_mfma_kernel<1>, dim3((m.n_items * c.n_kv_heads + 3) / 4), dim3(256), 0, s, a,
                       (const bf16_t*)q, ldq, (const bf16_t*)pool.k_pages, (const bf16_t*)pool.v_pages, part_ml, part_acc);
  else
    hipLaunchKernelGGL(attn_fwd_mfma_kernel<NC_MAX>, dim3((m.n_items * c.n_kv_heads + 3) / 4), dim3(256), 0, s, a,
                       (const bf16_t*)q, ldq, (const bf16_t*)pool.k_pages, (const bf16_t*)pool.v_pages, part_ml, part_acc);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(FLEXCO_EHIP, "launch of attn_fwd_mfma failed: %s", hipGetErrorString(e));
  return FLEXCO_OK;
}

}  // namespace flexco

// Mixed paged attention, the chunk items on their own: prefill chunks and finetune windows whose rows are many
// (Sec. 6.2: finetuning tokens follow the causal pattern of prefill).
//
// The one-launch kernel of attn_mfma.hip gives a work item - up to four column tiles of one request x one key
// split - to ONE wavefront, which fetches K / V pages from global memory into registers and multiplies them
// against its tiles one after the other.  That suits the decode stream (one tile per item, the time is HBM's).
// For long windows the time is the wavefront's own chain of products and exponentials per tile, four tiles deep,
// with one wavefront per SIMD to run it.  Here the same item goes to a BLOCK of four wavefronts, one tile each:
// the K / V pages of a step are staged once per block in LDS (straight from global memory, a ring of four stages
// of two pages) and every wavefront reads its operands from there; 64 KB of LDS and under 256 registers put two
// blocks on a CU.  The same products per tile and the same form of partial rows and direct outputs as the one-launch
// kernel, so the merge kernel and everything after see no difference; the reference point of a column's
// exponentials may lag its running maximum here (LAZY below), which moves results by rounding only.
//
// bf16, head_dim 128, page_size 16, at most 16 query heads per kv head.
#include "flexco_internal.h"
#include "device_types.h"

namespace flexco {

namespace {

constexpr int D = 128, PS = 16;
constexpr int PAGE_EL = PS * D;          // elements of one K page-head block (16 keys x 128) = of one V block (128 x 16)
constexpr int STAGE_EL = 4 * PAGE_EL;    // K page 0 | K page 1 | V page 0 | V page 1
constexpr int MAXSP = 256;               // pages of a key split at most
constexpr float LAZY = 8.f;              // how far (log2) a column's maximum may run ahead of its reference point
#define FLEXCO_GP(p) ((const __attribute__((address_space(1))) void*)(p))
#define FLEXCO_LP(p) ((__attribute__((address_space(3))) void*)(p))

struct ChunkArgs {
  const int32_t *tok_pos, *block_table, *tile_req, *tile_tok0, *tile_ntok, *tile_nsplit, *tile_part0, *item_tile,
      *item_split, *item_ntiles;
  int max_pages, nq, nkv, n_items, split_pages;
  float scale_log2;   // log2(e) / sqrt(d)
  bf16_t* out;
  size_t ldo;
  float* lse;         // or NULL
  AttnKeep keep;
};

// K rows in LDS ([16 keys][128] bf16, 256-byte rows): chunk cc of row r is stored at chunk cc ^ rsw(r), so that the
// ds_read_b128 of lane (key = lane % 16, g = lane / 16) - served 16 lanes a cycle in quads {0-3, 12-15, 20-23, 24-27},
// {4-7, 8-11, 16-19, 28-31} (+32) - touches 16 different chunks per cycle.
__device__ inline int rsw(int r) { return (((r + ((r >> 3) << 2)) & 7) << 1) | ((r >> 3) & 1); }

// One 8-byte LDS read that stays one: left to itself the compiler pairs the reads of two d tiles, 512 bytes apart,
// into a ds_read2st64_b64, whose two halves meet in the same banks (counted: 39 % of this kernel's LDS cycles were
// bank conflicts, all from these reads).  A volatile access is not merged and is still tracked by the compiler's waits.
__device__ inline bf16x4 lds_read_8(const bf16_t* p) {
  typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
  const u32x2 v = *(const volatile __attribute__((address_space(3))) u32x2*)FLEXCO_LP(p);
  return __builtin_bit_cast(bf16x4, v);
}

// RING = stages of the K / V ring.  4: 65 KB of LDS, two blocks per CU, two stages of loads in flight - the form that
// runs beside the decode tokens' kernel.  3: 49 KB and at most 168 registers, three blocks per CU, one stage in flight -
// 7 - 10 % faster when the kernel has the chip to itself (three wavefronts per SIMD fill each other's waits), no
// better beside the decode stream, which it crowds out of the CUs.
template <int RING>
__global__ __launch_bounds__(256, RING == 3 ? 3 : 2) void attn_fwd_chunk_kernel(ChunkArgs a, const bf16_t* __restrict__ q, size_t ldq,
                                                                const bf16_t* __restrict__ kp,
                                                                const bf16_t* __restrict__ vp,
                                                                float* __restrict__ part_ml,
                                                                float* __restrict__ part_acc) {
  __shared__ __attribute__((aligned(1024))) bf16_t ring0[STAGE_EL];
  __shared__ __attribute__((aligned(1024))) bf16_t ring1[STAGE_EL];
  __shared__ __attribute__((aligned(1024))) bf16_t ring2[STAGE_EL];
  __shared__ __attribute__((aligned(1024))) bf16_t ring3[RING == 4 ? STAGE_EL : 8];
  __shared__ int page_tab[MAXSP];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int item = blockIdx.x / a.nkv, kvh = blockIdx.x % a.nkv;
  const int tile0 = a.item_tile[item], split = a.item_split[item];
  const int ntl = a.item_ntiles[item];
  if (ntl == 1 && a.tile_ntok[tile0] == 1) return;   // a decode token: the one-launch kernel's (whole block, before any barrier)
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
  const int npg = pe - pb;                               // >= 1: an item exists for splits inside the visible range only
  page_tab[tid] = a.block_table[(size_t)r * a.max_pages + (tid < npg ? pb + tid : pb)];   // MAXSP = block size
  __syncthreads();

  // this wavefront's tile (wavefronts past the item's last tile only help with the loads and the barriers)
  const bool have = wave < ntl;
  const int tile = tile0 + (have ? wave : 0);
  bf16x8 qf[4];
  int pos_c = -1;
  f32x4 o[8];
  float m = -INFINITY, l = 0.f;
#pragma unroll
  for (int mt = 0; mt < 8; ++mt) o[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
  {
    const int t0 = a.tile_tok0[tile], ntok = a.tile_ntok[tile];
    const bool col_ok = have && c < ntok * group;
    const int t_c = col_ok ? t0 + c / group : t0;
    const int h_c = kvh * group + (col_ok ? c % group : 0);
    pos_c = col_ok ? a.tok_pos[t_c] : -1;
    const bf16_t* qr = q + (size_t)t_c * ldq + h_c * D + g * 8;
#pragma unroll
    for (int dc = 0; dc < 4; ++dc) qf[dc] = *reinterpret_cast<const bf16x8*>(qr + dc * 32);
  }

  // ---- tile loads: a stage = the two pages 2 st, 2 st + 1 of the split; wavefront w brings in, of each page, K rows
  // 4 w .. 4 w + 3 (lane -> row 4 w + lane / 16, physical chunk lane % 16) and the V chunks 64 w .. 64 w + 63 of the
  // page's 256 (a V page is [128 d][16 keys]: 32-byte rows, two chunks; physical chunk P holds logical chunk
  // P ^ (bit 4 of P), which swaps the halves of rows d = 8 .. 15 (mod 16) so that the 8-byte reads of 32 lanes - 16
  // rows, the same half of each - cover all banks).  Past the last stage the loads repeat it into a free buffer:
  // the count of loads in flight stays what the waits assume.
  const int nst = (npg + 1) / 2;
  const int k_row = 4 * wave + (lane >> 4);
  const int k_src = k_row * D + (((lane & 15) ^ rsw(k_row)) * 8);
  const int v_p = 64 * wave + lane;
  const int v_src = (v_p ^ ((v_p >> 4) & 1)) * 8;
#define FLEXCO_CH_ISSUE(ring_, st_)                                                                   \
  {                                                                                                   \
    const int s2_ = 2 * min((st_), nst - 1);                                                          \
    _Pragma("unroll") for (int x = 0; x < 2; ++x) {                                                   \
      const size_t page_ = (size_t)__builtin_amdgcn_readfirstlane(page_tab[min(s2_ + x, npg - 1)]);   \
      const bf16_t* kb_ = kp + (page_ * a.nkv + kvh) * (size_t)PAGE_EL;                               \
      const bf16_t* vb_ = vp + (page_ * a.nkv + kvh) * (size_t)PAGE_EL;                               \
      __builtin_amdgcn_global_load_lds(FLEXCO_GP(kb_ + k_src), FLEXCO_LP(ring_ + x * PAGE_EL + wave * 512), 16, 0, 0); \
      __builtin_amdgcn_global_load_lds(FLEXCO_GP(vb_ + v_src), FLEXCO_LP(ring_ + (2 + x) * PAGE_EL + wave * 512), 16, 0, 0); \
    }                                                                                                 \
  }
  // wait until this wavefront's loads of all stages but the last LATEST_ issued have landed (4 loads each), then a
  // barrier without memory fences
#define FLEXCO_CH_WAIT_BARRIER(LATEST_)                     \
  {                                                         \
    __builtin_amdgcn_s_waitcnt(0x0F70 | (4 * (LATEST_)));   \
    asm volatile("" ::: "memory");                          \
    __builtin_amdgcn_s_barrier();                           \
    asm volatile("" ::: "memory");                          \
  }

  // ---- operand fetches of one stage: K rows as A operand of S^T = K Q^T, lane (key c, g): d = 32 dc + 8 g .. + 8;
  // V as A operand of O^T += V^T P^T, lane (d = 16 mt + c, g): keys 4 g .. 4 g + 3 of each page
  const int kr_off = c * D;
  const int kr_sw = rsw(c);
  const int vr_off = ((2 * c + (g >> 1)) ^ ((c >> 3) & 1)) * 8 + (g & 1) * 4;   // + 256 elements (32 chunks) per d tile mt

  // A step = 32 keys (two pages) against the 16 columns of this wavefront's tile, in two halves that run one stage
  // apart: the score products of stage st + 1 are issued before the softmax of stage st, so that the matrix cores
  // work through them while the vector ALU does the maxima, exponentials and conversions.
  // first half: raw scores (before scale and mask) of the stage in ring_, into sc_[page]
#define FLEXCO_CH_SCORES(ring_, sc_)                                                                  \
  {                                                                                                   \
    bf16x8 kf[2][4];                                                                                  \
    _Pragma("unroll") for (int x = 0; x < 2; ++x)                                                     \
      _Pragma("unroll") for (int dc = 0; dc < 4; ++dc)                                                \
        kf[x][dc] = *reinterpret_cast<const bf16x8*>(ring_ + x * PAGE_EL + kr_off + (((dc * 4 + g) ^ kr_sw) * 8)); \
    _Pragma("unroll") for (int x = 0; x < 2; ++x) {                                                   \
      sc_[x] = f32x4{0.f, 0.f, 0.f, 0.f};                                                             \
      _Pragma("unroll") for (int dc = 0; dc < 4; ++dc)                                                \
        sc_[x] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[x][dc], qf[dc], sc_[x], 0, 0, 0);         \
    }                                                                                                 \
  }
  // second half: softmax of the scores sc_ of stage st_ and O^T += V^T P^T with the stage's V
  // V operands per d tile: keys 4 g .. 4 g + 3 of page 0 | of page 1, as the product takes them
#define FLEXCO_CH_LOAD_V(ring_, vf_)                                                                  \
    _Pragma("unroll") for (int mt = 0; mt < 8; ++mt)                                                  \
      vf_[mt] = __builtin_shufflevector(lds_read_8(ring_ + 2 * PAGE_EL + mt * 256 + vr_off),          \
                                        lds_read_8(ring_ + 3 * PAGE_EL + mt * 256 + vr_off), 0, 1, 2, 3, 4, 5, 6, 7);
#define FLEXCO_CH_PV(vf_, pf_, alpha_)                                                                \
    _Pragma("unroll") for (int mt = 0; mt < 8; ++mt) {                                                \
      f32x4 acc = o[mt];                                                                              \
      _Pragma("unroll") for (int j = 0; j < 4; ++j) acc[j] *= alpha_;                                 \
      o[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf_[mt], pf_, acc, 0, 0, 0);                    \
    }
  // ... of a stage that lies wholly before every column's own position (most stages of a long window): no masks, no
  // clearing of unwritten V slots, no branch - one basic block per step, which the compiler may order as it likes and
  // which keeps the accumulators where they are (every branch in a step cost a copy of all 32 of them at its end)
#define FLEXCO_CH_SOFTMAX_PV_VISIBLE(ring_, sc_)                                                      \
  {                                                                                                   \
    bf16x8 vf[8];                                                                                     \
    FLEXCO_CH_LOAD_V(ring_, vf)                                                                       \
    float s[8];                                                                                       \
    _Pragma("unroll") for (int x = 0; x < 2; ++x)                                                     \
      _Pragma("unroll") for (int j = 0; j < 4; ++j) s[x * 4 + j] = sc_[x][j] * a.scale_log2;          \
    float mx = s[0];                                                                                  \
    _Pragma("unroll") for (int j = 1; j < 8; ++j) mx = fmaxf(mx, s[j]);                               \
    mx = max_xor16(mx);                                                                               \
    mx = max_xor32(mx);                                                                               \
    /* The reference point m of a column's exponentials need not be its running maximum: any m gives the same */ \
    /* row after the final division by l.  It follows the maximum only when that has moved up by more than    */ \
    /* LAZY (exponentials then stay below 2^LAZY: no overflow, same relative rounding in bf16), so that the    */ \
    /* accumulators are rescaled in few steps - in place, inside a branch the wavefront takes as one - instead */ \
    /* of in every step (32 of a step's 80 vector instructions).                                              */ \
    if (__builtin_amdgcn_ballot_w64(mx > m + LAZY) != 0) {                                            \
      const float m_upd = mx > m + LAZY ? mx : m;                                                     \
      const float alpha = __builtin_amdgcn_exp2f(m - m_upd);                                          \
      l *= alpha;                                                                                     \
      m = m_upd;                                                                                      \
      _Pragma("unroll") for (int mt = 0; mt < 8; ++mt)                                                \
        _Pragma("unroll") for (int j = 0; j < 4; ++j) o[mt][j] *= alpha;                              \
    }                                                                                                 \
    float p[8], psum = 0.f;                                                                           \
    _Pragma("unroll") for (int j = 0; j < 8; ++j) {                                                   \
      p[j] = __builtin_amdgcn_exp2f(s[j] - m);                                                        \
      psum += p[j];                                                                                   \
    }                                                                                                 \
    l += psum;                                                                                        \
    bf16x8 pf;                                                                                        \
    _Pragma("unroll") for (int j = 0; j < 8; ++j) pf[j] = (bf16_t)p[j];                               \
    _Pragma("unroll") for (int mt = 0; mt < 8; ++mt)                                                  \
      o[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[mt], pf, o[mt], 0, 0, 0);                    \
  }
  // ... of any stage
#define FLEXCO_CH_SOFTMAX_PV(ring_, st_, sc_)                                                         \
  {                                                                                                   \
    const int pp = pb + 2 * (st_);                                                                    \
    bf16x8 vf[8];                                                                                     \
    FLEXCO_CH_LOAD_V(ring_, vf)                                                                       \
    /* V bits of slots past the item's last position may be unwritten memory */                       \
    if ((pp + 2) * PS > last_pos + 1) {                                                               \
      _Pragma("unroll") for (int x = 0; x < 2; ++x)                                                   \
        _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                               \
          const bool ok = (pp + x < pe) && ((pp + x) * PS + 4 * g + j <= last_pos);                   \
          if (!ok) {                                                                                  \
            _Pragma("unroll") for (int mt = 0; mt < 8; ++mt) vf[mt][4 * x + j] = (bf16_t)0.f;         \
          }                                                                                           \
        }                                                                                             \
    }                                                                                                 \
    float s[8];                                                                                       \
    _Pragma("unroll") for (int x = 0; x < 2; ++x) {                                                   \
      const bool page_ok = pp + x < pe;                                                               \
      _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                                 \
        const int kpos = (pp + x) * PS + 4 * g + j;                                                   \
        s[x * 4 + j] = (page_ok && kpos <= pos_c) ? sc_[x][j] * a.scale_log2 : -INFINITY;             \
      }                                                                                               \
    }                                                                                                 \
    float mx = s[0];                                                                                  \
    _Pragma("unroll") for (int j = 1; j < 8; ++j) mx = fmaxf(mx, s[j]);                               \
    mx = max_xor16(mx);                                                                               \
    mx = max_xor32(mx);                                                                               \
    const float m_new = fmaxf(m, mx);                                                                 \
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;                                           \
    const float alpha = __builtin_amdgcn_exp2f(m - m_use);                                            \
    float p[8], psum = 0.f;                                                                           \
    _Pragma("unroll") for (int j = 0; j < 8; ++j) {                                                   \
      p[j] = __builtin_amdgcn_exp2f(s[j] - m_use);                                                    \
      psum += p[j];                                                                                   \
    }                                                                                                 \
    l = l * alpha + psum;                                                                             \
    m = m_new;                                                                                        \
    bf16x8 pf;                                                                                        \
    _Pragma("unroll") for (int j = 0; j < 8; ++j) pf[j] = (bf16_t)p[j];                               \
    FLEXCO_CH_PV(vf, pf, alpha)                                                                       \
  }
  // step st (cur_ holds stage st, next_ stage st + 1, free_ held stage st - 1): my loads of stage st + 1 have landed
  // (those of stage st + 2 may be in flight) -> barrier -> everyone's have, and everyone is done with stage st - 1 ->
  // start the loads of stage st + 3 into its buffer -> scores of stage st + 1 -> softmax and V products of stage st.
  // Every form of a step has this one barrier, so the wavefronts of a block may each be in a loop of their own.
#define FLEXCO_CH_STEP_VISIBLE(cur_, next_, free_, st_, sc_cur_, sc_next_)                            \
  {                                                                                                   \
    FLEXCO_CH_WAIT_BARRIER(RING - 3)                                                                  \
    FLEXCO_CH_ISSUE(free_, (st_) + RING - 1)                                                          \
    FLEXCO_CH_SCORES(next_, sc_next_)                                                                 \
    FLEXCO_CH_SOFTMAX_PV_VISIBLE(cur_, sc_cur_)                                                       \
  }
#define FLEXCO_CH_STEP(cur_, next_, free_, st_, sc_cur_, sc_next_)                                    \
  {                                                                                                   \
    FLEXCO_CH_WAIT_BARRIER(RING - 3)                                                                  \
    FLEXCO_CH_ISSUE(free_, (st_) + RING - 1)                                                          \
    if ((st_) + 1 < nst) FLEXCO_CH_SCORES(next_, sc_next_)                                            \
    FLEXCO_CH_SOFTMAX_PV(cur_, st_, sc_cur_)                                                          \
  }
#define FLEXCO_CH_STEP_IDLE(free_, st_)                                                               \
  {                                                                                                   \
    FLEXCO_CH_WAIT_BARRIER(RING - 3)                                                                  \
    FLEXCO_CH_ISSUE(free_, (st_) + RING - 1)                                                          \
  }
  // three buffers: step st reads V of stage st in ring[st % 3] and K of stage st + 1 in ring[(st + 1) % 3] and refills
  // ring[(st + 2) % 3]; with the two score buffers in turn the pattern repeats every six steps
#define FLEXCO_CH_SIX(STEP_, st_)                                     \
      STEP_(ring0, ring1, ring2, (st_), sc_a, sc_b)                   \
      STEP_(ring1, ring2, ring0, (st_) + 1, sc_b, sc_a)               \
      STEP_(ring2, ring0, ring1, (st_) + 2, sc_a, sc_b)               \
      STEP_(ring0, ring1, ring2, (st_) + 3, sc_b, sc_a)               \
      STEP_(ring1, ring2, ring0, (st_) + 4, sc_a, sc_b)               \
      STEP_(ring2, ring0, ring1, (st_) + 5, sc_b, sc_a)
  if constexpr (RING == 4) {
    FLEXCO_CH_ISSUE(ring0, 0)
    FLEXCO_CH_ISSUE(ring1, 1)
    FLEXCO_CH_ISSUE(ring2, 2)
    FLEXCO_CH_WAIT_BARRIER(2)        // stage 0 is there
    int st = 0;
    if (have) {
      f32x4 sc_a[2], sc_b[2];
      FLEXCO_CH_SCORES(ring0, sc_a)
      // leading stages wholly before the item's first position and inside the split, in fours (the ring's period),
      // and never the last stage (the visible form computes the next stage's scores without asking)
      const int n_vis = max(min((first_pos + 1) / PS - pb, npg), 0) / 2;
      const int n_vis4 = min(n_vis, nst - 1) & ~3;
      for (; st < n_vis4; st += 4) {
        FLEXCO_CH_STEP_VISIBLE(ring0, ring1, ring3, st, sc_a, sc_b)
        FLEXCO_CH_STEP_VISIBLE(ring1, ring2, ring0, st + 1, sc_b, sc_a)
        FLEXCO_CH_STEP_VISIBLE(ring2, ring3, ring1, st + 2, sc_a, sc_b)
        FLEXCO_CH_STEP_VISIBLE(ring3, ring0, ring2, st + 3, sc_b, sc_a)
      }
      for (; st + 3 < nst; st += 4) {
        FLEXCO_CH_STEP(ring0, ring1, ring3, st, sc_a, sc_b)
        FLEXCO_CH_STEP(ring1, ring2, ring0, st + 1, sc_b, sc_a)
        FLEXCO_CH_STEP(ring2, ring3, ring1, st + 2, sc_a, sc_b)
        FLEXCO_CH_STEP(ring3, ring0, ring2, st + 3, sc_b, sc_a)
      }
      if (st < nst) FLEXCO_CH_STEP(ring0, ring1, ring3, st, sc_a, sc_b)
      if (st + 1 < nst) FLEXCO_CH_STEP(ring1, ring2, ring0, st + 1, sc_b, sc_a)
      if (st + 2 < nst) FLEXCO_CH_STEP(ring2, ring3, ring1, st + 2, sc_a, sc_b)
    } else {
      for (; st + 3 < nst; st += 4) {
        FLEXCO_CH_STEP_IDLE(ring3, st)
        FLEXCO_CH_STEP_IDLE(ring0, st + 1)
        FLEXCO_CH_STEP_IDLE(ring1, st + 2)
        FLEXCO_CH_STEP_IDLE(ring2, st + 3)
      }
      if (st < nst) FLEXCO_CH_STEP_IDLE(ring3, st)
      if (st + 1 < nst) FLEXCO_CH_STEP_IDLE(ring0, st + 1)
      if (st + 2 < nst) FLEXCO_CH_STEP_IDLE(ring1, st + 2)
    }
  } else {
    FLEXCO_CH_ISSUE(ring0, 0)
    FLEXCO_CH_ISSUE(ring1, 1)
    FLEXCO_CH_WAIT_BARRIER(1)        // stage 0 is there
    int st = 0;
    if (have) {
      f32x4 sc_a[2], sc_b[2];
      FLEXCO_CH_SCORES(ring0, sc_a)
      const int n_vis = max(min((first_pos + 1) / PS - pb, npg), 0) / 2;
      const int n_vis6 = (min(n_vis, nst - 1) / 6) * 6;
      for (; st < n_vis6; st += 6) { FLEXCO_CH_SIX(FLEXCO_CH_STEP_VISIBLE, st) }
      for (; st + 5 < nst; st += 6) { FLEXCO_CH_SIX(FLEXCO_CH_STEP, st) }
      if (st < nst) FLEXCO_CH_STEP(ring0, ring1, ring2, st, sc_a, sc_b)
      if (st + 1 < nst) FLEXCO_CH_STEP(ring1, ring2, ring0, st + 1, sc_b, sc_a)
      if (st + 2 < nst) FLEXCO_CH_STEP(ring2, ring0, ring1, st + 2, sc_a, sc_b)
      if (st + 3 < nst) FLEXCO_CH_STEP(ring0, ring1, ring2, st + 3, sc_b, sc_a)
      if (st + 4 < nst) FLEXCO_CH_STEP(ring1, ring2, ring0, st + 4, sc_a, sc_b)
    } else {
      for (; st + 2 < nst; st += 3) {
        FLEXCO_CH_STEP_IDLE(ring2, st)
        FLEXCO_CH_STEP_IDLE(ring0, st + 1)
        FLEXCO_CH_STEP_IDLE(ring1, st + 2)
      }
      if (st < nst) FLEXCO_CH_STEP_IDLE(ring2, st)
      if (st + 1 < nst) FLEXCO_CH_STEP_IDLE(ring0, st + 1)
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);   // nothing may land in LDS after the block ends

  // ---- write the tile's partial, or - the whole key range in one split - its output rows ---------------------
  if (!have) return;
  if (split >= a.tile_nsplit[tile]) return;   // the tile's own keys end before this split
  const int cpt = (16 / group > 1 ? 16 / group : 1) * group;
  float lsum = l;
  lsum = sum_xor16(lsum);
  lsum = sum_xor32(lsum);
  if (c >= a.tile_ntok[tile] * group) return;
  if (a.tile_nsplit[tile] == 1) {
    const int t = a.tile_tok0[tile] + c / group, h = kvh * group + c % group;
    const float inv = 1.0f / lsum;
    bf16_t* po = a.out + (size_t)t * a.ldo + h * D + 4 * g;
#pragma unroll
    for (int mt = 0; mt < 8; ++mt) {
      bf16x4 v;
#pragma unroll
      for (int qq = 0; qq < 4; ++qq) v[qq] = (bf16_t)(o[mt][qq] * inv);
      *reinterpret_cast<bf16x4*>(po + mt * 16) = v;
    }
    if (a.lse && g == 0) a.lse[(size_t)t * a.nq + h] = m * 0.6931471805599453f + __logf(lsum);
    if (a.keep.lse2 && t >= a.keep.tok0 && t < a.keep.tok0 + a.keep.n) {
      bf16_t* p2 = (bf16_t*)a.keep.out2 + ((size_t)(t - a.keep.tok0) * a.nq + h) * D + 4 * g;
#pragma unroll
      for (int mt = 0; mt < 8; ++mt) {
        bf16x4 v;
#pragma unroll
        for (int qq = 0; qq < 4; ++qq) v[qq] = (bf16_t)(o[mt][qq] * inv);
        *reinterpret_cast<bf16x4*>(p2 + mt * 16) = v;
      }
      if (g == 0) a.keep.lse2[(size_t)(t - a.keep.tok0) * a.nq + h] = m * 0.6931471805599453f + __logf(lsum);
    }
    return;
  }
  const size_t idx = ((size_t)(a.tile_part0[tile] + split) * a.nkv + kvh) * cpt + c;
  if (g == 0) {
    part_ml[idx * 2] = m * 0.6931471805599453f;     // back to the natural-log domain
    part_ml[idx * 2 + 1] = lsum;
  }
  float* pa = part_acc + idx * D + 4 * g;
#pragma unroll
  for (int mt = 0; mt < 8; ++mt) *reinterpret_cast<f32x4*>(pa + mt * 16) = o[mt];
}

}  // namespace

// The chunk items of the work list (everything but single decode tokens) on the four-wavefront kernel; the caller
// has the one-launch kernel skip them.  Same support test as launch_attention_mfma.  alone: no other kernel of the
// call runs beside this one (the work list has no decode token).
int32_t launch_attention_chunk_mfma(const flexco_layer_cfg& c, const flexco_maps& m, const void* q, size_t ldq,
                                    const flexco_kv_pool& pool, float* part_ml, float* part_acc, void* out, size_t ldo,
                                    float* lse, hipStream_t s, const AttnKeep* keep, bool alone) {
  const int group = c.n_q_heads / c.n_kv_heads;
  if (c.dtype != FLEXCO_BF16 || c.head_dim != D || c.page_size != PS || group > 16 || ldq % 8 != 0 ||
      m.kv_split_pages > MAXSP || ldo % 4 != 0 || ((uintptr_t)out & 7))
    return FLEXCO_EUNSUPPORTED;
  if (m.n_items == 0) return FLEXCO_OK;
  ChunkArgs a;
  a.tok_pos = m.tok_pos; a.block_table = m.block_table; a.tile_req = m.tile_req; a.tile_tok0 = m.tile_tok0;
  a.tile_ntok = m.tile_ntok; a.tile_nsplit = m.tile_nsplit; a.tile_part0 = m.tile_part0; a.item_tile = m.item_tile;
  a.item_split = m.item_split; a.item_ntiles = m.item_ntiles;
  a.max_pages = m.max_pages; a.nq = c.n_q_heads; a.nkv = c.n_kv_heads; a.n_items = m.n_items;
  a.split_pages = m.kv_split_pages;
  a.scale_log2 = 1.4426950408889634f / sqrtf((float)D);
  a.out = (bf16_t*)out; a.ldo = ldo; a.lse = lse;
  a.keep = keep ? *keep : AttnKeep{nullptr, nullptr, 0, 0};
  if (alone)
    hipLaunchKernelGGL(attn_fwd_chunk_kernel<3>, dim3((unsigned)m.n_items * c.n_kv_heads), dim3(256), 0, s, a,
                       (const bf16_t*)q, ldq, (const bf16_t*)pool.k_pages, (const bf16_t*)pool.v_pages, part_ml,
                       part_acc);
  else
    hipLaunchKernelGGL(attn_fwd_chunk_kernel<4>, dim3((unsigned)m.n_items * c.n_kv_heads), dim3(256), 0, s, a,
                       (const bf16_t*)q, ldq, (const bf16_t*)pool.k_pages, (const bf16_t*)pool.v_pages, part_ml,
                       part_acc);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(FLEXCO_EHIP, "launch of attn_fwd_chunk failed: %s", hipGetErrorString(e));
  return FLEXCO_OK;
}

}  // namespace flexco

// Internal declarations shared by the host API and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <stddef.h>

#include "flexco_host.h"
#include "device_types.h"

namespace flexco {

// ---- argument blocks of the bf16 LoRA kernels (up to 3 matrices per launch, grid.z) ----------
constexpr int LORA_MATS = 7;   // matrices one LoRA launch can batch: one per target (q, k, v, o, gate, up, down)
constexpr int LORA_SLOTS = 12;   // products of one shrink launch: (target, adapter) pairs or the 7 targets
struct LoraShrinkArgs {     // out[z][row][rank] = sum_k X[z][row, k] S[z][rank, k]   (skinny product with a rank-r matrix)
  const bf16_t* X[LORA_SLOTS]; size_t ldx[LORA_SLOTS];
  const bf16_t* S[LORA_SLOTS]; size_t lds[LORA_SLOTS];
  int K[LORA_SLOTS];                 // contracted width, per matrix
  float* out_f32[LORA_SLOTS];        // or NULL: rows [f32_lo, f32_hi) are written, row m at out_f32[(m - f32_lo) * r ..]
  bf16_t* out_ext[LORA_SLOTS];       // [rows, r], scaled by `scale`, or NULL (operand of the GEMM extension)
  // [rows] or NULL: adapter id per row.  A row takes part in product z iff its id is >= 0 and, where
  // want[z] >= 0, equals want[z]; the out_ext rows of the others are zero, their out_f32 rows untouched.
  const int32_t* row_adapter;
  int want[LORA_SLOTS];
  int rows, r;
  int f32_lo, f32_hi;
  float scale;
  // optional scratch of LORA_SHRINK_SPLITS * part_slots * rows * r floats: long contractions are then cut
  // over several blocks per row tile, whose partial products a second kernel adds in block order
  float* part;
  int part_slots;           // products the scratch is sized for
  int ksplit;               // set by the launcher
  int relu;                 // bit z set: product z passes through max(., 0) before it is written (bottleneck adapters)
};
constexpr int LORA_SHRINK_SPLITS = 8;
// t[i] <- 0 where u[i] <= 0 (the ReLU's backward mask, u = the ReLU's output); t_ext[i] = bf16(t[i])
int32_t launch_relu_bwd_mask(const float* u, float* t, void* t_ext, size_t count, hipStream_t s);
struct LoraTransposeArgs { const bf16_t* B[LORA_MATS]; bf16_t* Bt[LORA_MATS]; int out[LORA_MATS]; int r; };
// batch of rank-r gradient products  G_e(i, j) += scale * sum_m X_e[m, i] U_e[m, j], m < n, i < n_long_e, j < r
constexpr int LORA_OUTER_MAX = 2 * LORA_MATS;
struct LoraOuterArgs {
  const bf16_t* X[LORA_OUTER_MAX]; size_t ldx[LORA_OUTER_MAX];
  const float* U[LORA_OUTER_MAX];            // [n, r]
  float* G[LORA_OUTER_MAX]; size_t g_i[LORA_OUTER_MAX], g_j[LORA_OUTER_MAX];   // element (i, j) at G[i g_i + j g_j]
  int n_long[LORA_OUTER_MAX];
  int count, n, r;
  float scale;
};
// rank-r extension of a projection GEMM (see gemm_mfma.hip)
constexpr int GEMM_EXT_MAX = 12;   // (targets sharing a projection: <= 3) x (adapters on the matrix-core path: <= 4)
struct GemmExt {
  int n, r;
  int col0[GEMM_EXT_MAX], col1[GEMM_EXT_MAX];
  const bf16_t* A2[GEMM_EXT_MAX];
  const bf16_t* W2[GEMM_EXT_MAX];
  size_t ldw2[GEMM_EXT_MAX];
};

// Gated-linear-unit form of the forward GEMM: W = [gate rows ; up rows] ([2F, K]); the kernel multiplies
// both halves for the same F output columns and writes act = silu(gate) * up, plus - for rows
// [save_row0, save_row0 + save_rows) - the gate and up values themselves (the activations graph
// pruning keeps for the finetune rows).
struct GemmGlu {
  int F;                // columns of act = rows of each half of W
  int col0;             // first act column of this launch
  bf16_t* save_gate;    // [save_rows, ld_save] or NULL
  bf16_t* save_up;
  int save_row0, save_rows;
  size_t ld_save;
};


// Records a HIP event before and after the launches it brackets when a timer for `id` runs.
struct KernelTimerScope {
  int id; hipStream_t s; int slot;
  KernelTimerScope(int id, hipStream_t s);
  ~KernelTimerScope();
};

// Event pair for ONE kernel launch of class `id` while its timer runs (false: no timer, or its slots are
// used up).  The launch hands the pair to hipExtLaunchKernelGGL, which stamps the kernel's own start and
// end: no marker packets go on the stream, so the neighbouring kernels are not held apart.
// first_of_call: counts a new launch of the class (a call that issues several kernels passes false for
// the later ones; their durations add to the same launch).
bool kernel_timer_pair(int id, hipEvent_t* start, hipEvent_t* stop, bool first_of_call);

// ---- launchers: no validation, the entry points have done it -------------------------
// C[M,N] = A[M,K] W[N,K]^T (+bias) (+residual);  trans_w: W is [K,N].  Leading dimensions in elements.
// part / part_elems: optional fp32 scratch for split-K partial sums (input-gradient form)
int32_t launch_gemm(const void* A, const void* W, void* C, const void* bias, const void* residual, int M, int N,
                    int K, size_t lda, size_t ldw, size_t ldc, size_t ldr, bool trans_w, int dtype, hipStream_t s,
                    const GemmExt* ext = nullptr, float* part = nullptr, size_t part_elems = 0, int* splits_out = nullptr);
int32_t launch_gemm_generic(const void* A, const void* W, void* C, const void* bias, const void* residual, int M,
                            int N, int K, size_t lda, size_t ldw, size_t ldc, size_t ldr, bool trans_w, int dtype,
                            hipStream_t s);
// How the bf16 MFMA path tiles a product: one or two launches side by side in the output columns, each one tile
// shape (bm x bn), `cols` output columns, K cut over `splits` blocks, a ring of `stages` stages.  part_elems: floats of
// split-K scratch at hand (0 = none).  The gated form is the forward plan over its 2F interleaved columns.
struct GemmLaunchStep { int bm, bn, cols, splits, stages; };
struct GemmLaunchPlan { int n; GemmLaunchStep step[2]; };
GemmLaunchPlan plan_gemm_mfma(int M, int N, int K, bool trans_w, size_t part_elems);
// bf16 MFMA path; returns FLEXCO_EUNSUPPORTED (without launching) for shapes it does not cover
int32_t launch_gemm_mfma(const void* A, const void* W, void* C, const void* bias, const void* residual, int M,
                         int N, int K, size_t lda, size_t ldw, size_t ldc, size_t ldr, bool trans_w,
                         const GemmExt* ext, hipStream_t s, float* part = nullptr, size_t part_elems = 0,
                         int timer_id = -1, int* splits_out = nullptr);
// act[M, F] = silu(A Wg^T + ext) * (A Wu^T + ext), W = [Wg ; Wu]; ext entries address the 2F columns
// [gate | up].  Returns FLEXCO_EUNSUPPORTED (without launching) for shapes it does not cover.
int32_t launch_gemm_glu_mfma(const void* A, const void* W, void* act, int M, int F, int K, size_t lda, size_t ldw,
                             size_t ld_act, const GemmExt* ext, void* save_gate, void* save_up, int save_row0,
                             int save_rows, size_t ld_save, hipStream_t s, int timer_id);
int32_t launch_lora_shrink_mfma(const LoraShrinkArgs& a, int n_mats, hipStream_t s);
int32_t launch_lora_transpose(const LoraTransposeArgs& a, int n_mats, hipStream_t s);
int32_t launch_lora_outer_batch(const LoraOuterArgs& a, hipStream_t s);
int32_t launch_lora_outer_bf16(const void* X, size_t ldx, const float* U, float* G, size_t g_i, size_t g_j, int n,
                               int n_long, int r, float scale, hipStream_t s);

int32_t launch_rmsnorm(const void* x, const void* g, void* h, int T, int H, float eps, int dtype, hipStream_t s,
                       void* save = nullptr, int save_row0 = 0, int save_rows = 0);
// The LoRA backward's rank-r products t_z = dy_z B_z (Sec. 4.1 bypass form) of up to three targets whose dy_z are
// column ranges of ONE row that a row kernel has just produced: that kernel multiplies the row by B_z while it
// holds it (bf16 only, r = 16 or 32), instead of a shrink launch reading the row back.
struct RowLoraT {
  int n;                       // targets (0: nothing to do)
  int col0[3], col1[3];        // target z owns the row's columns [col0, col1)
  const void* B[3];            // B_z [col1 - col0, r], row-major
  float* t[3];                 // [rows, r] fp32, unscaled
  void* ext[3];                // [rows, r] bf16, times scale: operand of the GEMM extension
  int r;
  float scale;
};
inline bool row_lora_ok(int dtype, int r) { return dtype == FLEXCO_BF16 && (r == 16 || r == 32); }
int32_t launch_rmsnorm_bwd(const void* x, const void* g, const void* dh, const void* add, void* dx, int T, int H,
                           float eps, int dtype, hipStream_t s, void* hn = nullptr,
                           const float* dh_part = nullptr, int splits = 1, const RowLoraT* lt = nullptr);
// t = dy B for one target over n rows of width `width` (the same row product as a kernel of its own)
int32_t launch_lora_row_t(const void* dy, size_t lddy, int n, int width, const RowLoraT& lt, hipStream_t s);
int32_t launch_rope_append(const flexco_layer_cfg& c, void* qkv, const int32_t* tok_pos, const int32_t* slot,
                           const flexco_kv_pool& pool, int T, int ft_tok0, int n_ft, int ft_pos0, void* q_cache,
                           hipStream_t s);
int32_t launch_rope_bwd_pack(const flexco_layer_cfg& c, const void* dq, const float* dk_rows, const float* dv_rows,
                             void* dqkv, int win_start, int n, hipStream_t s, const RowLoraT* lt = nullptr);
int32_t launch_swiglu(const void* gu, void* act, int T, int F, int dtype, hipStream_t s);
int32_t launch_swiglu_bwd(const void* gate, const void* up, const void* dact, void* dgu, int n, int F, int dtype,
                          hipStream_t s, void* act = nullptr,
                          const float* dact_part = nullptr, int splits = 1);
int32_t launch_swiglu_remat(const void* gate, const void* up, void* act, int n, int F, int dtype, hipStream_t s);
// (IA)^3 forward scale of up to two column ranges of the listed token rows (see ia3_scale_rows_kernel)
struct Ia3ScaleArgs {
  int n_seg;
  int col0[2], width[2];
  const void* l[2];
  void* save[2];          // unscaled values of the finetune window's rows, or NULL
  size_t ld_save[2];
  int ft_tok0, n_ft, ft_pos0;
};
int32_t launch_ia3_scale_rows(void* buf, size_t ld, const int32_t* tok, int n_tok, const Ia3ScaleArgs& a, int dtype,
                              hipStream_t s);
// dl[c] += sum_r G[r, c] X[r, c];  G[r, c] *= l[c];  part: float [ceil(n / 8)][C] scratch
int32_t launch_ia3_colgrad(void* G, size_t ldg, const void* X, size_t ldx, const void* l, float* part, float* dl, int n,
                           int C, int dtype, hipStream_t s);
struct CopyRowsBatch {
  const char* src[8]; size_t ld_src[8];
  char* dst[8]; size_t ld_dst[8];
  int width16[8];       // row width in 16-byte units
  int count;
};
int32_t launch_copy_rows_batch(const CopyRowsBatch& b, int n_rows, size_t const* width_bytes, hipStream_t s);
int32_t launch_copy_rows(const void* src, size_t ld_src_bytes, void* dst, size_t ld_dst_bytes, int n_rows,
                         size_t width_bytes, hipStream_t s);

int32_t launch_lora_shrink(const void* x, size_t ldx, const void* A, float* u, int n, int in, int r, int dtype,
                           const int32_t* row_idx, hipStream_t s);
int32_t launch_lora_expand(const float* u, const void* B, void* y, size_t ldy, int n, int out, int r, float scale,
                           int dtype, const int32_t* row_idx, hipStream_t s);
int32_t launch_lora_bwd(const void* x, size_t ldx, const void* dy, size_t lddy, const void* A, const void* B,
                        float* dA, float* dB, void* dx, size_t lddx, float* u_ws, float* t_ws, int n, int in,
                        int out, int r, float scale, int dtype, hipStream_t s, bool relu = false);
int32_t launch_relu_mask(float* u, float* t, size_t count, hipStream_t s);

int32_t launch_attention_generic(const flexco_layer_cfg& c, const flexco_maps& m, const void* q, size_t ldq,
                                 const flexco_kv_pool& pool, float* part_ml, float* part_acc, hipStream_t s);
// bf16, head_dim 128, page_size 16, group <= 16; otherwise FLEXCO_EUNSUPPORTED without launching
// The finetune window's rows of the attention output and of the log-sum-exp, written a second time where the
// backward pass keeps them (row i of the window at out2 + i * nq d / lse2 + i * nq); lse2 = NULL: none.
struct AttnKeep {
  void* out2;
  float* lse2;
  int tok0, n;      // the window's token rows [tok0, tok0 + n)
};
int32_t launch_attention_mfma(const flexco_layer_cfg& c, const flexco_maps& m, const void* q, size_t ldq,
                              const flexco_kv_pool& pool, float* part_ml, float* part_acc, void* out, size_t ldo,
                              float* lse, hipStream_t s, const AttnKeep* keep = nullptr, bool skip_chunk = false,
                              bool nothing_to_do = false);
// the chunk items (everything but single decode tokens) of the same work list, four wavefronts per item, K / V staged in LDS
int32_t launch_attention_chunk_mfma(const flexco_layer_cfg& c, const flexco_maps& m, const void* q, size_t ldq,
                                    const flexco_kv_pool& pool, float* part_ml, float* part_acc, void* out, size_t ldo,
                                    float* lse, hipStream_t s, const AttnKeep* keep = nullptr, bool alone = false);
// bf16 window backward on the matrix cores; FLEXCO_EUNSUPPORTED (nothing launched) for other shapes
int32_t launch_attention_bwd_mfma(const flexco_layer_cfg& c, const flexco_kv_pool& pool, const int32_t* seq_pages,
                                  int win_start, int win_len, const void* q, const void* out, const float* lse,
                                  float* delta, const void* dout, void* dq, float* dk_accum, float* dv_accum,
                                  hipStream_t s);
int32_t launch_attention_merge(const flexco_layer_cfg& c, const flexco_maps& m, const float* part_ml,
                               const float* part_acc, void* out, size_t ldo, float* lse, hipStream_t s, bool skip_single_split = false,
                               const AttnKeep* keep = nullptr);
int32_t launch_attention_delta(const flexco_layer_cfg& c, const void* out, const void* dout, float* delta, int n,
                               hipStream_t s);
int32_t launch_attention_bwd_generic(const flexco_layer_cfg& c, const flexco_kv_pool& pool, const int32_t* seq_pages,
                                     int win_start, int win_len, const void* q, const float* lse, const float* delta,
                                     const void* dout, void* dq, float* dk_accum, float* dv_accum, hipStream_t s);

}  // namespace flexco

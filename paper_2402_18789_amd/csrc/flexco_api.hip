// Entry points of the C ABI: validation on the host, workspace carving, and the launch
// sequences of one forward iteration (Sec. 6.2) and one token-window backward step
// (Alg. 2) of a decoder layer.
#include <cmath>
#include <cstring>
#include <vector>

#include "flexco_internal.h"

using namespace flexco;

// ---- per-kernel event timers --------------------------------------------------------------
namespace flexco {
struct KTimer {
  std::vector<hipEvent_t> ev;   // 2 per launch
  int used = 0;
  bool on = false;
};
static KTimer g_timers[FLEXCO_N_KERNEL_IDS];

KernelTimerScope::KernelTimerScope(int id_, hipStream_t s_) : id(id_), s(s_), slot(-1) {
  KTimer& t = g_timers[id];
  if (t.on && 2 * (t.used + 1) <= (int)t.ev.size()) {
    slot = t.used++;
    (void)hipEventRecord(t.ev[2 * slot], s);
  }
}
KernelTimerScope::~KernelTimerScope() {
  if (slot >= 0) (void)hipEventRecord(g_timers[id].ev[2 * slot + 1], s);
}
}  // namespace flexco

extern "C" int32_t flexco_kernel_timer_start(int32_t kernel_id, int32_t max_launches) {
  clear_error();
  FLEXCO_CHECK(kernel_id >= 0 && kernel_id < FLEXCO_N_KERNEL_IDS, FLEXCO_EINVAL, "unknown kernel id %d", kernel_id);
  FLEXCO_CHECK(max_launches > 0 && max_launches <= (1 << 20), FLEXCO_EINVAL, "max_launches out of range");
  KTimer& t = g_timers[kernel_id];
  FLEXCO_CHECK(!t.on, FLEXCO_EINVAL, "timer %d is already running", kernel_id);
  t.ev.resize(2 * (size_t)max_launches);
  for (auto& e : t.ev) {
    hipError_t rc = hipEventCreate(&e);
    if (rc != hipSuccess) return fail(FLEXCO_EHIP, "hipEventCreate: %s", hipGetErrorString(rc));
  }
  t.used = 0;
  t.on = true;
  return FLEXCO_OK;
}

extern "C" int32_t flexco_kernel_timer_stop(int32_t kernel_id, double* total_ms, int64_t* launches) {
  clear_error();
  FLEXCO_CHECK(kernel_id >= 0 && kernel_id < FLEXCO_N_KERNEL_IDS, FLEXCO_EINVAL, "unknown kernel id %d", kernel_id);
  FLEXCO_CHECK(total_ms && launches, FLEXCO_EINVAL, "NULL output");
  KTimer& t = g_timers[kernel_id];
  FLEXCO_CHECK(t.on, FLEXCO_EINVAL, "timer %d is not running", kernel_id);
  double sum = 0.0;
  int32_t rc_out = FLEXCO_OK;
  for (int i = 0; i < t.used; ++i) {
    float ms = 0.f;
    hipError_t rc = hipEventSynchronize(t.ev[2 * i + 1]);
    if (rc == hipSuccess) rc = hipEventElapsedTime(&ms, t.ev[2 * i], t.ev[2 * i + 1]);
    if (rc != hipSuccess) { rc_out = fail(FLEXCO_EHIP, "event timing: %s", hipGetErrorString(rc)); break; }
    sum += ms;
  }
  *total_ms = sum;
  *launches = t.used;
  for (auto& e : t.ev) (void)hipEventDestroy(e);
  t.ev.clear();
  t.used = 0;
  t.on = false;
  return rc_out;
}

// launches bracketed by the event timer of their kernel class (stream variable `s` in scope)
#define EW(expr) do { KernelTimerScope ts_(FLEXCO_K_ELEMWISE, s); FLEXCO_TRY(expr); } while (0)
#define LR(expr) do { KernelTimerScope ts_(FLEXCO_K_LORA, s); FLEXCO_TRY(expr); } while (0)

namespace {

struct Carver {
  char* base;
  size_t off = 0;
  void* take(size_t bytes) {
    void* p = base ? base + off : nullptr;
    off += align_up(bytes, 256);
    return p;
  }
};

struct FwdWs {
  void *h, *qkv, *attn, *x2, *gu, *act;
  float *lse, *u, *part_ml, *part_acc;
  size_t bytes;
};
struct BwdWs {
  void *hn, *act, *dact, *dgu, *dh, *dx2, *dattn, *dq, *dqkv;
  float *delta, *u, *t;
  size_t bytes;
};

int cols_per_tile(const flexco_layer_cfg& c) {
  const int group = c.n_q_heads / c.n_kv_heads;
  return (16 / group > 1 ? 16 / group : 1) * group;
}

FwdWs carve_fwd(const flexco_layer_cfg& c, int T, int n_parts, void* base) {
  const size_t e = esize(c.dtype);
  const size_t qd = (size_t)c.n_q_heads * c.head_dim, qkvd = qd + 2 * (size_t)c.n_kv_heads * c.head_dim;
  Carver cv{(char*)base};
  FwdWs w;
  w.h = cv.take(e * T * c.hidden);
  w.qkv = cv.take(e * T * qkvd);
  w.attn = cv.take(e * T * qd);
  w.x2 = cv.take(e * T * c.hidden);
  w.gu = cv.take(e * T * 2 * c.ffn);
  w.act = cv.take(e * T * c.ffn);
  w.lse = (float*)cv.take(sizeof(float) * T * c.n_q_heads);
  w.u = (float*)cv.take(sizeof(float) * T * (c.lora_rank > 0 ? c.lora_rank : 1));
  const size_t prow = (size_t)n_parts * c.n_kv_heads * cols_per_tile(c);
  w.part_ml = (float*)cv.take(sizeof(float) * prow * 2);
  w.part_acc = (float*)cv.take(sizeof(float) * prow * c.head_dim);
  w.bytes = cv.off;
  return w;
}

BwdWs carve_bwd(const flexco_layer_cfg& c, int n, void* base) {
  const size_t e = esize(c.dtype);
  const size_t qd = (size_t)c.n_q_heads * c.head_dim, qkvd = qd + 2 * (size_t)c.n_kv_heads * c.head_dim;
  Carver cv{(char*)base};
  BwdWs w;
  w.hn = cv.take(e * n * c.hidden);
  w.act = cv.take(e * n * c.ffn);
  w.dact = cv.take(e * n * c.ffn);
  w.dgu = cv.take(e * n * 2 * c.ffn);
  w.dh = cv.take(e * n * c.hidden);
  w.dx2 = cv.take(e * n * c.hidden);
  w.dattn = cv.take(e * n * qd);
  w.dq = cv.take(e * n * qd);
  w.dqkv = cv.take(e * n * qkvd);
  w.delta = (float*)cv.take(sizeof(float) * n * c.n_q_heads);
  const int r = c.lora_rank > 0 ? c.lora_rank : 1;
  w.u = (float*)cv.take(sizeof(float) * n * r);
  w.t = (float*)cv.take(sizeof(float) * n * r);
  w.bytes = cv.off;
  return w;
}

int32_t check_cfg(const flexco_layer_cfg* c) {
  FLEXCO_CHECK(c != nullptr, FLEXCO_EINVAL, "cfg is NULL");
  FLEXCO_CHECK(c->hidden > 0 && c->n_q_heads > 0 && c->n_kv_heads > 0 && c->head_dim > 0 && c->ffn > 0,
               FLEXCO_EINVAL, "cfg has a non-positive dimension");
  FLEXCO_CHECK(c->n_q_heads % c->n_kv_heads == 0, FLEXCO_ESHAPE, "n_kv_heads (%d) must divide n_q_heads (%d)",
               c->n_kv_heads, c->n_q_heads);
  FLEXCO_CHECK(c->head_dim % 2 == 0 && c->head_dim <= 256, FLEXCO_ESHAPE, "head_dim %d must be even and <= 256",
               c->head_dim);
  FLEXCO_CHECK(c->dtype == FLEXCO_F32 || c->dtype == FLEXCO_BF16, FLEXCO_ESHAPE, "unknown dtype %d", c->dtype);
  FLEXCO_CHECK(c->page_size > 0, FLEXCO_EINVAL, "page_size must be positive");
  FLEXCO_CHECK(c->lora_rank >= 0 && c->lora_rank <= 64, FLEXCO_ESHAPE, "lora_rank %d outside [0, 64]", c->lora_rank);
  FLEXCO_CHECK(c->lora_targets >= 0 && c->lora_targets < (1 << FLEXCO_N_TARGETS), FLEXCO_EINVAL,
               "lora_targets 0x%x has unknown bits", c->lora_targets);
  FLEXCO_CHECK(c->lora_targets == 0 || c->lora_rank > 0, FLEXCO_ESHAPE, "lora_targets set but lora_rank is 0");
  // rows must keep 16-byte alignment
  const size_t e = esize(c->dtype);
  FLEXCO_CHECK((c->hidden * e) % 16 == 0 && (c->ffn * e) % 16 == 0 && (c->head_dim * e) % 16 == 0, FLEXCO_ESHAPE,
               "hidden, ffn and head_dim rows must be multiples of 16 bytes");
  FLEXCO_CHECK(std::isfinite(c->rms_eps) && c->rms_eps >= 0.f && c->rope_theta > 0.f, FLEXCO_EINVAL,
               "rms_eps / rope_theta out of range");
  return FLEXCO_OK;
}

int32_t check_weights(const flexco_base_weights* w) {
  FLEXCO_CHECK(w != nullptr, FLEXCO_EINVAL, "weights is NULL");
  FLEXCO_CHECK(w->wqkv && w->wo && w->wgu && w->wd && w->g1 && w->g2, FLEXCO_EINVAL, "a base weight is NULL");
  FLEXCO_CHECK(aligned16(w->wqkv) && aligned16(w->wo) && aligned16(w->wgu) && aligned16(w->wd) && aligned16(w->g1) &&
                   aligned16(w->g2) && aligned16(w->bqkv), FLEXCO_EINVAL, "a base weight is not 16-byte aligned");
  return FLEXCO_OK;
}

int32_t check_lora(const flexco_layer_cfg& c, const flexco_lora* l, bool need_grads) {
  if (c.lora_targets == 0) return FLEXCO_OK;
  FLEXCO_CHECK(l != nullptr, FLEXCO_EINVAL, "cfg names LoRA targets but lora is NULL");
  for (int t = 0; t < FLEXCO_N_TARGETS; ++t) {
    if (!(c.lora_targets >> t & 1)) continue;
    FLEXCO_CHECK(l->A[t] && l->B[t], FLEXCO_EINVAL, "LoRA target %d: A or B is NULL", t);
    FLEXCO_CHECK(aligned16(l->A[t]) && aligned16(l->B[t]), FLEXCO_EINVAL, "LoRA target %d: misaligned", t);
    if (need_grads) FLEXCO_CHECK(l->dA[t] && l->dB[t], FLEXCO_EINVAL, "LoRA target %d: dA or dB is NULL", t);
  }
  return FLEXCO_OK;
}

int32_t check_pool(const flexco_layer_cfg& c, const flexco_kv_pool* p) {
  FLEXCO_CHECK(p != nullptr && p->k_pages && p->v_pages, FLEXCO_EINVAL, "kv pool is NULL");
  FLEXCO_CHECK(aligned16(p->k_pages) && aligned16(p->v_pages), FLEXCO_EINVAL, "kv pool is not 16-byte aligned");
  FLEXCO_CHECK(p->num_pages > 0, FLEXCO_EINVAL, "kv pool has no pages");
  FLEXCO_CHECK(p->page_size == c.page_size, FLEXCO_ESHAPE, "pool page_size %d != cfg page_size %d", p->page_size,
               c.page_size);
  return FLEXCO_OK;
}

int32_t check_maps(const flexco_layer_cfg& c, const flexco_maps* m) {
  FLEXCO_CHECK(m != nullptr, FLEXCO_EINVAL, "maps is NULL");
  FLEXCO_CHECK(m->T > 0 && m->n_req > 0 && m->n_items > 0 && m->n_tiles > 0 && m->n_parts > 0, FLEXCO_EINVAL,
               "maps describe an empty batch");
  FLEXCO_CHECK(m->page_size == c.page_size, FLEXCO_ESHAPE, "maps page_size %d != cfg page_size %d", m->page_size,
               c.page_size);
  const int group = c.n_q_heads / c.n_kv_heads;
  FLEXCO_CHECK(m->tile_tokens == (16 / group > 1 ? 16 / group : 1), FLEXCO_ESHAPE,
               "maps were built for a different n_q_heads / n_kv_heads ratio");
  FLEXCO_CHECK(m->tok_req && m->tok_pos && m->slot && m->block_table && m->tile_req && m->item_tile && m->tok_tile,
               FLEXCO_EINVAL, "maps hold a NULL array");
  return FLEXCO_OK;
}

void target_dims(const flexco_layer_cfg& c, int t, int* in, int* out) {
  const int qd = c.n_q_heads * c.head_dim, kd = c.n_kv_heads * c.head_dim;
  switch (t) {
    case FLEXCO_T_Q: *in = c.hidden; *out = qd; break;
    case FLEXCO_T_K: *in = c.hidden; *out = kd; break;
    case FLEXCO_T_V: *in = c.hidden; *out = kd; break;
    case FLEXCO_T_O: *in = qd; *out = c.hidden; break;
    case FLEXCO_T_GATE: *in = c.hidden; *out = c.ffn; break;
    case FLEXCO_T_UP: *in = c.hidden; *out = c.ffn; break;
    default: *in = c.ffn; *out = c.hidden; break;
  }
}

inline char* boff(void* p, size_t elems, size_t e) { return (char*)p + elems * e; }
inline const char* boff(const void* p, size_t elems, size_t e) { return (const char*)p + elems * e; }

// y[lora rows, col0 : col0 + out] += scale (x[lora rows] A^T) B^T
int32_t lora_apply(const flexco_layer_cfg& c, const flexco_lora* l, int t, const flexco_maps& m, const void* x,
                   size_t ldx, void* y, size_t ldy, size_t col0, float* u, hipStream_t s) {
  if (!(c.lora_targets >> t & 1) || m.n_lora == 0) return FLEXCO_OK;
  int in, out;
  target_dims(c, t, &in, &out);
  FLEXCO_TRY(launch_lora_shrink(x, ldx, l->A[t], u, m.n_lora, in, c.lora_rank, c.dtype, m.lora_tok, s));
  return launch_lora_expand(u, l->B[t], boff(y, col0, esize(c.dtype)), ldy, m.n_lora, out, c.lora_rank,
                            c.lora_scale, c.dtype, m.lora_tok, s);
}

int32_t run_attention(const flexco_layer_cfg& c, const flexco_maps& m, const void* q, size_t ldq,
                      const flexco_kv_pool& pool, void* out, size_t ldo, float* lse, float* part_ml, float* part_acc,
                      hipStream_t s) {
  int32_t rc;
  {
    KernelTimerScope ts(FLEXCO_K_ATTN_FWD, s);
    rc = launch_attention_mfma(c, m, q, ldq, pool, part_ml, part_acc, s);
  }
  if (rc == FLEXCO_EUNSUPPORTED) {
    clear_error();
    KernelTimerScope ts(FLEXCO_K_GENERIC, s);
    rc = launch_attention_generic(c, m, q, ldq, pool, part_ml, part_acc, s);
  }
  if (rc) return rc;
  KernelTimerScope ts(FLEXCO_K_ATTN_MERGE, s);
  return launch_attention_merge(c, m, part_ml, part_acc, out, ldo, lse, s);
}

}  // namespace

namespace flexco {
int32_t launch_gemm(const void* A, const void* W, void* C, const void* bias, const void* residual, int M, int N,
                    int K, size_t lda, size_t ldw, size_t ldc, size_t ldr, bool trans_w, int dtype, hipStream_t s) {
  if (M == 0) return FLEXCO_OK;
  if (dtype == FLEXCO_BF16) {
    int32_t rc;
    {
      KernelTimerScope ts(trans_w ? FLEXCO_K_GEMM_BWD : FLEXCO_K_GEMM_FWD, s);
      rc = launch_gemm_mfma(A, W, C, bias, residual, M, N, K, lda, ldw, ldc, ldr, trans_w, s);
    }
    if (rc != FLEXCO_EUNSUPPORTED) return rc;
    clear_error();
  }
  KernelTimerScope ts(FLEXCO_K_GENERIC, s);
  return launch_gemm_generic(A, W, C, bias, residual, M, N, K, lda, ldw, ldc, ldr, trans_w, dtype, s);
}
}  // namespace flexco

extern "C" int32_t flexco_workspace_bytes(const flexco_layer_cfg* cfg, int32_t T_max, int32_t n_parts_max,
                                          int32_t win_max, int32_t kv_max, size_t* out_bytes) {
  clear_error();
  FLEXCO_TRY(check_cfg(cfg));
  FLEXCO_CHECK(out_bytes != nullptr, FLEXCO_EINVAL, "out_bytes is NULL");
  FLEXCO_CHECK(T_max >= 0 && n_parts_max >= 0 && win_max >= 0 && kv_max >= 0, FLEXCO_EINVAL, "negative size");
  const size_t f = carve_fwd(*cfg, T_max, n_parts_max, nullptr).bytes;
  const size_t b = carve_bwd(*cfg, win_max, nullptr).bytes;
  *out_bytes = f > b ? f : b;
  return FLEXCO_OK;
}

extern "C" int32_t flexco_gemm(const void* A, const void* W, void* C, const void* bias, const void* residual,
                               int32_t M, int32_t N, int32_t K, int32_t trans_w, int32_t dtype, void* stream) {
  clear_error();
  FLEXCO_CHECK(A && W && C, FLEXCO_EINVAL, "A, W or C is NULL");
  FLEXCO_CHECK(M > 0 && N > 0 && K > 0, FLEXCO_EINVAL, "M, N, K must be positive");
  FLEXCO_CHECK(dtype == FLEXCO_F32 || dtype == FLEXCO_BF16, FLEXCO_ESHAPE, "unknown dtype %d", dtype);
  FLEXCO_CHECK(aligned16(A) && aligned16(W) && aligned16(C) && aligned16(bias) && aligned16(residual), FLEXCO_EINVAL,
               "misaligned pointer");
  return launch_gemm(A, W, C, bias, residual, M, N, K, K, trans_w ? N : K, N, N, trans_w != 0, dtype,
                     (hipStream_t)stream);
}

extern "C" int32_t flexco_attention_mixed(const flexco_layer_cfg* cfg, const flexco_maps* maps, const void* q,
                                          const flexco_kv_pool* pool, void* out, float* lse, void* ws,
                                          size_t ws_bytes, void* stream) {
  clear_error();
  FLEXCO_TRY(check_cfg(cfg));
  FLEXCO_TRY(check_maps(*cfg, maps));
  FLEXCO_TRY(check_pool(*cfg, pool));
  FLEXCO_CHECK(q && out && ws, FLEXCO_EINVAL, "q, out or ws is NULL");
  FLEXCO_CHECK(aligned16(q) && aligned16(out) && aligned16(ws) && aligned16(lse), FLEXCO_EINVAL, "misaligned pointer");
  const size_t prow = (size_t)maps->n_parts * cfg->n_kv_heads * cols_per_tile(*cfg);
  const size_t ml_bytes = align_up(sizeof(float) * prow * 2, 256);
  const size_t need = ml_bytes + sizeof(float) * prow * cfg->head_dim;
  FLEXCO_CHECK(need <= ws_bytes, FLEXCO_EWORKSPACE, "attention needs %zu workspace bytes, got %zu", need, ws_bytes);
  const size_t qd = (size_t)cfg->n_q_heads * cfg->head_dim;
  return run_attention(*cfg, *maps, q, qd, *pool, out, qd, lse, (float*)ws, (float*)((char*)ws + ml_bytes),
                       (hipStream_t)stream);
}

extern "C" int32_t flexco_lora_fwd(const void* x, void* y, int32_t T, int32_t in_features, int32_t out_features,
                                   int32_t rank, float scale, int32_t dtype, const void* const* A_list,
                                   const void* const* B_list, int32_t n_adapters, const int32_t* seg_off,
                                   const int32_t* seg_adapter, int32_t n_seg, float* u_ws, void* stream) {
  clear_error();
  FLEXCO_CHECK(x && y && A_list && B_list && seg_off && seg_adapter && u_ws, FLEXCO_EINVAL, "NULL argument");
  FLEXCO_CHECK(T > 0 && in_features > 0 && out_features > 0 && n_seg > 0 && n_adapters > 0, FLEXCO_EINVAL,
               "non-positive size");
  FLEXCO_CHECK(rank > 0 && rank <= 64, FLEXCO_ESHAPE, "rank %d outside [1, 64]", rank);
  FLEXCO_CHECK(dtype == FLEXCO_F32 || dtype == FLEXCO_BF16, FLEXCO_ESHAPE, "unknown dtype %d", dtype);
  FLEXCO_CHECK(aligned16(x) && aligned16(y) && aligned16(u_ws), FLEXCO_EINVAL, "misaligned pointer");
  FLEXCO_CHECK(seg_off[0] == 0 && seg_off[n_seg] == T, FLEXCO_ESHAPE, "segments must cover rows [0, T)");
  for (int s = 0; s < n_seg; ++s) {
    FLEXCO_CHECK(seg_off[s + 1] > seg_off[s], FLEXCO_ESHAPE, "segment %d is empty or descending", s);
    FLEXCO_CHECK(seg_adapter[s] >= -1 && seg_adapter[s] < n_adapters, FLEXCO_EINVAL,
                 "segment %d: adapter %d outside [-1, %d)", s, seg_adapter[s], n_adapters);
    if (seg_adapter[s] >= 0)
      FLEXCO_CHECK(A_list[seg_adapter[s]] && B_list[seg_adapter[s]], FLEXCO_EINVAL, "adapter %d has a NULL matrix",
                   seg_adapter[s]);
  }
  const size_t e = esize(dtype);
  hipStream_t st = (hipStream_t)stream;
  for (int s = 0; s < n_seg; ++s) {
    const int a = seg_adapter[s];
    if (a < 0) continue;
    const int r0 = seg_off[s], n = seg_off[s + 1] - r0;
    FLEXCO_TRY(launch_lora_shrink(boff(x, (size_t)r0 * in_features, e), in_features, A_list[a], u_ws + (size_t)r0 * rank,
                                  n, in_features, rank, dtype, nullptr, st));
    FLEXCO_TRY(launch_lora_expand(u_ws + (size_t)r0 * rank, B_list[a], boff(y, (size_t)r0 * out_features, e),
                                  out_features, n, out_features, rank, scale, dtype, nullptr, st));
  }
  return FLEXCO_OK;
}

extern "C" int32_t flexco_layer_forward(const flexco_layer_cfg* cfg, const flexco_base_weights* w,
                                        const flexco_lora* lora, const flexco_maps* maps, const void* x_in,
                                        void* x_out, const flexco_kv_pool* pool, const flexco_ft_state* ft, void* ws,
                                        size_t ws_bytes, void* stream) {
  clear_error();
  FLEXCO_TRY(check_cfg(cfg));
  FLEXCO_TRY(check_weights(w));
  FLEXCO_TRY(check_maps(*cfg, maps));
  FLEXCO_TRY(check_pool(*cfg, pool));
  const flexco_layer_cfg& c = *cfg;
  const flexco_maps& m = *maps;
  if (m.n_lora > 0) FLEXCO_TRY(check_lora(c, lora, false));
  FLEXCO_CHECK(x_in && x_out && ws, FLEXCO_EINVAL, "x_in, x_out or ws is NULL");
  FLEXCO_CHECK(x_in != x_out, FLEXCO_EINVAL, "x_out may not alias x_in");
  FLEXCO_CHECK(aligned16(x_in) && aligned16(x_out) && aligned16(ws), FLEXCO_EINVAL, "misaligned pointer");
  FLEXCO_CHECK((m.n_ft > 0) == (ft != nullptr), FLEXCO_EINVAL,
               "ft state must be given exactly when the batch has a finetune request (n_ft = %d)", m.n_ft);
  if (ft) {
    FLEXCO_CHECK(ft->q_cache && ft->saved_x && ft->saved_x2 && ft->saved_gate && ft->saved_up && ft->saved_attn &&
                     ft->lse, FLEXCO_EINVAL, "ft state has a NULL buffer");
    FLEXCO_CHECK(m.ft_pos0 + m.n_ft <= ft->seq_len, FLEXCO_ESHAPE,
                 "finetune window [%d, %d) exceeds the state's seq_len %d", m.ft_pos0, m.ft_pos0 + m.n_ft, ft->seq_len);
  }
  FwdWs k = carve_fwd(c, m.T, m.n_parts, ws);
  FLEXCO_CHECK(k.bytes <= ws_bytes, FLEXCO_EWORKSPACE, "forward needs %zu workspace bytes, got %zu", k.bytes, ws_bytes);

  hipStream_t s = (hipStream_t)stream;
  const int T = m.T, H = c.hidden, F = c.ffn, dt = c.dtype;
  const size_t e = esize(dt);
  const size_t qd = (size_t)c.n_q_heads * c.head_dim, kd = (size_t)c.n_kv_heads * c.head_dim, qkvd = qd + 2 * kd;

  // attention side
  EW(launch_rmsnorm(x_in, w->g1, k.h, T, H, c.rms_eps, dt, s));
  FLEXCO_TRY(launch_gemm(k.h, w->wqkv, k.qkv, w->bqkv, nullptr, T, (int)qkvd, H, H, H, qkvd, 0, false, dt, s));
  LR(lora_apply(c, lora, FLEXCO_T_Q, m, k.h, H, k.qkv, qkvd, 0, k.u, s));
  LR(lora_apply(c, lora, FLEXCO_T_K, m, k.h, H, k.qkv, qkvd, qd, k.u, s));
  LR(lora_apply(c, lora, FLEXCO_T_V, m, k.h, H, k.qkv, qkvd, qd + kd, k.u, s));
  EW(launch_rope_append(c, k.qkv, m.tok_pos, m.slot, *pool, T, m.ft_tok0, m.n_ft, m.ft_pos0,
                                ft ? ft->q_cache : nullptr, s));
  FLEXCO_TRY(run_attention(c, m, k.qkv, qkvd, *pool, k.attn, qd, ft ? k.lse : nullptr, k.part_ml, k.part_acc, s));
  FLEXCO_TRY(launch_gemm(k.attn, w->wo, k.x2, nullptr, x_in, T, H, (int)qd, qd, qd, H, H, false, dt, s));
  LR(lora_apply(c, lora, FLEXCO_T_O, m, k.attn, qd, k.x2, H, 0, k.u, s));
  // MLP side
  EW(launch_rmsnorm(k.x2, w->g2, k.h, T, H, c.rms_eps, dt, s));
  FLEXCO_TRY(launch_gemm(k.h, w->wgu, k.gu, nullptr, nullptr, T, 2 * F, H, H, H, 2 * (size_t)F, 0, false, dt, s));
  LR(lora_apply(c, lora, FLEXCO_T_GATE, m, k.h, H, k.gu, 2 * (size_t)F, 0, k.u, s));
  LR(lora_apply(c, lora, FLEXCO_T_UP, m, k.h, H, k.gu, 2 * (size_t)F, F, k.u, s));
  EW(launch_swiglu(k.gu, k.act, T, F, dt, s));
  FLEXCO_TRY(launch_gemm(k.act, w->wd, x_out, nullptr, k.x2, T, H, F, F, F, H, H, false, dt, s));
  LR(lora_apply(c, lora, FLEXCO_T_DOWN, m, k.act, F, x_out, H, 0, k.u, s));
  // keep what graph pruning leaves alive for the finetune rows (Alg. 1), at their positions
  if (ft) {
    const int n = m.n_ft;
    const size_t t0 = m.ft_tok0, p0 = m.ft_pos0;
    EW(launch_copy_rows(boff(x_in, t0 * H, e), H * e, boff(ft->saved_x, p0 * H, e), H * e, n, H * e, s));
    EW(launch_copy_rows(boff(k.x2, t0 * H, e), H * e, boff(ft->saved_x2, p0 * H, e), H * e, n, H * e, s));
    EW(launch_copy_rows(boff(k.gu, t0 * 2 * F, e), 2 * F * e, boff(ft->saved_gate, p0 * F, e), F * e, n, F * e, s));
    EW(launch_copy_rows(boff(k.gu, t0 * 2 * F + F, e), 2 * F * e, boff(ft->saved_up, p0 * F, e), F * e, n, F * e, s));
    EW(launch_copy_rows(boff(k.attn, t0 * qd, e), qd * e, boff(ft->saved_attn, p0 * qd, e), qd * e, n, qd * e, s));
    EW(launch_copy_rows(k.lse + t0 * c.n_q_heads, c.n_q_heads * 4, ft->lse + p0 * c.n_q_heads,
                                c.n_q_heads * 4, n, c.n_q_heads * 4, s));
  }
  return FLEXCO_OK;
}

static int32_t attention_window_bwd_impl(const flexco_layer_cfg& c, const flexco_kv_pool& pool,
                                         const int32_t* seq_pages, int win_start, int win_len, const void* q,
                                         const void* out, const float* lse, const void* dout, void* dq,
                                         float* dk_accum, float* dv_accum, float* delta, hipStream_t s) {
  KernelTimerScope ts(FLEXCO_K_ATTN_BWD, s);
  FLEXCO_TRY(launch_attention_delta(c, out, dout, delta, win_len, s));
  return launch_attention_bwd_generic(c, pool, seq_pages, win_start, win_len, q, lse, delta, dout, dq, dk_accum,
                                      dv_accum, s);
}

extern "C" int32_t flexco_attention_window_bwd(const flexco_layer_cfg* cfg, const flexco_kv_pool* pool,
                                               const int32_t* seq_pages, int32_t n_seq_pages, int32_t win_start,
                                               int32_t win_len, const void* q, const void* out, const float* lse,
                                               const void* dout, void* dq, float* dk_accum, float* dv_accum,
                                               void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  FLEXCO_TRY(check_cfg(cfg));
  FLEXCO_TRY(check_pool(*cfg, pool));
  FLEXCO_CHECK(seq_pages && q && out && lse && dout && dq && dk_accum && dv_accum && ws, FLEXCO_EINVAL, "NULL argument");
  FLEXCO_CHECK(win_start >= 0 && win_len > 0, FLEXCO_EINVAL, "window [%d, +%d) is invalid", win_start, win_len);
  const int l = win_start + win_len;
  FLEXCO_CHECK((l + cfg->page_size - 1) / cfg->page_size <= n_seq_pages, FLEXCO_EPAGE,
               "window end %d exceeds the sequence's %d pages", l, n_seq_pages);
  const size_t need = sizeof(float) * (size_t)win_len * cfg->n_q_heads;
  FLEXCO_CHECK(need <= ws_bytes, FLEXCO_EWORKSPACE, "attention backward needs %zu workspace bytes, got %zu", need,
               ws_bytes);
  return attention_window_bwd_impl(*cfg, *pool, seq_pages, win_start, win_len, q, out, lse, dout, dq, dk_accum,
                                   dv_accum, (float*)ws, (hipStream_t)stream);
}

extern "C" int32_t flexco_lora_bwd(const flexco_layer_cfg* cfg, const flexco_base_weights* w,
                                   const flexco_lora* lora, const flexco_kv_pool* pool, const int32_t* seq_pages,
                                   int32_t n_seq_pages, const flexco_ft_state* ft, int32_t win_start, int32_t win_len,
                                   const void* dY, void* dX, void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  FLEXCO_TRY(check_cfg(cfg));
  FLEXCO_TRY(check_weights(w));
  FLEXCO_TRY(check_pool(*cfg, pool));
  const flexco_layer_cfg& c = *cfg;
  FLEXCO_TRY(check_lora(c, lora, true));
  FLEXCO_CHECK(ft && seq_pages && dY && ws, FLEXCO_EINVAL, "NULL argument");
  FLEXCO_CHECK(ft->q_cache && ft->saved_x && ft->saved_x2 && ft->saved_gate && ft->saved_up && ft->saved_attn &&
                   ft->lse && ft->dk_accum && ft->dv_accum, FLEXCO_EINVAL, "ft state has a NULL buffer");
  FLEXCO_CHECK(win_start >= 0 && win_len > 0, FLEXCO_EINVAL, "window [%d, +%d) is invalid", win_start, win_len);
  const int l = win_start + win_len;
  FLEXCO_CHECK(l <= ft->seq_len, FLEXCO_ESHAPE, "window end %d exceeds seq_len %d", l, ft->seq_len);
  FLEXCO_CHECK((l + c.page_size - 1) / c.page_size <= n_seq_pages, FLEXCO_EPAGE,
               "window end %d exceeds the sequence's %d pages", l, n_seq_pages);
  FLEXCO_CHECK(aligned16(dY) && aligned16(dX) && aligned16(ws), FLEXCO_EINVAL, "misaligned pointer");
  BwdWs k = carve_bwd(c, win_len, ws);
  FLEXCO_CHECK(k.bytes <= ws_bytes, FLEXCO_EWORKSPACE, "backward needs %zu workspace bytes, got %zu", k.bytes, ws_bytes);

  hipStream_t s = (hipStream_t)stream;
  const int n = win_len, H = c.hidden, F = c.ffn, dt = c.dtype, r = c.lora_rank;
  const size_t e = esize(dt), w0 = win_start;
  const size_t qd = (size_t)c.n_q_heads * c.head_dim, kd = (size_t)c.n_kv_heads * c.head_dim, qkvd = qd + 2 * kd;
  auto has = [&](int t) { return (c.lora_targets >> t & 1) != 0; };
  const void* x_w = boff(ft->saved_x, w0 * H, e);
  const void* x2_w = boff(ft->saved_x2, w0 * H, e);
  const void* gate_w = boff(ft->saved_gate, w0 * F, e);
  const void* up_w = boff(ft->saved_up, w0 * F, e);
  const void* attn_w = boff(ft->saved_attn, w0 * qd, e);
  const void* q_w = boff(ft->q_cache, w0 * qd, e);
  const float* lse_w = ft->lse + w0 * c.n_q_heads;

  // ---- MLP side: down projection, SwiGLU, gate/up projections, second norm -------------
  FLEXCO_TRY(launch_gemm(dY, w->wd, k.dact, nullptr, nullptr, n, F, H, H, F, F, 0, true, dt, s));
  if (has(FLEXCO_T_DOWN)) {
    EW(launch_swiglu_remat(gate_w, up_w, k.act, n, F, dt, s));
    LR(launch_lora_bwd(k.act, F, dY, H, lora->A[FLEXCO_T_DOWN], lora->B[FLEXCO_T_DOWN],
                               lora->dA[FLEXCO_T_DOWN], lora->dB[FLEXCO_T_DOWN], k.dact, F, k.u, k.t, n, F, H, r,
                               c.lora_scale, dt, s));
  }
  EW(launch_swiglu_bwd(gate_w, up_w, k.dact, k.dgu, n, F, dt, s));
  FLEXCO_TRY(launch_gemm(k.dgu, w->wgu, k.dh, nullptr, nullptr, n, H, 2 * F, 2 * (size_t)F, H, H, 0, true, dt, s));
  if (has(FLEXCO_T_GATE) || has(FLEXCO_T_UP)) {
    EW(launch_rmsnorm(x2_w, w->g2, k.hn, n, H, c.rms_eps, dt, s));
    for (int t : {FLEXCO_T_GATE, FLEXCO_T_UP}) {
      if (!has(t)) continue;
      const void* dy = boff(k.dgu, t == FLEXCO_T_UP ? F : 0, e);
      LR(launch_lora_bwd(k.hn, H, dy, 2 * (size_t)F, lora->A[t], lora->B[t], lora->dA[t], lora->dB[t], k.dh,
                                 H, k.u, k.t, n, H, F, r, c.lora_scale, dt, s));
    }
  }
  EW(launch_rmsnorm_bwd(x2_w, w->g2, k.dh, dY, k.dx2, n, H, c.rms_eps, dt, s));
  // ---- output projection ------------------------------------------------------------------
  FLEXCO_TRY(launch_gemm(k.dx2, w->wo, k.dattn, nullptr, nullptr, n, (int)qd, H, H, qd, qd, 0, true, dt, s));
  if (has(FLEXCO_T_O))
    LR(launch_lora_bwd(attn_w, qd, k.dx2, H, lora->A[FLEXCO_T_O], lora->B[FLEXCO_T_O], lora->dA[FLEXCO_T_O],
                               lora->dB[FLEXCO_T_O], k.dattn, qd, k.u, k.t, n, (int)qd, H, r, c.lora_scale, dt, s));
  // ---- attention: dQ of the window, dK/dV of every cached row before its end (Sec. 6.1) ---
  FLEXCO_TRY(attention_window_bwd_impl(c, *pool, seq_pages, win_start, win_len, q_w, attn_w, lse_w, k.dattn, k.dq,
                                       ft->dk_accum, ft->dv_accum, k.delta, s));
  // ---- q/k/v side: the window's accumulator rows are complete now (Sec. 7) ---------------
  const bool qkv_lora = has(FLEXCO_T_Q) || has(FLEXCO_T_K) || has(FLEXCO_T_V);
  if (!dX && !qkv_lora) return FLEXCO_OK;
  EW(launch_rope_bwd_pack(c, k.dq, ft->dk_accum + w0 * kd, ft->dv_accum + w0 * kd, k.dqkv, win_start, n, s));
  if (dX)
    FLEXCO_TRY(launch_gemm(k.dqkv, w->wqkv, k.dh, nullptr, nullptr, n, H, (int)qkvd, qkvd, H, H, 0, true, dt, s));
  if (qkv_lora) {
    EW(launch_rmsnorm(x_w, w->g1, k.hn, n, H, c.rms_eps, dt, s));
    const size_t col0[3] = {0, qd, qd + kd};
    for (int t : {FLEXCO_T_Q, FLEXCO_T_K, FLEXCO_T_V}) {
      if (!has(t)) continue;
      int in, out;
      target_dims(c, t, &in, &out);
      LR(launch_lora_bwd(k.hn, H, boff(k.dqkv, col0[t], e), qkvd, lora->A[t], lora->B[t], lora->dA[t],
                                 lora->dB[t], dX ? k.dh : nullptr, H, k.u, k.t, n, H, out, r, c.lora_scale, dt, s));
    }
  }
  if (dX) EW(launch_rmsnorm_bwd(x_w, w->g1, k.dh, k.dx2, dX, n, H, c.rms_eps, dt, s));
  return FLEXCO_OK;
}

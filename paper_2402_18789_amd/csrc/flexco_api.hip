// Entry points of the C ABI: validation on the host, workspace carving, and the launch
// sequences of one forward iteration (Sec. 6.2) and one token-window backward step
// (Alg. 2) of a decoder layer.
#include <cmath>
#include <cstring>
#include <atomic>
#include <mutex>
#include <vector>

#include "flexco_internal.h"

using namespace flexco;

// ---- per-kernel event timers --------------------------------------------------------------
namespace flexco {
struct KTimer {
  std::vector<hipEvent_t> ev;   // 2 per launch
  int used = 0;       // event pairs taken
  int launches = 0;   // timed launches of the class they belong to
  int seen = 0;       // launches of the class since the timer started
  int stride = 1;     // every stride-th launch is timed
  bool take = false;  // the current launch is a timed one
  bool on = false;
  bool begin_launch() {             // a new launch of the class: is it a timed one?
    take = on && (seen++ % stride == 0) && 2 * (used + 1) <= (int)ev.size();
    if (take) ++launches;
    return take;
  }
};
static KTimer g_timers[FLEXCO_N_KERNEL_IDS];
// The timers are process-wide tables.  Launches may come from several host threads (one per stream), so every
// access to a slot's counters goes through this lock; which launch gets which event pair is still decided in
// arrival order, so a measurement is only meaningful when one thread issues the timed class.
static std::mutex g_timer_mutex;

KernelTimerScope::KernelTimerScope(int id_, hipStream_t s_) : id(id_), s(s_), slot(-1) {
  std::lock_guard<std::mutex> lock(g_timer_mutex);
  KTimer& t = g_timers[id];
  if (t.begin_launch()) {
    slot = t.used++;
    (void)hipEventRecord(t.ev[2 * slot], s);
  }
}
bool kernel_timer_pair(int id, hipEvent_t* start, hipEvent_t* stop, bool first_of_call) {
  std::lock_guard<std::mutex> lock(g_timer_mutex);
  KTimer& t = g_timers[id];
  if (first_of_call) (void)t.begin_launch();
  if (!t.on || !t.take || 2 * (t.used + 1) > (int)t.ev.size()) return false;
  const int slot = t.used++;
  *start = t.ev[2 * slot];
  *stop = t.ev[2 * slot + 1];
  return true;
}
KernelTimerScope::~KernelTimerScope() {
  if (slot < 0) return;
  std::lock_guard<std::mutex> lock(g_timer_mutex);
  if (g_timers[id].on && 2 * slot + 1 < (int)g_timers[id].ev.size()) (void)hipEventRecord(g_timers[id].ev[2 * slot + 1], s);
}
}  // namespace flexco

extern "C" int32_t flexco_kernel_timer_start(int32_t kernel_id, int32_t max_launches) {
  clear_error();
  FLEXCO_CHECK(kernel_id >= 0 && kernel_id < FLEXCO_N_KERNEL_IDS, FLEXCO_EINVAL, "unknown kernel id %d", kernel_id);
  FLEXCO_CHECK(max_launches > 0 && max_launches <= (1 << 20), FLEXCO_EINVAL, "max_launches out of range");
  std::lock_guard<std::mutex> lock(g_timer_mutex);
  KTimer& t = g_timers[kernel_id];
  FLEXCO_CHECK(!t.on, FLEXCO_EINVAL, "timer %d is already running", kernel_id);
  t.ev.assign(2 * (size_t)max_launches, nullptr);
  for (size_t i = 0; i < t.ev.size(); ++i) {
    hipError_t rc = hipEventCreate(&t.ev[i]);
    if (rc != hipSuccess) {                       // release what was created before giving up
      for (size_t j = 0; j < i; ++j) (void)hipEventDestroy(t.ev[j]);
      t.ev.clear();
      return fail(FLEXCO_EHIP, "hipEventCreate: %s", hipGetErrorString(rc));
    }
  }
  t.used = 0;
  t.launches = 0;
  t.seen = 0;
  t.take = false;
  t.on = true;
  return FLEXCO_OK;
}

extern "C" int32_t flexco_kernel_timer_sample(int32_t kernel_id, int32_t stride) {
  clear_error();
  FLEXCO_CHECK(kernel_id >= 0 && kernel_id < FLEXCO_N_KERNEL_IDS, FLEXCO_EINVAL, "unknown kernel id %d", kernel_id);
  FLEXCO_CHECK(stride >= 1, FLEXCO_EINVAL, "stride must be at least 1");
  std::lock_guard<std::mutex> lock(g_timer_mutex);
  FLEXCO_CHECK(!g_timers[kernel_id].on, FLEXCO_EINVAL, "timer %d is running", kernel_id);
  g_timers[kernel_id].stride = stride;
  return FLEXCO_OK;
}

extern "C" int32_t flexco_kernel_timer_read(int32_t kernel_id, double* ms_each, int64_t capacity, int64_t* n) {
  clear_error();
  FLEXCO_CHECK(kernel_id >= 0 && kernel_id < FLEXCO_N_KERNEL_IDS, FLEXCO_EINVAL, "unknown kernel id %d", kernel_id);
  FLEXCO_CHECK(ms_each && n && capacity >= 0, FLEXCO_EINVAL, "NULL output or negative capacity");
  std::lock_guard<std::mutex> lock(g_timer_mutex);
  KTimer& t = g_timers[kernel_id];
  FLEXCO_CHECK(t.on, FLEXCO_EINVAL, "timer %d is not running", kernel_id);
  *n = t.used;
  for (int i = 0; i < t.used && i < capacity; ++i) {
    float ms = 0.f;
    hipError_t rc = hipEventSynchronize(t.ev[2 * i + 1]);
    if (rc == hipSuccess) rc = hipEventElapsedTime(&ms, t.ev[2 * i], t.ev[2 * i + 1]);
    if (rc != hipSuccess) return fail(FLEXCO_EHIP, "event timing: %s", hipGetErrorString(rc));
    ms_each[i] = ms;
  }
  return FLEXCO_OK;
}

extern "C" int32_t flexco_kernel_timer_stop(int32_t kernel_id, double* total_ms, int64_t* launches) {
  clear_error();
  FLEXCO_CHECK(kernel_id >= 0 && kernel_id < FLEXCO_N_KERNEL_IDS, FLEXCO_EINVAL, "unknown kernel id %d", kernel_id);
  FLEXCO_CHECK(total_ms && launches, FLEXCO_EINVAL, "NULL output");
  std::lock_guard<std::mutex> lock(g_timer_mutex);
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
  *launches = t.launches;
  for (auto& e : t.ev) (void)hipEventDestroy(e);
  t.ev.clear();
  t.used = 0;
  t.on = false;
  return rc_out;
}

// Which kernel takes the chunk items (prefill chunks, finetune windows) of the attention work list: -1 = by batch
// (the four-wavefront kernel alone when the work list has no single-token item, beside the decode tokens' kernel on a
// side stream when the chunks' products outweigh the decode stream, else the one-launch kernel: a light chunk load
// hides in the stream's waits there), 0 = the one-launch kernel, 1 = the four-wavefront kernel after the decode
// tokens' kernel, 2 = beside it.
static std::atomic<int> g_chunk_path{-1};

// bf16 calls that took a type-generic kernel because the matrix-core kernel of their class does not cover the
// shape (head_dim other than 128, page size other than 16, odd leading dimensions ...), per kernel class
static std::atomic<int64_t> g_bf16_fallbacks[FLEXCO_N_KERNEL_IDS];
static inline void note_fallback(int dtype, int kernel_id) {
  if (dtype == FLEXCO_BF16) g_bf16_fallbacks[kernel_id].fetch_add(1, std::memory_order_relaxed);
}

// Side stream of a device (default priority) and the two events that fork it from and join it to the caller's
// stream, made on first use and kept; the lock is held while a fork / join pair is enqueued, so that two host
// threads do not interleave their records and waits on the shared events.
namespace {
struct SideStream {
  hipStream_t stream = nullptr;
  hipEvent_t fork = nullptr, join = nullptr;
};
std::mutex g_side_mu;
SideStream g_side[64];
int32_t side_stream(SideStream** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= 64) return fail(FLEXCO_EHIP, "side stream: no current device");
  SideStream& ss = g_side[dev];
  if (!ss.stream) {
    if ((e = hipStreamCreateWithFlags(&ss.stream, hipStreamNonBlocking)) != hipSuccess ||
        (e = hipEventCreateWithFlags(&ss.fork, hipEventDisableTiming)) != hipSuccess ||
        (e = hipEventCreateWithFlags(&ss.join, hipEventDisableTiming)) != hipSuccess)
      return fail(FLEXCO_EHIP, "side stream: %s", hipGetErrorString(e));
  }
  *out = &ss;
  return FLEXCO_OK;
}
}  // namespace

extern "C" int32_t flexco_attention_chunk_path(int32_t mode) {
  clear_error();
  FLEXCO_CHECK(mode >= -1 && mode <= 2, FLEXCO_EINVAL, "mode %d: -1 (by batch), 0, 1 or 2", mode);
  g_chunk_path.store(mode);
  return FLEXCO_OK;
}

extern "C" int32_t flexco_bf16_fallbacks(int64_t* counts, int32_t reset) {
  clear_error();
  FLEXCO_CHECK(counts != nullptr, FLEXCO_EINVAL, "counts is NULL");
  for (int i = 0; i < FLEXCO_N_KERNEL_IDS; ++i)
    counts[i] = reset ? g_bf16_fallbacks[i].exchange(0) : g_bf16_fallbacks[i].load();
  return FLEXCO_OK;
}

// launches bracketed by the event timer of their kernel class (stream variable `s` in scope)
#define EW(expr) do { KernelTimerScope ts_(FLEXCO_K_ELEMWISE, s); FLEXCO_TRY(expr); } while (0)
#define LR(expr) do { KernelTimerScope ts_(FLEXCO_K_LORA, s); FLEXCO_TRY(expr); } while (0)

namespace {

constexpr size_t SPLITK_COLS = 32768;   // split-K scratch of the backward GEMMs: rows x this many floats
constexpr int FWD_SPLITK_MAX_T = 256;   // forward batches up to this many tokens get split-K scratch too
constexpr int ROW_T_MAX_ROWS = 512;     // windows up to this many rows take t = dy B inside the row kernels

struct Carver {
  char* base;
  size_t off = 0;
  void* take(size_t bytes) {
    void* p = base ? base + off : nullptr;
    off += align_up(bytes, 256);
    return p;
  }
};

void target_dims(const flexco_layer_cfg& c, int t, int* in, int* out);

// scratch of the bf16 LoRA path for `rows` token rows, one slot per target
constexpr int FUSED_ADAPTERS = 4;   // adapters of one batch the matrix-core LoRA path folds into a projection
constexpr int PART_SLOTS = 4;       // products of one shrink launch that may be cut over several blocks
struct LoraWs {
  bf16_t* ext[LORA_MATS];     // scaled bf16 [rows, r] operands of the GEMM extension (forward: one per adapter)
  float* part;                // partial products of a shrink cut over several blocks
  // backward only
  float* u[LORA_MATS];        // [rows, r]
  float* t[LORA_MATS];        // [rows, r]
  bf16_t* bt[LORA_MATS];      // transposed B_t, [r, out_t]
};

void carve_lora(const flexco_layer_cfg& c, int rows, bool backward, Carver& cv, LoraWs& w) {
  const int r = c.lora_rank > 0 ? c.lora_rank : 1;
  memset(&w, 0, sizeof(w));
  for (int t = 0; t < LORA_MATS; ++t) {
    if (!(c.lora_targets >> t & 1)) continue;
    int in, out;
    target_dims(c, t, &in, &out);
    w.ext[t] = (bf16_t*)cv.take(sizeof(bf16_t) * (size_t)rows * r * (backward ? 1 : FUSED_ADAPTERS));
    if (!w.part) w.part = (float*)cv.take(sizeof(float) * LORA_SHRINK_SPLITS * PART_SLOTS * (size_t)rows * r);
    if (!backward) continue;
    w.u[t] = (float*)cv.take(sizeof(float) * (size_t)rows * r);
    w.t[t] = (float*)cv.take(sizeof(float) * (size_t)rows * r);
    w.bt[t] = (bf16_t*)cv.take(sizeof(bf16_t) * (size_t)out * r);
  }
}

struct FwdWs {
  void *h, *qkv, *attn, *x2, *gu, *act;
  float *lse, *u, *part_ml, *part_acc;
  float* gemm_part;        // split-K partial sums of the forward projections of a small batch (last in the carve)
  size_t gemm_part_elems;
  LoraWs lw;
  size_t bytes, bytes_without_part;
};
struct BwdWs {
  void *hn, *hn2, *act, *dact, *dgu, *dh, *dx2, *dattn, *dq, *dqkv;   // hn = norm1(x), hn2 = norm2(x2)
  float *delta, *u, *t;
  float* gemm_part;        // split-K partial sums of the input-gradient GEMMs
  size_t gemm_part_elems;
  float* colsum_part;      // per-chunk column sums of the (IA)^3 vector gradients: [ceil(n / 8)][max(F, nkv d)]
  LoraWs lw;
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
  carve_lora(c, T, false, cv, w.lw);
  // A batch of few tokens has fewer output tiles than the chip has CUs: its projections cut K across
  // blocks like the backward window's do, and need the partial sums' scratch.
  w.bytes_without_part = cv.off;
  w.gemm_part_elems = (c.dtype == FLEXCO_BF16 && T <= FWD_SPLITK_MAX_T) ? (size_t)T * SPLITK_COLS : 0;
  w.gemm_part = (float*)cv.take(sizeof(float) * w.gemm_part_elems);
  w.bytes = cv.off;
  return w;
}

BwdWs carve_bwd(const flexco_layer_cfg& c, int n, void* base) {
  const size_t e = esize(c.dtype);
  const size_t qd = (size_t)c.n_q_heads * c.head_dim, qkvd = qd + 2 * (size_t)c.n_kv_heads * c.head_dim;
  Carver cv{(char*)base};
  BwdWs w;
  w.hn = cv.take(e * n * c.hidden);
  w.hn2 = cv.take(e * n * c.hidden);
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
  w.gemm_part_elems = c.dtype == FLEXCO_BF16 ? (size_t)n * SPLITK_COLS : 0;
  w.gemm_part = (float*)cv.take(sizeof(float) * w.gemm_part_elems);
  w.colsum_part = (float*)cv.take(sizeof(float) * (size_t)((n + 7) / 8) *
                                  std::max<size_t>(c.ffn, (size_t)c.n_kv_heads * c.head_dim));
  carve_lora(c, n, true, cv, w.lw);
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

int32_t check_ia3(const flexco_layer_cfg& c, const flexco_ia3* a, bool need_grads) {
  FLEXCO_CHECK(a != nullptr, FLEXCO_EINVAL, "ia3 is NULL");
  FLEXCO_CHECK(c.lora_targets == 0, FLEXCO_EUNSUPPORTED, "an (IA)^3 call takes a configuration without LoRA targets");
  FLEXCO_CHECK(a->l_k && a->l_v && a->l_ff, FLEXCO_EINVAL, "an (IA)^3 vector is NULL");
  FLEXCO_CHECK(aligned16(a->l_k) && aligned16(a->l_v) && aligned16(a->l_ff), FLEXCO_EINVAL, "an (IA)^3 vector is misaligned");
  if (need_grads) FLEXCO_CHECK(a->dl_k && a->dl_v && a->dl_ff, FLEXCO_EINVAL, "an (IA)^3 gradient vector is NULL");
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
  FLEXCO_CHECK(m->tok_req && m->tok_pos && m->slot && m->block_table && m->tile_req && m->item_tile && m->tok_tile &&
                   m->tok_lora && m->tok_adapter && m->item_ntiles && m->item_split && m->tile_nsplit && m->tile_part0,
               FLEXCO_EINVAL, "maps hold a NULL array");
  return FLEXCO_OK;
}

// the page ids inside the maps were validated against a pool of m.num_pages pages: a smaller pool would be
// read and written past its end
int32_t check_maps_pool(const flexco_maps& m, const flexco_kv_pool& p) {
  FLEXCO_CHECK(m.num_pages <= p.num_pages, FLEXCO_EPAGE,
               "maps were built for a pool of %d pages, the pool given has %d", m.num_pages, p.num_pages);
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
inline bool has_target(const flexco_layer_cfg& c, int t) { return (c.lora_targets >> t & 1) != 0; }

// unfused fallback: y[rows, col0 : col0 + out] += scale (x[rows] A^T) B^T for the n rows listed in row_idx
int32_t lora_apply(const flexco_layer_cfg& c, const flexco_lora* l, int t, const int32_t* row_idx, int n, const void* x,
                   size_t ldx, void* y, size_t ldy, size_t col0, float* u, hipStream_t s) {
  if (!has_target(c, t) || n == 0) return FLEXCO_OK;
  int in, out;
  target_dims(c, t, &in, &out);
  FLEXCO_TRY(launch_lora_shrink(x, ldx, l->A[t], u, n, in, c.lora_rank, c.dtype, row_idx, s));
  return launch_lora_expand(u, l->B[t], boff(y, col0, esize(c.dtype)), ldy, n, out, c.lora_rank, c.lora_scale, c.dtype,
                            row_idx, s);
}

// the bf16 LoRA path needs whole MFMA k-steps in the rank and in the contracted dimensions
bool lora_mfma_ok(const flexco_layer_cfg& c, int k_dim) {
  return c.dtype == FLEXCO_BF16 && c.lora_rank % 16 == 0 && k_dim % 128 == 0;
}

// saved_u: kept for every LoRA target of the configuration or for none; 16-byte aligned
int32_t check_saved_u(const flexco_layer_cfg& c, const flexco_ft_state* ft) {
  int have = 0, want = 0;
  for (int t = 0; t < FLEXCO_N_TARGETS; ++t) {
    if (!has_target(c, t)) continue;
    ++want;
    if (ft->saved_u[t]) ++have;
    FLEXCO_CHECK(aligned16(ft->saved_u[t]), FLEXCO_EINVAL, "ft state: saved_u[%d] is misaligned", t);
  }
  FLEXCO_CHECK(have == 0 || have == want, FLEXCO_EINVAL, "ft state keeps saved_u for %d of %d LoRA targets", have, want);
  return FLEXCO_OK;
}

// Gated form of the gate/up projection: where the bf16 kernels cover it, the projection writes
// act = silu(gate) * up straight away (`done` is set) and gate / up only for the finetune rows, into the
// sequence's saved buffers; otherwise y receives [gate | up] as usual and the caller runs SwiGLU.
struct GluOut {
  void* act;
  size_t ld_act;
  bool done;
};

int32_t gated_gemm(const flexco_layer_cfg& c, const flexco_maps& m, const void* x, int K, const void* W, int F,
                   const GemmExt* ext, const flexco_ft_state* ft, GluOut& glu, hipStream_t s) {
  if (c.dtype != FLEXCO_BF16) return FLEXCO_EUNSUPPORTED;
  const size_t e = esize(c.dtype);
  const int32_t rc = launch_gemm_glu_mfma(x, W, glu.act, m.T, F, K, K, K, glu.ld_act, ext,
                                          ft ? (void*)boff(ft->saved_gate, (size_t)m.ft_pos0 * F, e) : nullptr,
                                          ft ? (void*)boff(ft->saved_up, (size_t)m.ft_pos0 * F, e) : nullptr, m.ft_tok0,
                                          ft ? m.n_ft : 0, F, s, FLEXCO_K_GEMM_FWD);
  if (rc == FLEXCO_OK) glu.done = true;
  return rc;
}

// The adapters of a forward call: ads[a] serves the requests with adapter id a; with any_id (one
// adapter given) ads[0] serves every request with an id >= 0.
struct Adapters {
  const flexco_lora* ads;
  int n;
  bool any_id;
};

// One projection of the forward pass over all T tokens, with the LoRA bypass of up to three
// targets that share its input (q/k/v, gate/up) folded in:
//   y[:, col0_t : col1_t] = x W^T (+bias) (+res)  +  scale (x A_t^T) B_t^T on adapter rows,
// A_t, B_t those of each row's own adapter.
int32_t forward_projection(const flexco_layer_cfg& c, const Adapters& ad, const flexco_maps& m, const void* x,
                           int K, const void* W, const void* bias, const void* res, size_t ldr, void* y, int N,
                           const int* targets, const int* col0, int n_targets, FwdWs& k,
                           const flexco_ft_state* ft, hipStream_t s, GluOut* glu = nullptr) {
  int act[3], nact = 0;
  for (int i = 0; i < n_targets; ++i)
    if (m.n_lora > 0 && has_target(c, targets[i])) act[nact++] = i;
  // adapters with rows in this batch
  int used[FLEXCO_MAX_ADAPTERS], nused = 0;
  if (ad.any_id) { if (m.n_lora > 0) used[nused++] = 0; }
  else
    for (int a = 0; a < ad.n; ++a)
      if (m.adapter_tok_off[a + 1] > m.adapter_tok_off[a]) used[nused++] = a;
  const int T = m.T, dt = c.dtype, r = c.lora_rank;
  if (nact > 0 && nused > 0 && nused <= FUSED_ADAPTERS && lora_mfma_ok(c, K)) {
    LoraShrinkArgs sa;
    GemmExt ext;
    memset(&sa, 0, sizeof(sa)); memset(&ext, 0, sizeof(ext));
    // u_{t,a} = scale x A_{t,a}^T for every token row (zero rows where the token is not served by adapter a)
    sa.row_adapter = m.tok_adapter; sa.rows = T; sa.r = r; sa.scale = c.lora_scale;
    sa.part = k.lw.part; sa.part_slots = PART_SLOTS;
    // the finetune window's rows of the unscaled product are kept for the backward pass (dB_t)
    const int ft_ad = ad.any_id ? 0 : m.ft_adapter;
    const bool keep_u = ft && m.n_ft > 0 && ft->saved_u[targets[act[0]]] != nullptr;
    sa.f32_lo = m.ft_tok0; sa.f32_hi = keep_u ? m.ft_tok0 + m.n_ft : m.ft_tok0;
    ext.r = r;
    int z = 0;
    for (int ia = 0; ia < nact; ++ia)
      for (int iu = 0; iu < nused; ++iu, ++z) {
        const int t = targets[act[ia]], a = used[iu];
        const flexco_lora& l = ad.ads[a];
        int in, out;
        target_dims(c, t, &in, &out);
        bf16_t* ext_ta = k.lw.ext[t] + (size_t)iu * T * r;
        sa.X[z] = (const bf16_t*)x; sa.ldx[z] = K; sa.S[z] = (const bf16_t*)l.A[t]; sa.lds[z] = K; sa.K[z] = K;
        sa.want[z] = ad.any_id ? -1 : a;
        sa.out_f32[z] = (keep_u && a == ft_ad) ? ft->saved_u[t] + (size_t)m.ft_pos0 * r : nullptr;
        sa.out_ext[z] = ext_ta;
        ext.col0[z] = col0[act[ia]]; ext.col1[z] = col0[act[ia]] + out;
        ext.A2[z] = ext_ta; ext.W2[z] = (const bf16_t*)l.B[t]; ext.ldw2[z] = r;
      }
    ext.n = z;
    LR(launch_lora_shrink_mfma(sa, z, s));
    if (glu) {
      const int32_t rc = gated_gemm(c, m, x, K, W, N / 2, &ext, ft, *glu, s);
      if (rc != FLEXCO_EUNSUPPORTED) return rc;
      clear_error();
    }
    int32_t rc = launch_gemm(x, W, y, bias, res, T, N, K, K, K, N, ldr, false, dt, s, &ext, k.gemm_part, k.gemm_part_elems);
    if (rc != FLEXCO_EUNSUPPORTED) return rc;
    clear_error();   // e.g. a target boundary inside a 32-column fragment: run the bypass as separate kernels
  }
  if (glu && nact == 0) {
    const int32_t rc = gated_gemm(c, m, x, K, W, N / 2, nullptr, ft, *glu, s);
    if (rc != FLEXCO_EUNSUPPORTED) return rc;
    clear_error();
  }
  FLEXCO_TRY(launch_gemm(x, W, y, bias, res, T, N, K, K, K, N, ldr, false, dt, s, nullptr, k.gemm_part, k.gemm_part_elems));
  // more adapters than the folded path takes: the backward pass (which folds whenever it can) still
  // expects the finetune rows' rank-r products where the state keeps them
  if (nact > 0 && nused > FUSED_ADAPTERS && lora_mfma_ok(c, K) && ft && m.n_ft > 0 && ft->saved_u[targets[act[0]]]) {
    LoraShrinkArgs sa;
    memset(&sa, 0, sizeof(sa));
    const int a = ad.any_id ? 0 : m.ft_adapter;
    sa.row_adapter = m.tok_adapter; sa.rows = T; sa.r = r; sa.scale = 1.f;
    sa.f32_lo = m.ft_tok0; sa.f32_hi = m.ft_tok0 + m.n_ft;
    for (int z = 0; z < nact; ++z) {
      const int t = targets[act[z]];
      sa.X[z] = (const bf16_t*)x; sa.ldx[z] = K; sa.S[z] = (const bf16_t*)ad.ads[a].A[t]; sa.lds[z] = K; sa.K[z] = K;
      sa.want[z] = ad.any_id ? -1 : a;
      sa.out_f32[z] = ft->saved_u[t] + (size_t)m.ft_pos0 * r;
    }
    LR(launch_lora_shrink_mfma(sa, nact, s));
  }
  for (int ia = 0; ia < nact; ++ia)
    for (int iu = 0; iu < nused; ++iu) {
      const int a = used[iu];
      const int32_t* rows = ad.any_id ? m.lora_tok : m.lora_tok + m.adapter_tok_off[a];
      const int n = ad.any_id ? m.n_lora : m.adapter_tok_off[a + 1] - m.adapter_tok_off[a];
      LR(lora_apply(c, &ad.ads[a], targets[act[ia]], rows, n, x, K, y, N, col0[act[ia]], k.u, s));
    }
  return FLEXCO_OK;
}

// A group = the targets that feed one input-gradient projection (down | gate, up | o | q, k, v).
struct BwdGroup {
  int n_targets;
  int targets[3], col0[3];
  const void* xs[3];     // the targets' input rows
  int N_dx;              // width of the projection's input = in_t of every target
  bool fused;            // bf16 matrix-core path: LoRA folded into the GEMM, gradients batched
  int act[3], nact;      // active targets (indices into targets[])
  bool t_ready;          // fused only: a row kernel writes t_t = dy_t B_t (fp32 and the scaled bf16 copy) before the projection
};

void plan_group(const flexco_layer_cfg& c, BwdGroup& g) {
  g.nact = 0;
  for (int i = 0; i < g.n_targets; ++i)
    if (has_target(c, g.targets[i])) g.act[g.nact++] = i;
  g.fused = g.nact > 0 && lora_mfma_ok(c, g.N_dx);
  for (int z = 0; z < g.nact && g.fused; ++z) {
    int in, out;
    target_dims(c, g.targets[g.act[z]], &in, &out);
    if (out % 128 != 0 || in != g.N_dx) g.fused = false;
  }
}

// Start of a backward window, fused groups only: u_t = x_t A_t^T of every target in one launch,
// and the transposed B_t the t_t = dy_t B_t products contract against.
// Where the forward pass kept u_t (ft->saved_u), its window rows are used as they are.
int32_t lora_bwd_prepare(const flexco_layer_cfg& c, const flexco_lora* lora, int n, const BwdGroup* groups,
                         int n_groups, BwdWs& k, const flexco_ft_state* ft, int win_start, hipStream_t s) {
  LoraShrinkArgs su;
  LoraTransposeArgs ta;
  memset(&su, 0, sizeof(su)); memset(&ta, 0, sizeof(ta));
  const int r = c.lora_rank;
  su.rows = n; su.r = r; su.scale = 1.f; su.f32_lo = 0; su.f32_hi = n;   // (up to 7 matrices: no split scratch)
  ta.r = r;
  int nz = 0, nu = 0;
  for (int gi = 0; gi < n_groups; ++gi) {
    const BwdGroup& g = groups[gi];
    if (!g.fused) continue;
    for (int a = 0; a < g.nact; ++a, ++nz) {
      const int t = g.targets[g.act[a]];
      int in, out;
      target_dims(c, t, &in, &out);
      if (g.t_ready) { ta.B[nz] = nullptr; ta.Bt[nz] = nullptr; ta.out[nz] = 0; }   // (no transposed B needed)
      else { ta.B[nz] = (const bf16_t*)lora->B[t]; ta.Bt[nz] = k.lw.bt[t]; ta.out[nz] = out; }
      if (ft->saved_u[t]) {
        k.lw.u[t] = ft->saved_u[t] + (size_t)win_start * r;
        continue;
      }
      su.X[nu] = (const bf16_t*)g.xs[g.act[a]]; su.ldx[nu] = in; su.S[nu] = (const bf16_t*)lora->A[t]; su.lds[nu] = in;
      su.K[nu] = in; su.out_f32[nu] = k.lw.u[t]; su.out_ext[nu] = nullptr;
      ++nu;
    }
  }
  if (nu > 0) LR(launch_lora_shrink_mfma(su, nu, s));
  if (nz > 0) LR(launch_lora_transpose(ta, nz, s));
  return FLEXCO_OK;
}

// One input-gradient projection of the backward window with the LoRA gradients of the targets
// that feed it:   dx = dy W (+ sum_t scale (dy_t B_t) A_t);
//   dB_t += scale dy_t^T (x_t A_t^T);   dA_t += scale (dy_t B_t)^T x_t.
// dy_t = columns [col0_t, col0_t + out_t) of dy; x_t: the target's input rows (in_t wide).
// dx may be NULL (only the LoRA gradients are wanted).  On the fused path the dA / dB products are
// only queued in `outer` (one launch for the whole window at its end): dy, x_t and the u_t, t_t
// buffers stay untouched until then.
int32_t backward_projection(const flexco_layer_cfg& c, const flexco_lora* lora, int n, const void* dy, int K_dy,
                            const void* W, void* dx, const BwdGroup& g, BwdWs& k, LoraOuterArgs& outer,
                            hipStream_t s, int* splits_out = nullptr) {
  // splits_out: the caller's next kernel reads dx; where the product was cut over K, the partial sums stay in
  // k.gemm_part ([split][n][N_dx], *splits_out > 1) for that kernel to add, and dx is not written
  if (splits_out) *splits_out = 1;
  const int dt = c.dtype, r = c.lora_rank, N_dx = g.N_dx;
  const size_t e = esize(dt);
  if (g.fused) {
    // t_t = dy_t B_t of the group's targets in one launch (fp32, and the scaled bf16 copy the GEMM
    // extension reads)
    LoraShrinkArgs st;
    GemmExt ext;
    memset(&st, 0, sizeof(st)); memset(&ext, 0, sizeof(ext));
    st.rows = n; st.r = r; st.scale = c.lora_scale; st.f32_lo = 0; st.f32_hi = n; st.part = k.lw.part; st.part_slots = PART_SLOTS;
    ext.n = g.nact; ext.r = r;
    for (int z = 0; z < g.nact; ++z) {
      const int t = g.targets[g.act[z]];
      int in, out;
      target_dims(c, t, &in, &out);
      st.X[z] = (const bf16_t*)boff(dy, g.col0[g.act[z]], e); st.ldx[z] = K_dy; st.S[z] = k.lw.bt[t]; st.lds[z] = out;
      st.K[z] = out; st.out_f32[z] = k.lw.t[t]; st.out_ext[z] = k.lw.ext[t];
      ext.A2[z] = k.lw.ext[t]; ext.W2[z] = (const bf16_t*)lora->A[t]; ext.ldw2[z] = in;
      // dB_t[o, j] += scale sum_m dy_t[m, o] u_t[m, j];   dA_t[j, i] += scale sum_m x_t[m, i] t_t[m, j]
      int q = outer.count;
      outer.X[q] = (const bf16_t*)boff(dy, g.col0[g.act[z]], e); outer.ldx[q] = K_dy; outer.U[q] = k.lw.u[t];
      outer.G[q] = lora->dB[t]; outer.g_i[q] = r; outer.g_j[q] = 1; outer.n_long[q] = out;
      ++q;
      outer.X[q] = (const bf16_t*)g.xs[g.act[z]]; outer.ldx[q] = in; outer.U[q] = k.lw.t[t];
      outer.G[q] = lora->dA[t]; outer.g_i[q] = 1; outer.g_j[q] = in; outer.n_long[q] = in;
      outer.count = q + 1;
    }
    if (!g.t_ready) LR(launch_lora_shrink_mfma(st, g.nact, s));
    if (dx)
      return launch_gemm(dy, W, dx, nullptr, nullptr, n, N_dx, K_dy, K_dy, N_dx, N_dx, 0, true, dt, s, &ext,
                         k.gemm_part, k.gemm_part_elems, splits_out);
    return FLEXCO_OK;
  }
  // (the unfused LoRA kernels below add into dx: they need it complete)
  if (dx) FLEXCO_TRY(launch_gemm(dy, W, dx, nullptr, nullptr, n, N_dx, K_dy, K_dy, N_dx, N_dx, 0, true, dt, s, nullptr,
                                 k.gemm_part, k.gemm_part_elems, g.nact == 0 ? splits_out : nullptr));
  for (int z = 0; z < g.nact; ++z) {
    const int t = g.targets[g.act[z]];
    int in, out;
    target_dims(c, t, &in, &out);
    LR(launch_lora_bwd(g.xs[g.act[z]], in, boff(dy, g.col0[g.act[z]], e), K_dy, lora->A[t], lora->B[t], lora->dA[t],
                       lora->dB[t], dx, N_dx, k.u, k.t, n, in, out, r, c.lora_scale, dt, s));
  }
  return FLEXCO_OK;
}

int32_t run_attention(const flexco_layer_cfg& c, const flexco_maps& m, const void* q, size_t ldq,
                      const flexco_kv_pool& pool, void* out, size_t ldo, float* lse, float* part_ml, float* part_acc,
                      hipStream_t s, const AttnKeep* keep = nullptr) {
  int32_t rc;
  bool direct = true;    // the matrix-core kernel writes the rows of single-split tiles itself
  {
    KernelTimerScope ts(FLEXCO_K_ATTN_FWD, s);
    const int mode = g_chunk_path.load();
    const bool mixed = m.n_single > 0 && m.n_single < m.n_items;
    const bool beside = mixed && (mode == 2 || (mode < 0 && m.chunk_tile_pages >= m.stream_pages));
    const bool chunk = mode > 0 || (mode < 0 && m.n_single == 0) || beside;
    if (!beside) {
      // (with no single-token item the one-launch kernel has nothing left to do; its support test still decides)
      rc = launch_attention_mfma(c, m, q, ldq, pool, part_ml, part_acc, out, ldo, lse, s, keep, chunk, chunk && m.n_single == 0);
      if (rc == FLEXCO_OK && chunk)
        rc = launch_attention_chunk_mfma(c, m, q, ldq, pool, part_ml, part_acc, out, ldo, lse, s, keep, m.n_single == 0);
    } else {
      // the decode tokens' kernel on the caller's stream and the chunk items' kernel on the side stream, which
      // leaves the caller's stream before the first and rejoins it after the second: the two run beside each other
      // (one lives on HBM, the other on the matrix cores and the vector ALU) and write different rows
      std::lock_guard<std::mutex> lock(g_side_mu);
      SideStream* ss = nullptr;
      FLEXCO_TRY(side_stream(&ss));
      hipError_t e;
      if ((e = hipEventRecord(ss->fork, s)) != hipSuccess || (e = hipStreamWaitEvent(ss->stream, ss->fork, 0)) != hipSuccess)
        return fail(FLEXCO_EHIP, "attention: fork of the side stream failed: %s", hipGetErrorString(e));
      rc = launch_attention_mfma(c, m, q, ldq, pool, part_ml, part_acc, out, ldo, lse, s, keep, true, false);
      // (after the fork the side stream must rejoin whatever happens, a stream capture would not end otherwise)
      const int32_t rc2 = rc == FLEXCO_OK
                              ? launch_attention_chunk_mfma(c, m, q, ldq, pool, part_ml, part_acc, out, ldo, lse, ss->stream, keep)
                              : FLEXCO_OK;
      if ((e = hipEventRecord(ss->join, ss->stream)) != hipSuccess || (e = hipStreamWaitEvent(s, ss->join, 0)) != hipSuccess)
        return fail(FLEXCO_EHIP, "attention: join of the side stream failed: %s", hipGetErrorString(e));
      if (rc == FLEXCO_OK) rc = rc2;
    }
  }
  if (rc == FLEXCO_EUNSUPPORTED) {
    clear_error();
    direct = false;
    note_fallback(c.dtype, FLEXCO_K_ATTN_FWD);
    KernelTimerScope ts(FLEXCO_K_GENERIC, s);
    rc = launch_attention_generic(c, m, q, ldq, pool, part_ml, part_acc, s);
  }
  if (rc) return rc;
  if (direct && m.n_parts == m.n_tiles) return FLEXCO_OK;   // every tile had a single key split: nothing left to merge
  KernelTimerScope ts(FLEXCO_K_ATTN_MERGE, s);
  return launch_attention_merge(c, m, part_ml, part_acc, out, ldo, lse, s, direct, keep);
}

}  // namespace

namespace flexco {
int32_t launch_gemm(const void* A, const void* W, void* C, const void* bias, const void* residual, int M, int N,
                    int K, size_t lda, size_t ldw, size_t ldc, size_t ldr, bool trans_w, int dtype, hipStream_t s,
                    const GemmExt* ext, float* part, size_t part_elems, int* splits_out) {
  if (splits_out) *splits_out = 1;
  if (M == 0) return FLEXCO_OK;
  if (dtype == FLEXCO_BF16) {
    const int32_t rc = launch_gemm_mfma(A, W, C, bias, residual, M, N, K, lda, ldw, ldc, ldr, trans_w, ext, s, part,
                                        part_elems, trans_w ? FLEXCO_K_GEMM_BWD : FLEXCO_K_GEMM_FWD, splits_out);
    if (rc != FLEXCO_EUNSUPPORTED) return rc;
    clear_error();
  }
  if (ext && ext->n > 0) return FLEXCO_EUNSUPPORTED;   // the generic kernel has no rank-r extension
  note_fallback(dtype, trans_w ? FLEXCO_K_GEMM_BWD : FLEXCO_K_GEMM_FWD);
  if (splits_out) *splits_out = 1;
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
  // (a batch of at most FWD_SPLITK_MAX_T tokens also asks for split-K scratch: cover the largest such batch)
  const size_t f = std::max(carve_fwd(*cfg, T_max, n_parts_max, nullptr).bytes,
                            carve_fwd(*cfg, std::min(T_max, FWD_SPLITK_MAX_T), n_parts_max, nullptr).bytes);
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

extern "C" int32_t flexco_gemm_plan(int32_t M, int32_t N, int32_t K, int32_t trans_w, int64_t part_elems, int32_t* out) {
  clear_error();
  FLEXCO_CHECK(out != nullptr, FLEXCO_EINVAL, "out is NULL");
  FLEXCO_CHECK(M > 0 && N > 0 && K > 0 && part_elems >= 0, FLEXCO_EINVAL, "M, N, K must be positive, part_elems not negative");
  FLEXCO_CHECK(K % 64 == 0 && N % 8 == 0, FLEXCO_ESHAPE, "the matrix-core path takes K in multiples of 64 and N in multiples of 8");
  const GemmLaunchPlan pl = plan_gemm_mfma(M, N, K, trans_w != 0, (size_t)part_elems);
  for (int i = 0; i < 11; ++i) out[i] = 0;
  out[0] = pl.n;
  for (int i = 0; i < pl.n; ++i) {
    int32_t* o = out + 1 + 5 * i;
    o[0] = pl.step[i].bm; o[1] = pl.step[i].bn; o[2] = pl.step[i].cols; o[3] = pl.step[i].splits; o[4] = pl.step[i].stages;
  }
  return FLEXCO_OK;
}

extern "C" int32_t flexco_attention_mixed(const flexco_layer_cfg* cfg, const flexco_maps* maps, const void* q,
                                          const flexco_kv_pool* pool, void* out, float* lse, void* ws,
                                          size_t ws_bytes, void* stream) {
  clear_error();
  FLEXCO_TRY(check_cfg(cfg));
  FLEXCO_TRY(check_maps(*cfg, maps));
  FLEXCO_TRY(check_pool(*cfg, pool));
  FLEXCO_TRY(check_maps_pool(*maps, *pool));
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

static int32_t lora_fwd_impl(const void* x, void* y, int32_t T, int32_t in_features, int32_t out_features,
                             int32_t rank, float scale, int32_t dtype, const void* const* A_list,
                             const void* const* B_list, int32_t n_adapters, const int32_t* seg_off,
                             const int32_t* seg_adapter, int32_t n_seg, float* u_ws, void* stream) {
  FLEXCO_CHECK(x && y && A_list && B_list && seg_off && seg_adapter && u_ws, FLEXCO_EINVAL, "NULL argument");
  FLEXCO_CHECK(T > 0 && in_features > 0 && out_features > 0 && n_seg > 0 && n_adapters > 0, FLEXCO_EINVAL,
               "non-positive size");
  FLEXCO_CHECK(rank > 0 && rank <= 64, FLEXCO_ESHAPE, "rank %d outside [1, 64]", rank);
  FLEXCO_CHECK(dtype == FLEXCO_F32 || dtype == FLEXCO_BF16, FLEXCO_ESHAPE, "unknown dtype %d", dtype);
  FLEXCO_CHECK(aligned16(x) && aligned16(y) && aligned16(u_ws), FLEXCO_EINVAL, "misaligned pointer");
  FLEXCO_CHECK(seg_off[0] == 0 && seg_off[n_seg] == T, FLEXCO_ESHAPE, "segments must cover rows [0, T)");
  for (int sg = 0; sg < n_seg; ++sg) {
    FLEXCO_CHECK(seg_off[sg + 1] > seg_off[sg], FLEXCO_ESHAPE, "segment %d is empty or descending", sg);
    FLEXCO_CHECK(seg_adapter[sg] >= -1 && seg_adapter[sg] < n_adapters, FLEXCO_EINVAL,
                 "segment %d: adapter %d outside [-1, %d)", sg, seg_adapter[sg], n_adapters);
    if (seg_adapter[sg] >= 0)
      FLEXCO_CHECK(A_list[seg_adapter[sg]] && B_list[seg_adapter[sg]], FLEXCO_EINVAL, "adapter %d has a NULL matrix",
                   seg_adapter[sg]);
  }
  const size_t e = esize(dtype);
  hipStream_t s = (hipStream_t)stream;
  for (int sg = 0; sg < n_seg; ++sg) {
    const int a = seg_adapter[sg];
    if (a < 0) continue;
    const int r0 = seg_off[sg], n = seg_off[sg + 1] - r0;
    LR(launch_lora_shrink(boff(x, (size_t)r0 * in_features, e), in_features, A_list[a], u_ws + (size_t)r0 * rank, n,
                          in_features, rank, dtype, nullptr, s));
    LR(launch_lora_expand(u_ws + (size_t)r0 * rank, B_list[a], boff(y, (size_t)r0 * out_features, e), out_features,
                          n, out_features, rank, scale, dtype, nullptr, s));
  }
  return FLEXCO_OK;
}

extern "C" int32_t flexco_lora_fwd(const void* x, void* y, int32_t T, int32_t in_features, int32_t out_features,
                                   int32_t rank, float scale, int32_t dtype, const void* const* A_list,
                                   const void* const* B_list, int32_t n_adapters, const int32_t* seg_off,
                                   const int32_t* seg_adapter, int32_t n_seg, float* u_ws, void* stream) {
  clear_error();
  return lora_fwd_impl(x, y, T, in_features, out_features, rank, scale, dtype, A_list, B_list, n_adapters, seg_off,
                       seg_adapter, n_seg, u_ws, stream);
}

// ---- flexco_lora_fwd_static: the same call with the rank-r scratch in the library's own image ----
// For callers that cannot allocate device memory.  `scratch` is the device array; on the host its name is
// only a handle for hipGetSymbolAddress, never an address: the per-device address is looked up once per
// device and everything below uses that pointer.
static __device__ __align__(256) float scratch[FLEXCO_STATIC_SCRATCH_FLOATS];

namespace {
constexpr int STATIC_MAX_DEVICES = 64;
float* g_scratch_ptr[STATIC_MAX_DEVICES];   // address of `scratch` on each device, filled on first use
std::mutex g_scratch_mutex;

int32_t static_scratch(float** out) {
  int dev = -1;
  hipError_t rc = hipGetDevice(&dev);
  if (rc != hipSuccess) return fail(FLEXCO_EHIP, "hipGetDevice: %s", hipGetErrorString(rc));
  FLEXCO_CHECK(dev >= 0 && dev < STATIC_MAX_DEVICES, FLEXCO_EUNSUPPORTED, "device %d beyond the %d devices supported",
               dev, STATIC_MAX_DEVICES);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    float* p = nullptr;
    rc = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
    if (rc != hipSuccess || !p)
      return fail(FLEXCO_EHIP, "hipGetSymbolAddress(scratch) on device %d: %s", dev, hipGetErrorString(rc));
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return FLEXCO_OK;
}
}  // namespace

extern "C" int32_t flexco_lora_fwd_static(const void* x, void* y, int32_t T, int32_t in_features,
                                          int32_t out_features, int32_t rank, float scale, int32_t dtype,
                                          const void* const* A_list, const void* const* B_list, int32_t n_adapters,
                                          const int32_t* seg_off, const int32_t* seg_adapter, int32_t n_seg,
                                          void* stream) {
  clear_error();
  FLEXCO_CHECK(T > 0 && rank > 0, FLEXCO_EINVAL, "non-positive size");
  FLEXCO_CHECK((size_t)T * (size_t)rank <= (size_t)FLEXCO_STATIC_SCRATCH_FLOATS, FLEXCO_EWORKSPACE,
               "T * rank = %zu exceeds the built-in scratch of %zu floats; use flexco_lora_fwd with a buffer of the caller's",
               (size_t)T * (size_t)rank, (size_t)FLEXCO_STATIC_SCRATCH_FLOATS);
  float* u = nullptr;
  FLEXCO_TRY(static_scratch(&u));
  // every row of u that the expansion reads is written by the shrink launched just before it: nothing of the
  // previous call's contents is read, so nothing has to be cleared
  return lora_fwd_impl(x, y, T, in_features, out_features, rank, scale, dtype, A_list, B_list, n_adapters, seg_off,
                       seg_adapter, n_seg, u, stream);
}

static int32_t layer_forward_impl(const flexco_layer_cfg* cfg, const flexco_base_weights* w, const Adapters& ad,
                                  const flexco_maps* maps, const void* x_in, void* x_out, const flexco_kv_pool* pool,
                                  const flexco_ft_state* ft, void* ws, size_t ws_bytes, void* stream,
                                  const flexco_ia3* ia3 = nullptr) {
  FLEXCO_TRY(check_cfg(cfg));
  FLEXCO_TRY(check_weights(w));
  FLEXCO_TRY(check_maps(*cfg, maps));
  FLEXCO_TRY(check_pool(*cfg, pool));
  FLEXCO_TRY(check_maps_pool(*maps, *pool));
  const flexco_layer_cfg& c = *cfg;
  const flexco_maps& m = *maps;
  if (ia3) {
    FLEXCO_TRY(check_ia3(c, ia3, false));
    FLEXCO_CHECK(!ft || (ft->saved_k0 && ft->saved_v0 && aligned16(ft->saved_k0) && aligned16(ft->saved_v0)),
                 FLEXCO_EINVAL, "ft state: saved_k0 / saved_v0 are required with (IA)^3");
  }
  if (m.n_lora > 0 && c.lora_targets != 0) {
    FLEXCO_CHECK(ad.ads != nullptr && ad.n >= 1, FLEXCO_EINVAL, "the batch has adapter tokens but no adapter is given");
    FLEXCO_CHECK(ad.any_id || m.n_adapters <= ad.n, FLEXCO_EINVAL, "the batch uses adapter id %d, %d adapters are given",
                 m.n_adapters - 1, ad.n);
    for (int a = 0; a < ad.n; ++a)
      if (ad.any_id || m.adapter_tok_off[a + 1] > m.adapter_tok_off[a]) FLEXCO_TRY(check_lora(c, &ad.ads[a], false));
  }
  FLEXCO_CHECK(x_in && x_out && ws, FLEXCO_EINVAL, "x_in, x_out or ws is NULL");
  FLEXCO_CHECK(x_in != x_out, FLEXCO_EINVAL, "x_out may not alias x_in");
  FLEXCO_CHECK(aligned16(x_in) && aligned16(x_out) && aligned16(ws), FLEXCO_EINVAL, "misaligned pointer");
  FLEXCO_CHECK((m.n_ft > 0) == (ft != nullptr), FLEXCO_EINVAL,
               "ft state must be given exactly when the batch has a finetune request (n_ft = %d)", m.n_ft);
  if (ft) {
    FLEXCO_CHECK(ft->q_cache && ft->saved_x && ft->saved_x2 && ft->saved_gate && ft->saved_up && ft->saved_attn &&
                     ft->lse, FLEXCO_EINVAL, "ft state has a NULL buffer");
    FLEXCO_TRY(check_saved_u(c, ft));
    FLEXCO_CHECK(c.lora_targets == 0 || m.ft_adapter >= 0, FLEXCO_EINVAL,
                 "the finetune request carries no adapter id (its window trains one)");
    FLEXCO_CHECK(m.ft_pos0 + m.n_ft <= ft->seq_len, FLEXCO_ESHAPE,
                 "finetune window [%d, %d) exceeds the state's seq_len %d", m.ft_pos0, m.ft_pos0 + m.n_ft, ft->seq_len);
  }
  FwdWs k = carve_fwd(c, m.T, m.n_parts, ws);
  if (k.bytes > ws_bytes && k.bytes_without_part <= ws_bytes) {   // no room for the split-K scratch: run unsplit
    k.gemm_part = nullptr;
    k.gemm_part_elems = 0;
    k.bytes = k.bytes_without_part;
  }
  FLEXCO_CHECK(k.bytes <= ws_bytes, FLEXCO_EWORKSPACE, "forward needs %zu workspace bytes, got %zu", k.bytes, ws_bytes);

  hipStream_t s = (hipStream_t)stream;
  const int T = m.T, H = c.hidden, F = c.ffn, dt = c.dtype;
  const size_t e = esize(dt);
  const int qd = c.n_q_heads * c.head_dim, kd = c.n_kv_heads * c.head_dim, qkvd = qd + 2 * kd;

  // attention side
  // (the finetune window's rows of x, x2, the attention output and its log-sum-exp - what graph pruning keeps,
  // Alg. 1 - are written to the sequence's state by the kernels that read or produce them anyway)
  const size_t p0 = m.ft_pos0;
  EW(launch_rmsnorm(x_in, w->g1, k.h, T, H, c.rms_eps, dt, s, ft ? (void*)boff(ft->saved_x, p0 * H, e) : nullptr, m.ft_tok0,
                    m.n_ft));
  {
    const int tg[3] = {FLEXCO_T_Q, FLEXCO_T_K, FLEXCO_T_V}, c0[3] = {0, qd, qd + kd};
    FLEXCO_TRY(forward_projection(c, ad, m, k.h, H, w->wqkv, w->bqkv, nullptr, 0, k.qkv, qkvd, tg, c0, 3, k, ft, s));
  }
  if (ia3 && m.n_lora > 0) {   // keys and values of the adapter's rows, scaled before the rotation and the append
    Ia3ScaleArgs sa;
    memset(&sa, 0, sizeof(sa));
    sa.n_seg = 2;
    sa.col0[0] = qd; sa.width[0] = kd; sa.l[0] = ia3->l_k; sa.save[0] = ft ? ft->saved_k0 : nullptr; sa.ld_save[0] = kd;
    sa.col0[1] = qd + kd; sa.width[1] = kd; sa.l[1] = ia3->l_v; sa.save[1] = ft ? ft->saved_v0 : nullptr; sa.ld_save[1] = kd;
    sa.ft_tok0 = m.ft_tok0; sa.n_ft = ft ? m.n_ft : 0; sa.ft_pos0 = m.ft_pos0;
    EW(launch_ia3_scale_rows(k.qkv, qkvd, m.lora_tok, m.n_lora, sa, dt, s));
  }
  EW(launch_rope_append(c, k.qkv, m.tok_pos, m.slot, *pool, T, m.ft_tok0, m.n_ft, m.ft_pos0,
                        ft ? ft->q_cache : nullptr, s));
  const AttnKeep keep{ft ? (void*)boff(ft->saved_attn, p0 * qd, e) : nullptr, ft ? ft->lse + p0 * c.n_q_heads : nullptr,
                      m.ft_tok0, ft ? m.n_ft : 0};
  FLEXCO_TRY(run_attention(c, m, k.qkv, qkvd, *pool, k.attn, qd, nullptr, k.part_ml, k.part_acc, s, &keep));
  {
    const int tg[1] = {FLEXCO_T_O}, c0[1] = {0};
    FLEXCO_TRY(forward_projection(c, ad, m, k.attn, qd, w->wo, nullptr, x_in, H, k.x2, H, tg, c0, 1, k, ft, s));
  }
  // MLP side
  EW(launch_rmsnorm(k.x2, w->g2, k.h, T, H, c.rms_eps, dt, s, ft ? (void*)boff(ft->saved_x2, p0 * H, e) : nullptr, m.ft_tok0,
                    m.n_ft));
  GluOut glu{k.act, (size_t)F, false};
  {
    const int tg[2] = {FLEXCO_T_GATE, FLEXCO_T_UP}, c0[2] = {0, F};
    FLEXCO_TRY(forward_projection(c, ad, m, k.h, H, w->wgu, nullptr, nullptr, 0, k.gu, 2 * F, tg, c0, 2, k, ft, s, &glu));
  }
  if (!glu.done) EW(launch_swiglu(k.gu, k.act, T, F, dt, s));
  if (ia3 && m.n_lora > 0) {   // the SwiGLU product of the adapter's rows
    Ia3ScaleArgs sa;
    memset(&sa, 0, sizeof(sa));
    sa.n_seg = 1; sa.col0[0] = 0; sa.width[0] = F; sa.l[0] = ia3->l_ff;
    EW(launch_ia3_scale_rows(k.act, F, m.lora_tok, m.n_lora, sa, dt, s));
  }
  {
    const int tg[1] = {FLEXCO_T_DOWN}, c0[1] = {0};
    FLEXCO_TRY(forward_projection(c, ad, m, k.act, F, w->wd, nullptr, k.x2, H, x_out, H, tg, c0, 1, k, ft, s));
  }
  // where the gated projection did not run (fp32), gate and up are still in the workspace: copy the window's rows
  if (ft && !glu.done) {
    const int n = m.n_ft;
    const size_t t0 = m.ft_tok0;
    CopyRowsBatch cb;
    size_t wb[8];
    memset(&cb, 0, sizeof(cb));
    auto add = [&](const void* src, size_t ld_src, void* dst, size_t ld_dst, size_t width) {
      const int q = cb.count++;
      cb.src[q] = (const char*)src; cb.ld_src[q] = ld_src; cb.dst[q] = (char*)dst; cb.ld_dst[q] = ld_dst;
      cb.width16[q] = (int)(width / 16); wb[q] = width;
    };
    add(boff(k.gu, t0 * 2 * F, e), 2 * F * e, boff(ft->saved_gate, p0 * F, e), F * e, F * e);
    add(boff(k.gu, t0 * 2 * F + F, e), 2 * F * e, boff(ft->saved_up, p0 * F, e), F * e, F * e);
    EW(launch_copy_rows_batch(cb, n, wb, s));
  }
  return FLEXCO_OK;
}

extern "C" int32_t flexco_layer_forward(const flexco_layer_cfg* cfg, const flexco_base_weights* w,
                                        const flexco_lora* lora, const flexco_maps* maps, const void* x_in,
                                        void* x_out, const flexco_kv_pool* pool, const flexco_ft_state* ft, void* ws,
                                        size_t ws_bytes, void* stream) {
  clear_error();
  const Adapters ad{lora, lora ? 1 : 0, true};
  return layer_forward_impl(cfg, w, ad, maps, x_in, x_out, pool, ft, ws, ws_bytes, stream);
}

extern "C" int32_t flexco_layer_forward_ia3(const flexco_layer_cfg* cfg, const flexco_base_weights* w,
                                            const flexco_ia3* ia3, const flexco_maps* maps, const void* x_in,
                                            void* x_out, const flexco_kv_pool* pool, const flexco_ft_state* ft,
                                            void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  FLEXCO_CHECK(ia3 != nullptr, FLEXCO_EINVAL, "ia3 is NULL");
  const Adapters ad{nullptr, 0, true};
  return layer_forward_impl(cfg, w, ad, maps, x_in, x_out, pool, ft, ws, ws_bytes, stream, ia3);
}

extern "C" int32_t flexco_layer_forward_multi(const flexco_layer_cfg* cfg, const flexco_base_weights* w,
                                              const flexco_lora* adapters, int32_t n_adapters,
                                              const flexco_maps* maps, const void* x_in, void* x_out,
                                              const flexco_kv_pool* pool, const flexco_ft_state* ft, void* ws,
                                              size_t ws_bytes, void* stream) {
  clear_error();
  FLEXCO_CHECK(n_adapters >= 0 && n_adapters <= FLEXCO_MAX_ADAPTERS, FLEXCO_EINVAL, "n_adapters %d outside [0, %d]",
               n_adapters, FLEXCO_MAX_ADAPTERS);
  FLEXCO_CHECK(n_adapters == 0 || adapters != nullptr, FLEXCO_EINVAL, "adapters is NULL");
  const Adapters ad{adapters, n_adapters, false};
  return layer_forward_impl(cfg, w, ad, maps, x_in, x_out, pool, ft, ws, ws_bytes, stream);
}

static int32_t attention_window_bwd_impl(const flexco_layer_cfg& c, const flexco_kv_pool& pool,
                                         const int32_t* seq_pages, int win_start, int win_len, const void* q,
                                         const void* out, const float* lse, const void* dout, void* dq,
                                         float* dk_accum, float* dv_accum, float* delta, hipStream_t s) {
  KernelTimerScope ts(FLEXCO_K_ATTN_BWD, s);
  // (the matrix-core dQ kernel computes delta = rowsum(dO (.) O) of its rows itself and leaves it for the dK/dV kernel)
  int32_t rc = launch_attention_bwd_mfma(c, pool, seq_pages, win_start, win_len, q, out, lse, delta, dout, dq, dk_accum,
                                         dv_accum, s);
  if (rc != FLEXCO_EUNSUPPORTED) return rc;
  clear_error();
  note_fallback(c.dtype, FLEXCO_K_ATTN_BWD);
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

// One token window backward through the layer; the bypass network is LoRA (`lora`, per cfg.lora_targets) or
// (IA)^3 (`ia3`, cfg without LoRA targets) or none.
static int32_t layer_backward_impl(const flexco_layer_cfg* cfg, const flexco_base_weights* w,
                                   const flexco_lora* lora, const flexco_ia3* ia3, const flexco_kv_pool* pool,
                                   const int32_t* seq_pages, int32_t n_seq_pages, const flexco_ft_state* ft,
                                   int32_t win_start, int32_t win_len, const void* dY, void* dX, void* ws,
                                   size_t ws_bytes, void* stream) {
  FLEXCO_TRY(check_cfg(cfg));
  FLEXCO_TRY(check_weights(w));
  FLEXCO_TRY(check_pool(*cfg, pool));
  const flexco_layer_cfg& c = *cfg;
  FLEXCO_TRY(check_lora(c, lora, true));
  if (ia3) FLEXCO_TRY(check_ia3(c, ia3, true));
  FLEXCO_CHECK(ft && seq_pages && dY && ws, FLEXCO_EINVAL, "NULL argument");
  FLEXCO_CHECK(!ia3 || (ft->saved_k0 && ft->saved_v0 && aligned16(ft->saved_k0) && aligned16(ft->saved_v0)),
               FLEXCO_EINVAL, "ft state: saved_k0 / saved_v0 are required with (IA)^3");
  FLEXCO_CHECK(ft->q_cache && ft->saved_x && ft->saved_x2 && ft->saved_gate && ft->saved_up && ft->saved_attn &&
                   ft->lse && ft->dk_accum && ft->dv_accum, FLEXCO_EINVAL, "ft state has a NULL buffer");
  FLEXCO_TRY(check_saved_u(c, ft));
  FLEXCO_CHECK(win_start >= 0 && win_len > 0, FLEXCO_EINVAL, "window [%d, +%d) is invalid", win_start, win_len);
  const int l = win_start + win_len;
  FLEXCO_CHECK(l <= ft->seq_len, FLEXCO_ESHAPE, "window end %d exceeds seq_len %d", l, ft->seq_len);
  FLEXCO_CHECK((l + c.page_size - 1) / c.page_size <= n_seq_pages, FLEXCO_EPAGE,
               "window end %d exceeds the sequence's %d pages", l, n_seq_pages);
  FLEXCO_CHECK(aligned16(dY) && aligned16(dX) && aligned16(ws), FLEXCO_EINVAL, "misaligned pointer");
  BwdWs k = carve_bwd(c, win_len, ws);
  FLEXCO_CHECK(k.bytes <= ws_bytes, FLEXCO_EWORKSPACE, "backward needs %zu workspace bytes, got %zu", k.bytes, ws_bytes);

  hipStream_t s = (hipStream_t)stream;
  const int n = win_len, H = c.hidden, F = c.ffn, dt = c.dtype;
  const size_t e = esize(dt), w0 = win_start;
  const int qd = c.n_q_heads * c.head_dim, kd = c.n_kv_heads * c.head_dim, qkvd = qd + 2 * kd;
  const void* x_w = boff(ft->saved_x, w0 * H, e);
  const void* x2_w = boff(ft->saved_x2, w0 * H, e);
  const void* gate_w = boff(ft->saved_gate, w0 * F, e);
  const void* up_w = boff(ft->saved_up, w0 * F, e);
  const void* attn_w = boff(ft->saved_attn, w0 * qd, e);
  const void* q_w = boff(ft->q_cache, w0 * qd, e);
  const float* lse_w = ft->lse + w0 * c.n_q_heads;

  // ---- the four projection groups and what their LoRA gradients need ----------------------
  const bool qkv_lora = has_target(c, FLEXCO_T_Q) || has_target(c, FLEXCO_T_K) || has_target(c, FLEXCO_T_V);
  const bool gu_lora = has_target(c, FLEXCO_T_GATE) || has_target(c, FLEXCO_T_UP);
  BwdGroup grp[4];
  memset(grp, 0, sizeof(grp));
  grp[0].n_targets = 1; grp[0].targets[0] = FLEXCO_T_DOWN; grp[0].xs[0] = k.act; grp[0].N_dx = F;
  grp[1].n_targets = 2; grp[1].targets[0] = FLEXCO_T_GATE; grp[1].targets[1] = FLEXCO_T_UP; grp[1].col0[1] = F;
  grp[1].xs[0] = grp[1].xs[1] = k.hn2; grp[1].N_dx = H;
  grp[2].n_targets = 1; grp[2].targets[0] = FLEXCO_T_O; grp[2].xs[0] = attn_w; grp[2].N_dx = qd;
  grp[3].n_targets = 3; grp[3].targets[0] = FLEXCO_T_Q; grp[3].targets[1] = FLEXCO_T_K; grp[3].targets[2] = FLEXCO_T_V;
  grp[3].col0[1] = qd; grp[3].col0[2] = qd + kd; grp[3].xs[0] = grp[3].xs[1] = grp[3].xs[2] = k.hn; grp[3].N_dx = H;
  for (int gi = 0; gi < 4; ++gi) plan_group(c, grp[gi]);
  // t_t = dy_t B_t of the down, o and q/k/v targets: by the row kernels that hold the rows of dy_t anyway (dY has a
  // kernel of its own), where rank and type allow; gate / up keep the shrink launch (their dy comes out of a
  // kernel that does not own whole rows)
  // (windows of up to ROW_T_MAX_ROWS rows: a row kernel's product costs its row a fixed few microseconds, a shrink
  // launch costs about 12 us whatever the window; measured per layer at the 14B shape's 1024-row window: 287 us of
  // small backward kernels with the row products, 238 with three shrink launches; even at 512 rows)
  const bool row_t = row_lora_ok(dt, c.lora_rank) && n <= ROW_T_MAX_ROWS;
  grp[0].t_ready = grp[0].fused && row_t;
  grp[2].t_ready = grp[2].fused && row_t;
  grp[3].t_ready = grp[3].fused && row_t;
  auto row_lora = [&](const BwdGroup& g) {
    RowLoraT lt = {};
    if (!g.t_ready) return lt;
    lt.r = c.lora_rank; lt.scale = c.lora_scale;
    for (int i = 0; i < g.n_targets; ++i) {
      const int t = g.targets[i];
      if (!has_target(c, t)) continue;
      // one target: entry 0; the q/k/v group: entry = role (0 q, 1 k, 2 v)
      const int z = g.n_targets == 1 ? 0 : i;
      int in, out;
      target_dims(c, t, &in, &out);
      lt.col0[z] = g.col0[i]; lt.col1[z] = g.col0[i] + out; lt.B[z] = lora->B[t]; lt.t[z] = k.lw.t[t]; lt.ext[z] = k.lw.ext[t];
      ++lt.n;
    }
    return lt;
  };
  LoraOuterArgs outer;
  memset(&outer, 0, sizeof(outer));
  outer.n = n; outer.r = c.lora_rank; outer.scale = c.lora_scale;

  // inputs of the adapted projections: rematerialised SwiGLU output (Alg. 1), the two norms
  // Where the state keeps the rank-r products of the forward pass, these inputs are only read by the
  // dA products at the window's end, and the kernels that walk the same rows anyway (SwiGLU backward,
  // the two norm backwards) write them as a by-product; otherwise they are needed up front.
  bool late_inputs = true;
  for (int t = 0; t < FLEXCO_N_TARGETS; ++t)
    if (has_target(c, t) && !ft->saved_u[t]) late_inputs = false;
  for (int gi = 0; gi < 4; ++gi)
    if (grp[gi].nact > 0 && !grp[gi].fused) late_inputs = false;   // the unfused path multiplies by A up front
  const bool act_late = late_inputs && has_target(c, FLEXCO_T_DOWN);
  const bool hn2_late = late_inputs && gu_lora;
  const bool hn_late = late_inputs && qkv_lora && dX != nullptr;
  if (has_target(c, FLEXCO_T_DOWN) && !act_late) EW(launch_swiglu_remat(gate_w, up_w, k.act, n, F, dt, s));
  if (gu_lora && !hn2_late) EW(launch_rmsnorm(x2_w, w->g2, k.hn2, n, H, c.rms_eps, dt, s));
  if (qkv_lora && !hn_late) EW(launch_rmsnorm(x_w, w->g1, k.hn, n, H, c.rms_eps, dt, s));
  FLEXCO_TRY(lora_bwd_prepare(c, lora, n, grp, 4, k, ft, win_start, s));
  if (grp[0].t_ready) LR(launch_lora_row_t(dY, H, n, H, row_lora(grp[0]), s));

  // ---- MLP side: down projection, SwiGLU, gate/up projections, second norm -------------
  // (where an input-gradient product was cut over K, the kernel that reads it next adds the partial sums itself)
  int sp_dact = 1, sp_dh2 = 1, sp_dh1 = 1;
  FLEXCO_TRY(backward_projection(c, lora, n, dY, H, w->wd, k.dact, grp[0], k, outer, s, ia3 ? nullptr : &sp_dact));
  if (ia3) {   // dl_ff += colsum(dact (.) act0) with the rematerialised SwiGLU product; dact <- dact (.) l_ff
    EW(launch_swiglu_remat(gate_w, up_w, k.act, n, F, dt, s));
    EW(launch_ia3_colgrad(k.dact, F, k.act, F, ia3->l_ff, k.colsum_part, ia3->dl_ff, n, F, dt, s));
  }
  EW(launch_swiglu_bwd(gate_w, up_w, k.dact, k.dgu, n, F, dt, s, act_late ? k.act : nullptr,
                       sp_dact > 1 ? k.gemm_part : nullptr, sp_dact));
  FLEXCO_TRY(backward_projection(c, lora, n, k.dgu, 2 * F, w->wgu, k.dh, grp[1], k, outer, s, &sp_dh2));
  {
    const RowLoraT lt = row_lora(grp[2]);   // dx2 is the output projection's dy
    EW(launch_rmsnorm_bwd(x2_w, w->g2, k.dh, dY, k.dx2, n, H, c.rms_eps, dt, s, hn2_late ? k.hn2 : nullptr,
                          sp_dh2 > 1 ? k.gemm_part : nullptr, sp_dh2, &lt));
  }
  // ---- output projection ------------------------------------------------------------------
  FLEXCO_TRY(backward_projection(c, lora, n, k.dx2, H, w->wo, k.dattn, grp[2], k, outer, s));
  // ---- attention: dQ of the window, dK/dV of every cached row before its end (Sec. 6.1) ---
  FLEXCO_TRY(attention_window_bwd_impl(c, *pool, seq_pages, win_start, win_len, q_w, attn_w, lse_w, k.dattn, k.dq,
                                       ft->dk_accum, ft->dv_accum, k.delta, s));
  // ---- q/k/v side: the window's accumulator rows are complete now (Sec. 7) ---------------
  if (dX || qkv_lora || ia3) {
    const RowLoraT lt_qkv = ia3 ? RowLoraT{} : row_lora(grp[3]);
    EW(launch_rope_bwd_pack(c, k.dq, ft->dk_accum + w0 * kd, ft->dv_accum + w0 * kd, k.dqkv, win_start, n, s, &lt_qkv));
    if (ia3) {   // the k and v column ranges of the packed rows: dl += colsum(d (.) unscaled rows), d <- d (.) l
      EW(launch_ia3_colgrad(boff(k.dqkv, qd, e), qkvd, boff(ft->saved_k0, w0 * kd, e), kd, ia3->l_k, k.colsum_part,
                            ia3->dl_k, n, kd, dt, s));
      EW(launch_ia3_colgrad(boff(k.dqkv, qd + kd, e), qkvd, boff(ft->saved_v0, w0 * kd, e), kd, ia3->l_v, k.colsum_part,
                            ia3->dl_v, n, kd, dt, s));
    }
    if (dX || qkv_lora)
      FLEXCO_TRY(backward_projection(c, lora, n, k.dqkv, qkvd, w->wqkv, dX ? k.dh : nullptr, grp[3], k, outer, s,
                                     dX ? &sp_dh1 : nullptr));
  }
  // ---- every queued dA / dB product of the window in one launch ----------------------------
  if (dX) EW(launch_rmsnorm_bwd(x_w, w->g1, k.dh, k.dx2, dX, n, H, c.rms_eps, dt, s, hn_late ? k.hn : nullptr,
                                sp_dh1 > 1 ? k.gemm_part : nullptr, sp_dh1));
  LR(launch_lora_outer_batch(outer, s));
  return FLEXCO_OK;
}

extern "C" int32_t flexco_lora_bwd(const flexco_layer_cfg* cfg, const flexco_base_weights* w,
                                   const flexco_lora* lora, const flexco_kv_pool* pool, const int32_t* seq_pages,
                                   int32_t n_seq_pages, const flexco_ft_state* ft, int32_t win_start, int32_t win_len,
                                   const void* dY, void* dX, void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  return layer_backward_impl(cfg, w, lora, nullptr, pool, seq_pages, n_seq_pages, ft, win_start, win_len, dY, dX, ws,
                             ws_bytes, stream);
}

extern "C" int32_t flexco_ia3_bwd(const flexco_layer_cfg* cfg, const flexco_base_weights* w, const flexco_ia3* ia3,
                                  const flexco_kv_pool* pool, const int32_t* seq_pages, int32_t n_seq_pages,
                                  const flexco_ft_state* ft, int32_t win_start, int32_t win_len, const void* dY,
                                  void* dX, void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  FLEXCO_CHECK(ia3 != nullptr, FLEXCO_EINVAL, "ia3 is NULL");
  return layer_backward_impl(cfg, w, nullptr, ia3, pool, seq_pages, n_seq_pages, ft, win_start, win_len, dY, dX, ws,
                             ws_bytes, stream);
}

namespace {
int32_t check_adapter(int32_t dtype, int32_t hidden, const flexco_adapter* ad, bool need_grads) {
  FLEXCO_CHECK(dtype == FLEXCO_F32 || dtype == FLEXCO_BF16, FLEXCO_ESHAPE, "unknown dtype %d", dtype);
  FLEXCO_CHECK(hidden > 0 && (hidden * esize(dtype)) % 16 == 0, FLEXCO_ESHAPE, "hidden rows must be multiples of 16 bytes");
  FLEXCO_CHECK(ad != nullptr, FLEXCO_EINVAL, "adapter is NULL");
  FLEXCO_CHECK(ad->bottleneck >= 1 && ad->bottleneck <= 64, FLEXCO_ESHAPE, "bottleneck %d outside [1, 64]", ad->bottleneck);
  FLEXCO_CHECK(ad->w_down && ad->w_up, FLEXCO_EINVAL, "an adapter weight is NULL");
  if (need_grads) FLEXCO_CHECK(ad->dw_down && ad->dw_up, FLEXCO_EINVAL, "an adapter gradient buffer is NULL");
  return FLEXCO_OK;
}
}  // namespace

// The adapter's scratch.  Matrix-core path (bf16, b = 64, hidden a multiple of 128): forward = the bf16 ReLU output
// of every token row; backward = u, t (fp32), t in bf16 and the transposed up-projection.  Otherwise the
// rank-r fallback kernels: one / two fp32 [rows, b] arrays.
namespace {
bool adapter_mfma_ok(int32_t dtype, int32_t hidden, int b) { return dtype == FLEXCO_BF16 && b == 64 && hidden % 128 == 0; }
size_t adapter_fwd_bytes(int32_t dtype, int32_t hidden, int b, size_t T, size_t n_rows) {
  return adapter_mfma_ok(dtype, hidden, b) ? align_up(sizeof(bf16_t) * T * b, 256) : sizeof(float) * n_rows * b;
}
size_t adapter_bwd_bytes(int32_t dtype, int32_t hidden, int b, size_t n) {
  size_t need = 2 * align_up(sizeof(float) * n * b, 256);
  if (adapter_mfma_ok(dtype, hidden, b)) need += align_up(sizeof(bf16_t) * n * b, 256) + align_up(sizeof(bf16_t) * (size_t)b * hidden, 256);
  return need;
}
}  // namespace

extern "C" int32_t flexco_adapter_workspace_bytes(int32_t dtype, int32_t hidden, int32_t bottleneck, int32_t T_max,
                                                  int32_t win_max, size_t* out_bytes) {
  clear_error();
  FLEXCO_CHECK(out_bytes != nullptr, FLEXCO_EINVAL, "out_bytes is NULL");
  FLEXCO_CHECK(hidden > 0 && bottleneck >= 1 && bottleneck <= 64 && T_max >= 0 && win_max >= 0, FLEXCO_EINVAL,
               "size out of range");
  *out_bytes = std::max(adapter_fwd_bytes(dtype, hidden, bottleneck, T_max, T_max),
                        adapter_bwd_bytes(dtype, hidden, bottleneck, win_max));
  return FLEXCO_OK;
}

extern "C" int32_t flexco_adapter_fwd(int32_t dtype, int32_t hidden, const flexco_adapter* ad, const flexco_maps* maps,
                                      void* y, void* saved_in, int32_t seq_len, void* ws, size_t ws_bytes,
                                      void* stream) {
  clear_error();
  FLEXCO_TRY(check_adapter(dtype, hidden, ad, false));
  FLEXCO_CHECK(maps != nullptr && y != nullptr, FLEXCO_EINVAL, "maps or y is NULL");
  const flexco_maps& m = *maps;
  FLEXCO_CHECK(m.T > 0 && m.n_lora >= 0 && m.n_lora <= m.T && (m.n_lora == 0 || (m.lora_tok && m.tok_adapter)),
               FLEXCO_EINVAL, "maps describe no adapter token list");
  FLEXCO_CHECK(aligned16(y) && aligned16(saved_in) && aligned16(ws) && aligned16(ad->w_down) && aligned16(ad->w_up),
               FLEXCO_EINVAL, "misaligned pointer");
  hipStream_t s = (hipStream_t)stream;
  const size_t e = esize(dtype);
  const int b = ad->bottleneck;
  if (saved_in && m.n_ft > 0) {   // the window's input rows, kept for the backward pass
    FLEXCO_CHECK(m.ft_pos0 + m.n_ft <= seq_len, FLEXCO_ESHAPE, "finetune window [%d, %d) exceeds seq_len %d", m.ft_pos0,
                 m.ft_pos0 + m.n_ft, seq_len);
    EW(launch_copy_rows(boff(y, (size_t)m.ft_tok0 * hidden, e), hidden * e, boff(saved_in, (size_t)m.ft_pos0 * hidden, e),
                        hidden * e, m.n_ft, hidden * e, s));
  }
  if (m.n_lora == 0) return FLEXCO_OK;
  const size_t need = adapter_fwd_bytes(dtype, hidden, b, m.T, m.n_lora);
  FLEXCO_CHECK(ws != nullptr && ws_bytes >= need, FLEXCO_EWORKSPACE, "adapter forward needs %zu workspace bytes, got %zu",
               need, ws_bytes);
  if (adapter_mfma_ok(dtype, hidden, b)) {
    // r = relu(y W_down^T) for every token row in bf16 (zero rows where the token carries no adapter), then
    // y += r W_up^T as a projection with K = b whose residual is y itself
    LoraShrinkArgs sa;
    memset(&sa, 0, sizeof(sa));
    sa.X[0] = (const bf16_t*)y; sa.ldx[0] = hidden; sa.S[0] = (const bf16_t*)ad->w_down; sa.lds[0] = hidden; sa.K[0] = hidden;
    sa.out_ext[0] = (bf16_t*)ws; sa.row_adapter = m.tok_adapter; sa.want[0] = -1; sa.rows = m.T; sa.r = b; sa.scale = 1.f;
    sa.relu = 1;
    LR(launch_lora_shrink_mfma(sa, 1, s));
    const int32_t rc = launch_gemm(ws, ad->w_up, y, nullptr, y, m.T, hidden, b, b, b, hidden, hidden, false, dtype, s, nullptr,
                                   nullptr, 0);
    if (rc != FLEXCO_EUNSUPPORTED) return rc;
    return fail(FLEXCO_EUNSUPPORTED, "adapter forward: the K = %d projection is not covered", b);
  }
  float* u = (float*)ws;
  KernelTimerScope ts(FLEXCO_K_LORA, s);
  FLEXCO_TRY(launch_lora_shrink(y, hidden, ad->w_down, u, m.n_lora, hidden, b, dtype, m.lora_tok, s));
  FLEXCO_TRY(launch_relu_mask(u, nullptr, (size_t)m.n_lora * b, s));
  return launch_lora_expand(u, ad->w_up, y, hidden, m.n_lora, hidden, b, 1.f, dtype, m.lora_tok, s);
}

extern "C" int32_t flexco_adapter_bwd(int32_t dtype, int32_t hidden, const flexco_adapter* ad, const void* saved_in,
                                      int32_t seq_len, int32_t win_start, int32_t win_len, void* dY, void* ws,
                                      size_t ws_bytes, void* stream) {
  clear_error();
  FLEXCO_TRY(check_adapter(dtype, hidden, ad, true));
  FLEXCO_CHECK(saved_in && dY && ws, FLEXCO_EINVAL, "NULL argument");
  FLEXCO_CHECK(win_start >= 0 && win_len > 0, FLEXCO_EINVAL, "window [%d, +%d) is invalid", win_start, win_len);
  FLEXCO_CHECK(win_start + win_len <= seq_len, FLEXCO_ESHAPE, "window end %d exceeds seq_len %d", win_start + win_len, seq_len);
  FLEXCO_CHECK(aligned16(saved_in) && aligned16(dY) && aligned16(ws) && aligned16(ad->w_down) && aligned16(ad->w_up),
               FLEXCO_EINVAL, "misaligned pointer");
  const int b = ad->bottleneck, n = win_len;
  const size_t need = adapter_bwd_bytes(dtype, hidden, b, n);
  FLEXCO_CHECK(ws_bytes >= need, FLEXCO_EWORKSPACE, "adapter backward needs %zu workspace bytes, got %zu", need, ws_bytes);
  hipStream_t s = (hipStream_t)stream;
  Carver cv{(char*)ws};
  float* u = (float*)cv.take(sizeof(float) * (size_t)n * b);
  float* t = (float*)cv.take(sizeof(float) * (size_t)n * b);
  const void* x_w = boff(saved_in, (size_t)win_start * hidden, esize(dtype));
  if (adapter_mfma_ok(dtype, hidden, b)) {
    bf16_t* t_ext = (bf16_t*)cv.take(sizeof(bf16_t) * (size_t)n * b);
    bf16_t* w_up_t = (bf16_t*)cv.take(sizeof(bf16_t) * (size_t)b * hidden);
    // u = relu(x W_down^T) and t = dY W_up in one launch, t masked by the ReLU
    LoraTransposeArgs ta;
    memset(&ta, 0, sizeof(ta));
    ta.B[0] = (const bf16_t*)ad->w_up; ta.Bt[0] = w_up_t; ta.out[0] = hidden; ta.r = b;
    LR(launch_lora_transpose(ta, 1, s));
    LoraShrinkArgs sa;
    memset(&sa, 0, sizeof(sa));
    sa.rows = n; sa.r = b; sa.scale = 1.f; sa.f32_lo = 0; sa.f32_hi = n; sa.relu = 1;
    sa.X[0] = (const bf16_t*)x_w; sa.ldx[0] = hidden; sa.S[0] = (const bf16_t*)ad->w_down; sa.lds[0] = hidden; sa.K[0] = hidden;
    sa.out_f32[0] = u;
    sa.X[1] = (const bf16_t*)dY; sa.ldx[1] = hidden; sa.S[1] = w_up_t; sa.lds[1] = hidden; sa.K[1] = hidden; sa.out_f32[1] = t;
    LR(launch_lora_shrink_mfma(sa, 2, s));
    LR(launch_relu_bwd_mask(u, t, t_ext, (size_t)n * b, s));
    // dW_up[o, j] += sum_m dY[m, o] u[m, j];  dW_down[j, i] += sum_m x[m, i] t[m, j]   (before dY changes)
    LoraOuterArgs outer;
    memset(&outer, 0, sizeof(outer));
    outer.n = n; outer.r = b; outer.scale = 1.f; outer.count = 2;
    outer.X[0] = (const bf16_t*)dY; outer.ldx[0] = hidden; outer.U[0] = u; outer.G[0] = ad->dw_up; outer.g_i[0] = b;
    outer.g_j[0] = 1; outer.n_long[0] = hidden;
    outer.X[1] = (const bf16_t*)x_w; outer.ldx[1] = hidden; outer.U[1] = t; outer.G[1] = ad->dw_down; outer.g_i[1] = 1;
    outer.g_j[1] = hidden; outer.n_long[1] = hidden;
    LR(launch_lora_outer_batch(outer, s));
    // dY += t W_down: the input-gradient form with K = b, dY as its own residual
    const int32_t rc = launch_gemm(t_ext, ad->w_down, dY, nullptr, dY, n, hidden, b, b, hidden, hidden, hidden, true, dtype, s,
                                   nullptr, nullptr, 0);
    if (rc != FLEXCO_EUNSUPPORTED) return rc;
    return fail(FLEXCO_EUNSUPPORTED, "adapter backward: the K = %d projection is not covered", b);
  }
  KernelTimerScope ts(FLEXCO_K_LORA, s);
  // u = relu(x W_down^T); t = (dY W_up) masked; dW_up += dY^T u; dW_down += t^T x; dY += t W_down
  return launch_lora_bwd(x_w, hidden, dY, hidden, ad->w_down, ad->w_up, ad->dw_down, ad->dw_up, dY, hidden, u, t, n, hidden,
                         hidden, b, 1.f, dtype, s, true);
}

// ---- all layers of a model in one call ---------------------------------------------------------------
// The loops of Alg. 2 over the layers (its Forward loop and its Backward loop for one window), on the host side
// of the boundary: one call enqueues every layer's kernels, so a caller's per-layer loop - and whatever its
// language costs per call - is gone.  Every layer is validated before the first launch of its own pass.
extern "C" int32_t flexco_model_forward(const flexco_layer_cfg* cfg, const flexco_model_layer* layers, int32_t n_layers,
                                        const flexco_maps* maps, const void* x_in, void* x_out, void* x_tmp, void* ws,
                                        size_t ws_bytes, void* stream) {
  clear_error();
  FLEXCO_CHECK(layers != nullptr && n_layers > 0, FLEXCO_EINVAL, "no layers");
  FLEXCO_CHECK(x_in && x_out, FLEXCO_EINVAL, "x_in or x_out is NULL");
  FLEXCO_CHECK(n_layers == 1 || x_tmp, FLEXCO_EINVAL, "more than one layer needs the second activation buffer x_tmp");
  FLEXCO_CHECK(x_tmp != x_out && x_tmp != x_in && x_in != x_out, FLEXCO_EINVAL, "x_in, x_out and x_tmp must be three buffers");
  // layer i writes x_out when the number of layers after it is even, so that the last one does
  const void* src = x_in;
  for (int i = 0; i < n_layers; ++i) {
    void* dst = ((n_layers - 1 - i) % 2 == 0) ? x_out : x_tmp;
    const flexco_model_layer& l = layers[i];
    const Adapters ad{l.lora, l.lora ? 1 : 0, true};
    const int32_t rc = layer_forward_impl(cfg, &l.w, ad, maps, src, dst, &l.pool, l.ft, ws, ws_bytes, stream);
    if (rc != FLEXCO_OK) return rc;
    src = dst;
  }
  return FLEXCO_OK;
}

extern "C" int32_t flexco_model_backward(const flexco_layer_cfg* cfg, const flexco_model_layer* layers, int32_t n_layers,
                                         const int32_t* seq_pages, int32_t n_seq_pages, int32_t win_start, int32_t win_len,
                                         void* dY, void* d_tmp, int32_t need_dx0, void** dx0_out, void* ws, size_t ws_bytes,
                                         void* stream) {
  clear_error();
  FLEXCO_CHECK(layers != nullptr && n_layers > 0, FLEXCO_EINVAL, "no layers");
  FLEXCO_CHECK(dY && d_tmp && dY != d_tmp, FLEXCO_EINVAL, "dY and d_tmp must be two buffers");
  void* cur = dY;
  void* nxt = d_tmp;
  for (int i = n_layers - 1; i >= 0; --i) {
    const flexco_model_layer& l = layers[i];
    FLEXCO_CHECK(l.ft != nullptr, FLEXCO_EINVAL, "layer %d has no finetune state", i);
    void* dx = (i > 0 || need_dx0) ? nxt : nullptr;       // nothing trainable below the bottom layer (Alg. 1)
    const int32_t rc = layer_backward_impl(cfg, &l.w, l.lora, nullptr, &l.pool, seq_pages, n_seq_pages, l.ft, win_start,
                                           win_len, cur, dx, ws, ws_bytes, stream);
    if (rc != FLEXCO_OK) return rc;
    if (dx) { void* t = cur; cur = nxt; nxt = t; }
  }
  if (dx0_out) *dx0_out = need_dx0 ? cur : nullptr;
  return FLEXCO_OK;
}


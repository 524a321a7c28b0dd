/*
 * flexco — one co-serving iteration of a LoRA-augmented decoder layer over a mixed
 * token batch, for AMD MI355X (gfx950).  C ABI.
 *
 * Method: FlexLLM, "Co-Serving Large Language Model Inference and Parameter-Efficient
 * Finetuning" (arXiv 2402.18789).  Section / algorithm numbers below refer to it.
 *
 * Conventions (all entry points)
 *   - Every function returns an int32 status: FLEXCO_OK or a negative FLEXCO_E* code.
 *     flexco_last_error() gives a thread-local, human-readable message for the last
 *     failure on the calling thread.  No exception crosses this boundary.
 *   - The caller owns ALL memory.  The library never allocates or frees device memory
 *     and never synchronises: work is enqueued on `stream` (a hipStream_t passed as
 *     void*, NULL = the default stream) and the call returns.
 *   - "device" pointers are GPU global memory, 16-byte aligned, dense, row-major.
 *     "host" pointers are ordinary process memory.  Which is which is stated per
 *     argument; the library cannot check it.
 *   - Validation is done on the host before anything is launched; a failing call
 *     launches nothing.
 *   - Storage type `dtype`: FLEXCO_F32 or FLEXCO_BF16 for activations, weights, LoRA
 *     matrices and the caches.  Accumulators (LoRA gradients, KV-gradient accumulator,
 *     log-sum-exp) are always float.
 *   - Every weight matrix, LoRA matrices included, is stored [out_features, in_features]
 *     (the layout of the HuggingFace checkpoints the paper's runtime loads, Sec. 7).
 *     In the paper's notation Y = f_B(X) + f_A(X) (Sec. 4.1) with
 *     f_A(X) = scale * (X A^T) B^T,  A [r, in],  B [out, r].
 *   - Gradients are ACCUMULATED into (dA, dB, dk_accum, dv_accum): the caller zeroes
 *     them when a new finetuning mini-batch starts.
 */
#ifndef FLEXCO_H
#define FLEXCO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FLEXCO_OK            0
#define FLEXCO_EINVAL       (-1)  /* null / misaligned pointer, negative or zero size            */
#define FLEXCO_ESHAPE       (-2)  /* inconsistent dimensions                                     */
#define FLEXCO_EWORKSPACE   (-3)  /* workspace or blob too small                                 */
#define FLEXCO_EPAGE        (-4)  /* page id out of range, kv_len beyond pages, duplicate slot   */
#define FLEXCO_EUNSUPPORTED (-5)  /* valid request this build cannot run                         */
#define FLEXCO_EHIP         (-6)  /* a HIP runtime call failed                                   */

#define FLEXCO_F32  0
#define FLEXCO_BF16 1

/* LoRA targets, bit order of lora_targets and index order of flexco_lora arrays. */
#define FLEXCO_T_Q 0
#define FLEXCO_T_K 1
#define FLEXCO_T_V 2
#define FLEXCO_T_O 3
#define FLEXCO_T_GATE 4
#define FLEXCO_T_UP 5
#define FLEXCO_T_DOWN 6
#define FLEXCO_N_TARGETS 7

/* Request kinds of the mixed batch (Sec. 6.2: inference tokens scheduled first, then a
 * window of finetuning tokens appended). */
#define FLEXCO_DECODE   0
#define FLEXCO_PREFILL  1
#define FLEXCO_FINETUNE 2

/* Column tiles one attention work item carries at most (neighbouring tiles of one request). */
#define FLEXCO_ATTN_ITEM_TILES 4

/* Adapter ids of a batch are indices into the adapter array of the forward call: 0 .. 7. */
#define FLEXCO_MAX_ADAPTERS 8

typedef struct flexco_layer_cfg {
  int32_t hidden;        /* H                                             */
  int32_t n_q_heads;     /* nq                                            */
  int32_t n_kv_heads;    /* nkv, divides nq                               */
  int32_t head_dim;      /* d, even                                       */
  int32_t ffn;           /* F                                             */
  int32_t dtype;         /* FLEXCO_F32 | FLEXCO_BF16                      */
  int32_t page_size;     /* positions per KV page                         */
  int32_t lora_rank;     /* r (<= 64)                                     */
  int32_t lora_targets;  /* bitmask, bit FLEXCO_T_*                       */
  float   rms_eps;
  float   rope_theta;    /* rotary base; pairs (i, i + d/2), angle pos * theta^(-2i/d) */
  float   lora_scale;    /* alpha / r                                     */
} flexco_layer_cfg;

/* Frozen backbone weights of one layer (device, dtype of cfg). */
typedef struct flexco_base_weights {
  const void* wqkv;  /* [(nq + 2 nkv) d, H]: q rows, then k rows, then v rows      */
  const void* bqkv;  /* [(nq + 2 nkv) d] or NULL                                   */
  const void* wo;    /* [H, nq d]                                                  */
  const void* wgu;   /* [2F, H]: gate rows, then up rows                           */
  const void* wd;    /* [H, F]                                                     */
  const void* g1;    /* [H] RMSNorm gain before attention                          */
  const void* g2;    /* [H] RMSNorm gain before the MLP                            */
} flexco_base_weights;

/* One LoRA adapter (device).  Entry t is used iff bit t of cfg.lora_targets is set. */
typedef struct flexco_lora {
  const void* A[FLEXCO_N_TARGETS];   /* [r, in]   dtype of cfg                     */
  const void* B[FLEXCO_N_TARGETS];   /* [out, r]  dtype of cfg                     */
  float*      dA[FLEXCO_N_TARGETS];  /* [r, in]   float, accumulated (backward)    */
  float*      dB[FLEXCO_N_TARGETS];  /* [out, r]  float, accumulated (backward)    */
} flexco_lora;

/* The mixed batch as the scheduler hands it over (host arrays of n_req entries). */
typedef struct flexco_batch_desc {
  int32_t        n_req;
  const int32_t* kind;          /* FLEXCO_DECODE | PREFILL | FINETUNE                      */
  const int32_t* start_pos;     /* positions [0, start_pos) of the sequence are cached     */
  const int32_t* n_new;         /* tokens of this request in the batch (> 0)               */
  const int32_t* adapter;       /* -1: base model only; >= 0: LoRA adapter id              */
  const int32_t* req_page_off;  /* [n_req + 1] offsets into req_pages                      */
  const int32_t* req_pages;     /* physical page ids of each request's sequence, in order  */
} flexco_batch_desc;

/* Index maps of a mixed batch.  All arrays are int32 and live in ONE caller-owned blob,
 * so a batch is uploaded with a single copy; the struct holds pointers into the blob
 * (host pointers as filled by flexco_build_maps, device pointers after
 * flexco_maps_rebase).  The scalar fields are always host values.
 *
 * Conventions (the paper fixes none of them): tokens are laid out request by request in
 * the order given; token i of a request has position start_pos + i; kv_len = start_pos +
 * n_new; slot = pages[pos / page_size] * page_size + pos % page_size; block_table row r
 * = the first ceil(kv_len_r / page_size) pages of request r padded with -1 to max_pages
 * (>= 1) columns; ft_tok = ascending indices of finetune tokens; LoRA segments = maximal
 * runs of tokens with equal adapter id; adapter ids are -1 (base model only) or
 * 0 .. FLEXCO_MAX_ADAPTERS - 1.
 *
 * The attention work list is a pure function of the batch: each request's tokens are cut
 * into column tiles of tile_tokens = max(1, 16 / (nq / nkv)) tokens (a decode request is
 * one tile); a tile's visible key range [0, last position of the tile] is cut into splits
 * of kv_split_pages pages and has one partial-result row per split.  A work item = up to
 * FLEXCO_ATTN_ITEM_TILES neighbouring tiles of one request x one split of the last of these
 * tiles' key range (an earlier tile of the item whose own range ends before that split has no
 * partial row for it).  Order of the items: see flexco_build_maps. */
typedef struct flexco_maps {
  int32_t T, n_req, n_ft, n_seg, max_pages, page_size;
  int32_t n_tiles, n_items, n_parts;   /* n_parts = sum over tiles of their split count   */
  int32_t tile_tokens, kv_split_pages;
  int32_t ft_req;                      /* index of the finetune request, -1 if none       */
  int32_t ft_tok0, ft_pos0;            /* its first token index and first position        */
  int32_t n_lora;                      /* tokens whose segment has adapter >= 0           */
  int32_t max_kv_len;
  int32_t blob_ints;                   /* int32 words used in the blob                    */
  int32_t n_adapters;                  /* 1 + the largest adapter id of the batch (0: none) */
  int32_t ft_adapter;                  /* adapter id of the finetune request (-1: none)   */
  int32_t num_pages;                   /* pool size the page ids were checked against: a call that takes
                                          these maps and a pool with fewer pages fails with FLEXCO_EPAGE */
  int32_t n_single;                    /* work items that are one tile of one token: the decode stream (and a
                                          chunk's last token where it falls into an item of its own)          */
  int32_t stream_pages;                /* K / V pages those items read (what the decode stream costs)         */
  int32_t chunk_tile_pages;            /* sum over the other items of pages x column tiles (what the chunks'
                                          products cost); both capped at INT32_MAX                            */
  int32_t adapter_tok_off[FLEXCO_MAX_ADAPTERS + 1];   /* lora_tok[off[a] .. off[a+1]) = tokens of adapter a */
  const int32_t* tok_req;       /* [T]                                                    */
  const int32_t* tok_pos;       /* [T]                                                    */
  const int32_t* slot;          /* [T]                                                    */
  const int32_t* req_tok_off;   /* [n_req + 1]                                            */
  const int32_t* req_kv_len;    /* [n_req]                                                */
  const int32_t* req_kind;      /* [n_req]                                                */
  const int32_t* block_table;   /* [n_req, max_pages]                                     */
  const int32_t* ft_tok;        /* [n_ft]                                                 */
  const int32_t* seg_off;       /* [n_seg + 1]                                            */
  const int32_t* seg_adapter;   /* [n_seg]                                                */
  const int32_t* lora_tok;      /* [n_lora] tokens with adapter >= 0, grouped by adapter id
                                   (ascending), ascending inside a group                  */
  const int32_t* tile_req;      /* [n_tiles]                                              */
  const int32_t* tile_tok0;     /* [n_tiles] first token of the tile                      */
  const int32_t* tile_ntok;     /* [n_tiles] tokens in the tile                           */
  const int32_t* tile_nsplit;   /* [n_tiles]                                              */
  const int32_t* tile_part0;    /* [n_tiles] first partial-result row of the tile         */
  const int32_t* item_tile;     /* [n_items] first tile of the work item                  */
  const int32_t* item_split;    /* [n_items] its key split                                */
  const int32_t* tok_tile;      /* [T] tile of each token                                 */
  const int32_t* tok_lora;      /* [T] index of the token in lora_tok, -1 without adapter */
  const int32_t* tok_adapter;   /* [T] adapter id of the token's request                  */
  const int32_t* item_ntiles;   /* [n_items] tiles of the work item: item_tile .. + ntiles */
} flexco_maps;

/* Paged KV cache of one layer (device, dtype of cfg).  Sec. 7, memory management.
 *   k_pages [num_pages, nkv, page_size, d]   keys after RoPE
 *   v_pages [num_pages, nkv, d, page_size]   values, position-minor inside a page     */
typedef struct flexco_kv_pool {
  void*   k_pages;
  void*   v_pages;
  int32_t num_pages;
  int32_t page_size;
} flexco_kv_pool;

/* Per-layer state of ONE finetuning sequence of seq_len rows (device).  Alg. 2 keeps a
 * Q/K/V cache per layer: K and V live in the paged pool like any sequence's, Q here.
 * saved_* are the activations graph pruning (Alg. 1) leaves alive for this layer:
 * x, x2 (input of the second norm), gate, up; the attention output and the softmax
 * log-sum-exp are kept in addition (8 KB + 128 B per token at 8B shape) so that the
 * backward pass needs no second forward pass over the keys.
 * saved_u[t] (optional, NULL = not kept): the rank-r product x_t A_t^T of LoRA target t in fp32
 * (4 r bytes per token and target): with it the backward pass does not multiply the saved inputs
 * by A_t again for the dB_t gradient.  Either every target of cfg.lora_targets has one or none.
 * saved_k0 / saved_v0: only for the (IA)^3 entry points, the other operand of the two products whose
 * vectors are trained (2 nkv d elements per token on top of the set above).
 * dk_accum / dv_accum: the statically allocated KV-gradient accumulator of Sec. 7. */
typedef struct flexco_ft_state {
  int32_t seq_len;
  void*  q_cache;     /* [L, nq d]  after RoPE        */
  void*  saved_x;     /* [L, H]                       */
  void*  saved_x2;    /* [L, H]                       */
  void*  saved_gate;  /* [L, F]                       */
  void*  saved_up;    /* [L, F]                       */
  void*  saved_attn;  /* [L, nq d]                    */
  float* lse;         /* [L, nq]                      */
  float* dk_accum;    /* [L, nkv d] float             */
  float* dv_accum;    /* [L, nkv d] float             */
  float* saved_u[FLEXCO_N_TARGETS];   /* [L, r] float or NULL */
  void*  saved_k0;    /* [L, nkv d] key projection output before the (IA)^3 scale; NULL unless (IA)^3 */
  void*  saved_v0;    /* [L, nkv d] value projection output before the (IA)^3 scale; NULL unless (IA)^3 */
} flexco_ft_state;

/* Message for the last failing call on this thread ("" if none). */
const char* flexco_last_error(void);

/* Library ABI version (increases when a struct above changes). */
int32_t flexco_abi_version(void);

/* Upper bound of the int32 words flexco_build_maps needs for `desc` (host only). */
int32_t flexco_maps_blob_ints(const flexco_batch_desc* desc, int32_t page_size,
                              int32_t n_q_heads, int32_t n_kv_heads, int32_t kv_split_pages,
                              size_t* out_ints);

/* Builds the index maps of a mixed batch on the host (Sec. 6.2: the scheduler's output is
 * this call's input).  desc, blob: host.  blob_ints: capacity of blob in int32 words.
 * num_pages: size of the pool the page ids refer to.  kv_split_pages: 0 = default (128 - 256 when no request sees more pages than that, so that nothing needs merging, or when the one-token requests' pages outweigh the other requests' pages x column tiles -, or down to 8 for batches too small to fill the chip); at most 256 on the matrix-core path.
 * Errors: EINVAL (null, non-positive sizes, unknown kind), EPAGE (page id outside
 * [0, num_pages), kv_len beyond the request's pages, two tokens on one slot),
 * EUNSUPPORTED (more than one finetune request), EWORKSPACE (blob too small). */
int32_t flexco_build_maps(const flexco_batch_desc* desc, int32_t page_size, int32_t num_pages,
                          int32_t n_q_heads, int32_t n_kv_heads, int32_t kv_split_pages,
                          int32_t* blob, size_t blob_ints, flexco_maps* out);

/* Rewrites the pointers of `host_maps` (pointing into host_blob) so that they point into
 * a copy of the blob at `other_blob` (typically device memory).  Host only. */
int32_t flexco_maps_rebase(const flexco_maps* host_maps, const int32_t* host_blob,
                           const int32_t* other_blob, flexco_maps* out);

/* Bytes of device workspace that flexco_layer_forward / flexco_attention_mixed /
 * flexco_lora_bwd need for batches of at most T_max tokens with at most n_parts_max
 * attention partial rows, and backward windows of at most win_max rows over at most
 * kv_max cached positions. */
int32_t flexco_workspace_bytes(const flexco_layer_cfg* cfg, int32_t T_max, int32_t n_parts_max,
                               int32_t win_max, int32_t kv_max, size_t* out_bytes);

/* One forward iteration of the layer over the mixed batch (Sec. 6.2 fused forward;
 * Alg. 2 Forward + Append for the finetune window).
 *   maps     : device-rebased maps of the batch
 *   x_in     : device [T, H]; x_out: device [T, H] (may not alias x_in)
 *   pool     : this layer's cache; K/V of the batch's tokens are appended at their slots
 *   ft       : state of the finetune sequence, NULL iff the batch has no finetune request;
 *              rows [start_pos, start_pos + n_new) of q_cache, saved_*, lse are written
 *   lora     : adapter applied to tokens whose segment has adapter >= 0 (NULL: none)
 * Base projections run over all T tokens at once; LoRA only on adapter rows. */
int32_t flexco_layer_forward(const flexco_layer_cfg* cfg, const flexco_base_weights* w,
                             const flexco_lora* lora, const flexco_maps* maps,
                             const void* x_in, void* x_out, const flexco_kv_pool* pool,
                             const flexco_ft_state* ft, void* ws, size_t ws_bytes, void* stream);

/* The same forward pass with the requests of the batch served by several LoRA adapters (Sec. 6.2:
 * the inference requests co-served with a finetuning job may belong to different PEFT models of
 * the one backbone): a request with adapter id a >= 0 uses adapters[a], a < n_adapters <=
 * FLEXCO_MAX_ADAPTERS; id -1 is the base model alone.  All adapters have cfg's rank, targets and
 * scale.  The finetune window's rows use the adapter of its request, which is the one
 * flexco_lora_bwd then trains.  (flexco_layer_forward applies its one adapter to every request
 * with an id >= 0.) */
int32_t flexco_layer_forward_multi(const flexco_layer_cfg* cfg, const flexco_base_weights* w,
                                   const flexco_lora* adapters, int32_t n_adapters, const flexco_maps* maps,
                                   const void* x_in, void* x_out, const flexco_kv_pool* pool,
                                   const flexco_ft_state* ft, void* ws, size_t ws_bytes, void* stream);

/* Mixed attention (Sec. 6.2): every token attends to positions 0..own position of its
 * own sequence through the block table; decode tokens, prefill chunks and finetune
 * windows in one launch sequence.
 *   q   : device [T, nq d], after RoPE; the batch's K/V must already be in the pool
 *   out : device [T, nq d];  lse: device float [T, nq] or NULL */
int32_t flexco_attention_mixed(const flexco_layer_cfg* cfg, const flexco_maps* maps,
                               const void* q, const flexco_kv_pool* pool, void* out, float* lse,
                               void* ws, size_t ws_bytes, void* stream);

/* Segmented LoRA forward (Sec. 4.1 bypass network): for every segment s with adapter
 * a = seg_adapter[s] >= 0 and rows [seg_off[s], seg_off[s+1]):
 *     y[rows] += scale * (x[rows] A_a^T) B_a^T.
 *   x: device [T, in]; y: device [T, out], updated in place; rows of other segments are
 *   untouched.  A_list / B_list: HOST arrays of n_adapters device pointers ([r, in] and
 *   [out, r]).  seg_off / seg_adapter: HOST arrays (n_seg + 1 and n_seg entries).
 *   u_ws: device scratch of at least T * r floats. */
int32_t flexco_lora_fwd(const void* x, void* y, int32_t T, int32_t in_features, int32_t out_features,
                        int32_t rank, float scale, int32_t dtype,
                        const void* const* A_list, const void* const* B_list, int32_t n_adapters,
                        const int32_t* seg_off, const int32_t* seg_adapter, int32_t n_seg,
                        float* u_ws, void* stream);

/* flexco_lora_fwd for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid allocation): the same call without u_ws.  The rank-r products live in
 * an array of FLEXCO_STATIC_SCRATCH_FLOATS floats (2 MiB) that is part of the library's image on every GPU
 * it runs on, held until the process ends.  The call allocates and frees nothing and does not synchronise;
 * the first call on a device looks the array's address up once (make that call outside a graph capture).
 * Errors as flexco_lora_fwd, plus EWORKSPACE when T * rank > FLEXCO_STATIC_SCRATCH_FLOATS (nothing is
 * launched).  All calls on one GPU share the one array: calls that overlap on a GPU (different streams,
 * or threads) race on it; calls ordered on one stream do not.  Nothing of an earlier call's contents is
 * read (every row is written before it is used), so the array needs no clearing. */
#define FLEXCO_STATIC_SCRATCH_FLOATS (1 << 19)
int32_t flexco_lora_fwd_static(const void* x, void* y, int32_t T, int32_t in_features, int32_t out_features,
                               int32_t rank, float scale, int32_t dtype,
                               const void* const* A_list, const void* const* B_list, int32_t n_adapters,
                               const int32_t* seg_off, const int32_t* seg_adapter, int32_t n_seg,
                               void* stream);

/* Token-level LoRA backward of one window through one layer (Alg. 2, the Backward / Add /
 * Slice / CalculateGrads steps; Sec. 6.1; Sec. 7 KV-gradient accumulator).
 * Window = rows [win_start, win_start + win_len) of the finetune sequence; windows of a
 * sequence must be visited from its end downwards.
 *   seq_pages : device int32 page ids of the sequence, n_seq_pages >= ceil(l / page_size),
 *               l = win_start + win_len; every id must lie in [0, pool->num_pages) - the array is
 *               device memory, the call cannot check it
 *   ft        : the state the forward windows filled
 *   dY        : device [win_len, H] gradient of the layer output rows
 *   dX        : device [win_len, H] gradient of the layer input rows, or NULL when no
 *               trainable parameter sits below this layer (Alg. 1 dead-output pruning)
 *   lora      : A, B read; dA, dB accumulated for every target of cfg.lora_targets
 * Effects: ft->dk_accum / dv_accum rows [0, l) += this window's contributions; rows
 * [win_start, l) are then complete and are consumed for the k/v-side gradients. */
int32_t flexco_lora_bwd(const flexco_layer_cfg* cfg, const flexco_base_weights* w,
                        const flexco_lora* lora, const flexco_kv_pool* pool,
                        const int32_t* seq_pages, int32_t n_seq_pages,
                        const flexco_ft_state* ft, int32_t win_start, int32_t win_len,
                        const void* dY, void* dX, void* ws, size_t ws_bytes, void* stream);

/* (IA)^3 as a bypass network (Sec. 4.1: Y = X (.) l = X + X (.) (l - 1)): three learned vectors per
 * layer, on the key projection's output (before its rotation), on the value projection's output and
 * on the SwiGLU product the down projection reads.  Device pointers; l_* in the dtype of cfg;
 * dl_* fp32, accumulated into by flexco_ia3_bwd (may be NULL for the forward pass). */
typedef struct flexco_ia3 {
  const void* l_k;    /* [nkv d] */
  const void* l_v;    /* [nkv d] */
  const void* l_ff;   /* [F]     */
  float* dl_k;        /* [nkv d] */
  float* dl_v;        /* [nkv d] */
  float* dl_ff;       /* [F]     */
} flexco_ia3;

/* flexco_layer_forward with an (IA)^3 network in place of LoRA (cfg->lora_targets must be 0): rows of
 * requests with adapter >= 0 are scaled, rows with adapter -1 run the base model.  Rows of the finetune
 * window store, besides the set of flexco_layer_forward, the unscaled key and value rows in
 * ft->saved_k0 / saved_v0 (both required when ft is given).  Everything else as flexco_layer_forward. */
int32_t flexco_layer_forward_ia3(const flexco_layer_cfg* cfg, const flexco_base_weights* w,
                                 const flexco_ia3* ia3, const flexco_maps* maps, const void* x_in,
                                 void* x_out, const flexco_kv_pool* pool, const flexco_ft_state* ft,
                                 void* ws, size_t ws_bytes, void* stream);

/* Token-level backward of one window through a layer with an (IA)^3 network (Alg. 2's Backward / Add /
 * Slice / CalculateGrads steps with the products' gradients in place of LoRA's): dl_k, dl_v, dl_ff are
 * accumulated (column sums over the window's rows, added in a fixed order), dX as in flexco_lora_bwd
 * (NULL: not computed; the vectors are still trained).  Arguments and effects as flexco_lora_bwd. */
int32_t flexco_ia3_bwd(const flexco_layer_cfg* cfg, const flexco_base_weights* w, const flexco_ia3* ia3,
                       const flexco_kv_pool* pool, const int32_t* seq_pages, int32_t n_seq_pages,
                       const flexco_ft_state* ft, int32_t win_start, int32_t win_len, const void* dY,
                       void* dX, void* ws, size_t ws_bytes, void* stream);

/* Bottleneck adapter as a bypass network on a layer's output rows (Sec. 4.1: a bypass network reads one
 * backbone tensor X and its output is added to one backbone tensor; here Y = X + relu(X W_down^T) W_up^T,
 * no biases).  Device pointers; weights in the call's dtype, gradients fp32 and accumulated into. */
typedef struct flexco_adapter {
  int32_t bottleneck;    /* b, 1..64 */
  const void* w_down;    /* [b, H]   */
  const void* w_up;      /* [H, b]   */
  float* dw_down;        /* [b, H], may be NULL for the forward pass */
  float* dw_up;          /* [H, b]   */
} flexco_adapter;

/* Scratch bytes of the two adapter calls for batches of at most T_max tokens and windows of at most win_max rows. */
int32_t flexco_adapter_workspace_bytes(int32_t dtype, int32_t hidden, int32_t bottleneck, int32_t T_max,
                                       int32_t win_max, size_t* out_bytes);

/* Forward of the adapter, in place on the rows of y [T, hidden] whose request carries an adapter
 * (maps->lora_tok); other rows are untouched.  Rows of the finetune window first copy their input into
 * saved_in [seq_len, hidden] at their positions (what graph pruning keeps for this network; NULL when the
 * batch has no finetune request).  ws: device scratch of flexco_adapter_workspace_bytes.
 * Call it after flexco_layer_forward on that call's x_out. */
int32_t flexco_adapter_fwd(int32_t dtype, int32_t hidden, const flexco_adapter* ad, const flexco_maps* maps,
                           void* y, void* saved_in, int32_t seq_len, void* ws, size_t ws_bytes, void* stream);

/* Backward of the adapter over the window rows [win_start, win_start + win_len) of the finetune sequence:
 * dY [win_len, hidden] holds the gradient of the adapter's output on entry and of its input on return
 * (in place); dw_down, dw_up += the window's contributions.  The ReLU output is recomputed from saved_in.
 * ws: device scratch of flexco_adapter_workspace_bytes.  Call it before flexco_lora_bwd / flexco_ia3_bwd of the
 * same layer. */
int32_t flexco_adapter_bwd(int32_t dtype, int32_t hidden, const flexco_adapter* ad, const void* saved_in,
                           int32_t seq_len, int32_t win_start, int32_t win_len, void* dY, void* ws,
                           size_t ws_bytes, void* stream);

/* ReLU that keeps a sign bitmask instead of its output (Sec. 5.2: the backward of a ReLU reads only the sign of its
 * output, so a ReLU whose output no other backward operator reads - FLEXCO_KEEP_BITMASK of flexco_prune_graph -
 * stores 1 bit per element).  x, y, dy, dx: device [n, width] dense, dtype; y may alias x and dx may alias dy.
 * mask: device [n, ceil(width / 32)] 32-bit words, bit j of word w of a row = element 32 w + j of the row is
 * > 0 (decided on the stored value of x); the unused high bits of a row's last word are written as zero.
 *   fwd: y = max(x, 0), mask written.     bwd: dx = dy where the bit is set, 0 elsewhere.
 * n <= 65535 rows per call.  Errors: EINVAL, ESHAPE, EHIP. */
int32_t flexco_relu_bitmask_fwd(const void* x, void* y, uint32_t* mask, int32_t n, int32_t width, int32_t dtype,
                                void* stream);
int32_t flexco_relu_bitmask_bwd(const void* dy, const uint32_t* mask, void* dx, int32_t n, int32_t width,
                                int32_t dtype, void* stream);

/* Attention backward of one window (the attention part of flexco_lora_bwd, exported for
 * unit parity).  q, out, dout: device [win_len, nq d] rows of the window (q after RoPE);
 * lse: device float [win_len, nq].  dq: device [win_len, nq d] (dtype of cfg), written.
 * dk_accum / dv_accum: device float [>= l, nkv d], rows [0, l) accumulated into. */
int32_t flexco_attention_window_bwd(const flexco_layer_cfg* cfg, const flexco_kv_pool* pool,
                                    const int32_t* seq_pages, int32_t n_seq_pages,
                                    int32_t win_start, int32_t win_len,
                                    const void* q, const void* out, const float* lse,
                                    const void* dout, void* dq, float* dk_accum, float* dv_accum,
                                    void* ws, size_t ws_bytes, void* stream);

/* Dense projection used by the layer (exported for unit parity and roofline timing):
 *   trans_w = 0:  C[M, N] = A[M, K] W[N, K]^T (+ bias[N]) (+ residual[M, N])
 *   trans_w = 1:  C[M, N] = A[M, K] W[K, N]                 (input-gradient form)
 * A, W, C, bias, residual: device, dtype; bias / residual may be NULL. */
int32_t flexco_gemm(const void* A, const void* W, void* C, const void* bias, const void* residual,
                    int32_t M, int32_t N, int32_t K, int32_t trans_w, int32_t dtype, void* stream);

/* How the bf16 matrix-core path would tile a product of these sizes (host arithmetic only: no GPU is touched, nothing
 * is launched) - the plan flexco_gemm, the frozen base projections over all tokens of the batch (Sec. 6.2; the gated
 * gate/up projection with N = 2 ffn) and the window backward's input-gradient products (Alg. 2; trans_w = 1) follow.
 * part_elems: floats of split-K scratch the caller has (0 = none: flexco_gemm; the layer calls bring rows x 32768 for
 * the window backward and for forward batches of at most 256 tokens).  out (host, 11 ints): out[0] = launches (1 or 2,
 * side by side in the output columns), then per launch: tile rows, tile columns, output columns covered, blocks K is
 * cut over, stages of the LDS ring; unused entries 0.  Errors: EINVAL (NULL, non-positive sizes), ESHAPE (K not a
 * multiple of 64 or N not a multiple of 8: such products run on the type-generic kernels). */
int32_t flexco_gemm_plan(int32_t M, int32_t N, int32_t K, int32_t trans_w, int64_t part_elems, int32_t* out);

/* Per-kernel timing with HIP events, for roofline measurement.  While a timer is running the
 * library records one event before and one after every launch of the kernel class
 * `kernel_id` on that launch's stream (the bf16 GEMM kernels carry the two events in their own
 * dispatch; at most max_launches launches, later ones are not timed).  flexco_kernel_timer_stop waits for the recorded events, returns the summed
 * duration in milliseconds and the number of timed launches, and releases the events.
 * Events are host-side runtime objects; no device memory is allocated.  The timer tables are
 * guarded by a lock, so launches from several host threads do not corrupt them; a measurement is only
 * meaningful when one thread issues the timed class (event pairs are handed out in arrival order). */
#define FLEXCO_K_GEMM_FWD   0   /* bf16 MFMA projection, forward form              */
#define FLEXCO_K_GEMM_BWD   1   /* bf16 MFMA projection, input-gradient form       */
#define FLEXCO_K_ATTN_FWD   2   /* bf16 MFMA mixed paged attention (partials)      */
#define FLEXCO_K_ATTN_MERGE 3   /* split merge                                     */
#define FLEXCO_K_ATTN_BWD   4   /* attention window backward (all its kernels)     */
#define FLEXCO_K_ELEMWISE   5   /* norms, RoPE/append, SwiGLU, row copies          */
#define FLEXCO_K_LORA       6   /* rank-r LoRA kernels                             */
#define FLEXCO_K_GENERIC    7   /* type-generic fallbacks (fp32 path)              */
#define FLEXCO_N_KERNEL_IDS 8
int32_t flexco_kernel_timer_start(int32_t kernel_id, int32_t max_launches);
int32_t flexco_kernel_timer_stop(int32_t kernel_id, double* total_ms, int64_t* launches);
/* Before stop: waits for the event pairs recorded so far and writes their durations in milliseconds, in issue
 * order, to ms_each[0 .. min(*n, capacity)); *n = pairs recorded (a call that issues several kernels of the
 * class - a projection whose tile plan is two launches - records one pair per kernel). */
int32_t flexco_kernel_timer_read(int32_t kernel_id, double* ms_each, int64_t capacity, int64_t* n);
/* From the next start on, only every stride-th launch of the class is timed (1, the initial
 * setting: all of them); stop then returns the sum and the count of the timed launches.  A timed
 * launch holds its neighbours on the stream apart by a few microseconds, which a caller that also
 * measures end-to-end time may not want on every launch. */
int32_t flexco_kernel_timer_sample(int32_t kernel_id, int32_t stride);

/* The matrix-core kernels cover the shapes of the configurations this library was built for (attention: bf16,
 * head_dim 128, page size 16, at most 16 query heads per kv head; projections: K a multiple of 64, 16-byte aligned
 * rows); a bf16 call outside them runs on the type-generic kernels instead, correct but far slower.  counts
 * [FLEXCO_N_KERNEL_IDS] (host) receives, per kernel class (FLEXCO_K_GEMM_FWD, _GEMM_BWD, _ATTN_FWD, _ATTN_BWD; the
 * other entries stay 0), how many bf16 launches of this process took that route; reset != 0 clears the counters. */
int32_t flexco_bf16_fallbacks(int64_t* counts, int32_t reset);

/* Which kernel takes the chunk items of the attention work list - prefill chunks and finetune windows, whose tokens
 * follow the causal pattern of prefill (Sec. 6.2) - in flexco_layer_forward*, flexco_model_forward and
 * flexco_attention_mixed: 0 = the kernel that also streams the decode tokens (one wavefront per work item), 1 = a
 * kernel of their own (four wavefronts per work item, K / V pages staged in LDS; the decode tokens stay where they
 * are) launched after the decode tokens' kernel, 2 = that kernel launched beside the decode tokens' kernel, on a side
 * stream of the library's own (default priority; created on the device's first such call, which therefore must not
 * fall inside a stream capture) that leaves the caller's stream before the attention and rejoins it after: to the
 * caller's stream the call behaves as before, also under capture; -1 = chosen by batch, the default: the kernel of
 * their own alone when the work list has no single-token item, beside the decode stream when the chunks' products
 * outweigh it (flexco_maps.chunk_tile_pages >= stream_pages), else the one kernel for everything (a light chunk load
 * hides in the decode stream's waits).  Both kernels take the same products per column tile; their results agree to
 * rounding (the kernels scale their running sums at different steps).  Process-wide; returns FLEXCO_EINVAL for other
 * values. */
int32_t flexco_attention_chunk_path(int32_t mode);

/* ---- Static graph pruning (Alg. 1, Sec. 5.2), host only -------------------------------------
 * The forward graph of a PEFT model as integer arrays: operator o has kind op_kind[o], one output
 * tensor op_out[o] and the input tensors op_in[op_in_off[o] .. op_in_off[o + 1]) in the order of
 * its kind (matmul: x, w; rmsnorm: x, gain; swiglu: gate, up; mul: a, b; attention: q, k, v; add:
 * any number; rope, relu: one; source: none - a tensor that enters the graph).  op_cheap[o] != 0
 * marks operators whose output may be recomputed rather than stored (Alg. 1's cost threshold:
 * elementwise operators, norms, rank-r products).  tensor_class says which tensors are frozen base
 * weights (their gradients are what pruning removes), which are trainable (bypass-network) weights;
 * need_grad[t] != 0 marks tensors whose gradient is handed on outside the graph (the graph input
 * when a trainable layer sits below).
 * Result, per tensor: what the backward pass needs of it.  Deterministic; no device work. */
#define FLEXCO_OP_SOURCE    0
#define FLEXCO_OP_MATMUL    1
#define FLEXCO_OP_ADD       2
#define FLEXCO_OP_RMSNORM   3
#define FLEXCO_OP_ROPE      4
#define FLEXCO_OP_ATTENTION 5
#define FLEXCO_OP_SWIGLU    6
#define FLEXCO_OP_MUL       7   /* elementwise product, e.g. the learned scaling vectors of (IA)^3 */
#define FLEXCO_OP_RELU      8   /* backward reads only the sign of the output                       */
#define FLEXCO_TENSOR_ACTIVATION 0
#define FLEXCO_TENSOR_FROZEN     1
#define FLEXCO_TENSOR_TRAINABLE  2
#define FLEXCO_KEEP_NONE    0   /* not needed by the backward pass (or a weight)                     */
#define FLEXCO_KEEP_STORE   1   /* store the activation                                              */
#define FLEXCO_KEEP_REMAT   2   /* recompute it from stored tensors and weights                      */
#define FLEXCO_KEEP_BITMASK 3   /* store its sign bitmask only (1 bit per element; Sec. 5.2)         */
typedef struct flexco_graph {
  int32_t n_ops, n_tensors;
  const int32_t* op_kind;       /* [n_ops]                        */
  const int32_t* op_cheap;      /* [n_ops]                        */
  const int32_t* op_in_off;     /* [n_ops + 1]                    */
  const int32_t* op_in;         /* [op_in_off[n_ops]] tensor ids  */
  const int32_t* op_out;        /* [n_ops] tensor ids             */
  const int32_t* tensor_class;  /* [n_tensors]                    */
  const int32_t* need_grad;     /* [n_tensors]                    */
} flexco_graph;
int32_t flexco_prune_graph(const flexco_graph* graph, int32_t* keep /* [n_tensors], FLEXCO_KEEP_* */);

/* ---- Hybrid token scheduler (Sec. 6.2), host only ------------------------------------------
 * Stage 1 chooses the inference work of an iteration (iteration-level scheduling with chunked
 * prefill); stage 2 appends the largest finetuning window that keeps the estimated iteration
 * latency within the SLO:  s = argmax f(c, s) <= SLO, c = inference tokens of the iteration, f from
 * offline profiling.  Conventions the paper leaves open: f is a table over a (c, s) grid,
 * interpolated bilinearly (beyond the grid the nearest segment is extended linearly); candidate
 * windows are the multiples of `quantum` up to s_avail, and s_avail itself; requests are served in
 * arrival (index) order; an iteration lists its decode entries first, then its prefill chunks. */
typedef struct flexco_latency_model {
  int32_t n_c, n_s;          /* grid sizes, each >= 2                                           */
  const int32_t* c_grid;     /* [n_c] inference-token counts, strictly ascending (host)         */
  const int32_t* s_grid;     /* [n_s] finetune-token counts, strictly ascending (host)          */
  const float* ms;           /* [n_c, n_s] profiled latency of one iteration, any unit (host)   */
} flexco_latency_model;

#define FLEXCO_REQ_WAITING  0
#define FLEXCO_REQ_RUNNING  1
#define FLEXCO_REQ_FINISHED 2

/* f(c, s) in double precision.  Errors: EINVAL (null, grids too short or not ascending). */
int32_t flexco_latency_estimate(const flexco_latency_model* model, int32_t c, int32_t s, double* out_ms);

/* Stage 2: *out_s = the largest candidate s <= s_avail with f(c, s) <= slo_ms, 0 if none.  Every
 * candidate is evaluated (a profiled table need not be monotone).  Errors: EINVAL. */
int32_t flexco_sched_window(const flexco_latency_model* model, int32_t c, double slo_ms, int32_t s_avail,
                            int32_t quantum, int32_t* out_s);

/* Stage 1, one iteration.  The five request arrays (host, n_req entries, arrival order) hold each
 * request's prompt length (> 0), prompt tokens already processed, tokens to generate, tokens
 * generated, and FLEXCO_REQ_* state; `state` is updated (waiting requests are admitted while fewer
 * than max_batch run).  Every running request past its prompt gets one decode token at position
 * prompt_len + generated; running requests still in their prompt get chunks of at most `chunk`
 * tokens, in order, while the iteration's token_budget lasts.  The entries (request index, kind,
 * start_pos, n_new) go to the four out arrays of out_capacity entries each; *out_n = their number,
 * *out_tokens = c.  Errors: EINVAL, EWORKSPACE (out_capacity too small). */
int32_t flexco_sched_inference(int32_t n_req, const int32_t* prompt_len, const int32_t* prefilled,
                               const int32_t* gen_len, const int32_t* generated, int32_t* state,
                               int32_t max_batch, int32_t token_budget, int32_t chunk,
                               int32_t* out_req, int32_t* out_kind, int32_t* out_start_pos, int32_t* out_n_new,
                               int32_t out_capacity, int32_t* out_n, int32_t* out_tokens);

/* Books an executed iteration: prefilled / generated advance by what the entries processed, and a
 * request with its prompt done and nothing left to generate becomes FLEXCO_REQ_FINISHED. */
int32_t flexco_sched_advance(int32_t n_entries, const int32_t* req, const int32_t* kind, const int32_t* n_new,
                             int32_t n_req, const int32_t* prompt_len, int32_t* prefilled,
                             const int32_t* gen_len, int32_t* generated, int32_t* state);

/* ---- The two ends of a finetuning step around the decoder layers ----------------------------
 * Generative loss of a forward window (Alg. 2, forward loop) and the gradient its backward pass
 * starts from.  Reading (the paper names neither head nor normalisation): next-token cross-entropy
 * through a final RMSNorm and an LM head,
 *     h = rmsnorm(x; g_final),  z = h w_lm^T,  loss_i = logsumexp(z_i) - z_i[targets_i],
 * over the rows with 0 <= targets_i < vocab (any other value: the row has no next token and
 * contributes neither loss nor gradient), times `scale` (1 / tokens of the whole sequence makes the windows of a
 * sequence add up to its mean loss). */
typedef struct flexco_lm_head {
  int32_t hidden, vocab, dtype;   /* dtype: FLEXCO_F32 | FLEXCO_BF16 (storage of g_final, w_lm, x, dX) */
  float   rms_eps;
  const void* g_final;            /* [hidden]         device */
  const void* w_lm;               /* [vocab, hidden]  device, frozen */
} flexco_lm_head;

int32_t flexco_lm_loss_workspace_bytes(const flexco_lm_head* head, int32_t n_max, size_t* out_bytes);

/* x: device [n, hidden], the window's rows of the last layer's output; targets: device int32 [n];
 * loss_accum: device float[1], scale * sum_i loss_i is ADDED to it (rows summed in a fixed order);
 * dX: device [n, hidden], written = d(scale * sum loss_i) / dx, what flexco_lora_bwd of the last
 * layer takes as dY.  ws: device workspace of flexco_lm_loss_workspace_bytes(head, >= n) bytes.
 * Errors: EINVAL, EWORKSPACE, EHIP. */
int32_t flexco_lm_loss(const flexco_lm_head* head, const void* x, const int32_t* targets, int32_t n,
                       float scale, float* loss_accum, void* dX, void* ws, size_t ws_bytes, void* stream);

/* One Adam update (Kingma & Ba, with bias correction, no weight decay; the optimizer named in the
 * paper's setup) of n parameters:  m <- b1 m + (1 - b1) g,  v <- b2 v + (1 - b2) g^2,
 * p <- p - lr (m / (1 - b1^step)) / (sqrt(v / (1 - b2^step)) + eps).  param: device, dtype (bf16
 * or f32); master: device float[n] or NULL - with a master copy the update is applied to it in
 * fp32 and param receives its rounded value; grad, m, v: device float[n].  step counts from 1. */
int32_t flexco_adam_step(void* param, float* master, const float* grad, float* m, float* v, size_t n,
                         int32_t dtype, float lr, float beta1, float beta2, float eps, int32_t step,
                         void* stream);

/* ---- A whole model in one call (Alg. 2: its Forward and Backward loops over the layers) -------------
 * One layer's device objects.  lora: NULL when the configuration has no LoRA targets.  ft: the finetune
 * sequence's state in this layer (NULL only for flexco_model_forward on a batch without a finetune request). */
typedef struct flexco_model_layer {
  flexco_base_weights    w;
  const flexco_lora*     lora;
  flexco_kv_pool         pool;
  const flexco_ft_state* ft;
} flexco_model_layer;

/* flexco_layer_forward through layers[0 .. n_layers) in order, all with the same configuration and the same
 * batch (maps).  x_in: device [T, H], not modified; x_out: device [T, H], the last layer's output; x_tmp: device
 * [T, H], scratch for the layers in between (may be NULL when n_layers == 1); the three must be distinct.
 * ws as for one layer (the layers run one after the other on `stream`).  Errors: those of flexco_layer_forward;
 * a failing layer stops the call (earlier layers' work stays enqueued). */
int32_t flexco_model_forward(const flexco_layer_cfg* cfg, const flexco_model_layer* layers, int32_t n_layers,
                             const flexco_maps* maps, const void* x_in, void* x_out, void* x_tmp, void* ws,
                             size_t ws_bytes, void* stream);

/* flexco_lora_bwd of one window through layers[n_layers - 1] down to layers[0].  dY: device [win_len, H], the
 * gradient of the top layer's output rows on entry; dY and d_tmp (device [win_len, H]) are used in turn for the
 * gradients handed down, so dY is overwritten.  need_dx0 == 0: the bottom layer computes no input gradient
 * (nothing trainable below it).  *dx0_out (host, may be NULL) receives the buffer (dY or d_tmp) that holds the
 * bottom layer's input gradient, or NULL.  Errors: those of flexco_lora_bwd. */
int32_t flexco_model_backward(const flexco_layer_cfg* cfg, const flexco_model_layer* layers, int32_t n_layers,
                              const int32_t* seq_pages, int32_t n_seq_pages, int32_t win_start, int32_t win_len,
                              void* dY, void* d_tmp, int32_t need_dx0, void** dx0_out, void* ws, size_t ws_bytes,
                              void* stream);

/* Machine-ceiling probes for the benchmark (they compute nothing of the method): what this GPU
 * sustains for the two resources the rooflines are quoted against.  Both only enqueue one kernel
 * on `stream`; the caller times it with events.  sink: device, >= 4 bytes, never written in
 * practice (it keeps the compiler from removing the work).
 *   flexco_probe_mfma: `blocks` blocks of 4 wavefronts, each `iters` x 16 back-to-back
 *     v_mfma_f32_32x32x16_bf16 on register operands with values in [-1, 1); *flops = work enqueued.
 *   flexco_probe_read: `blocks` blocks each stream their own contiguous piece of src[0, bytes) with
 *     16-byte loads; *bytes_read = bytes actually read (bytes rounded down to whole rounds).
 *   flexco_probe_mfma_lds: the same products with the operands fetched from LDS as the projection kernels fetch
 *     them, one 16-column slice ahead of the products (tile = 128: 2 x 2 wavefronts on a 128 x 128 tile, where the
 *     LDS reads take as long as the products; tile = 256: a 256 x 256 tile, half as long); `iters` 64-column
 *     stages per wavefront.  src == NULL: no global memory traffic and no barriers.  src != NULL (device, 16-byte
 *     aligned, at least 8 x 2 x tile x 64 x 2 bytes of finite bf16 values): every stage also loads a stage of tile
 *     bytes from src straight into LDS and ends with a barrier - the projection kernels' k-loop without its wait
 *     for memory. */
int32_t flexco_probe_mfma(int32_t blocks, int32_t iters, void* sink, double* flops, void* stream);
int32_t flexco_probe_mfma_lds(int32_t blocks, int32_t iters, int32_t tile, const void* src, size_t src_bytes,
                              void* sink, double* flops, void* stream);
int32_t flexco_probe_read(const void* src, size_t bytes, int32_t blocks, void* sink, double* bytes_read,
                          void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FLEXCO_H */

// Host side of the boundary: error reporting and the index maps of a mixed batch.
//
// The hybrid token scheduler (Sec. 6.2 of the paper) decides which inference requests and
// how many finetuning tokens share an iteration; this file turns that decision into the
// integer arrays the kernels index with.  Pure host code, no device calls.
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <algorithm>
#include <unordered_set>
#include <vector>

#include "flexco_host.h"

namespace flexco {

static thread_local char g_err[512] = "";

int32_t fail(int32_t code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}
void clear_error() { g_err[0] = 0; }

namespace {

struct Built {
  std::vector<int32_t> tok_req, tok_pos, slot, req_tok_off, req_kv_len, req_kind, block_table, ft_tok,
      seg_off, seg_adapter, lora_tok, tile_req, tile_tok0, tile_ntok, tile_nsplit, tile_part0, item_tile,
      item_split, tok_tile, tok_lora, tok_adapter, item_ntiles;
  int32_t n_adapters = 0, adapter_tok_off[FLEXCO_MAX_ADAPTERS + 1] = {0};
  int32_t T = 0, n_ft = 0, n_seg = 0, max_pages = 1, n_parts = 0, ft_req = -1, max_kv_len = 0;
  int32_t tile_tokens = 1, split_pages = 64, ft_pos0 = 0;
};

int32_t validate_desc(const flexco_batch_desc* d, int32_t page_size, int32_t nq, int32_t nkv) {
  FLEXCO_CHECK(d != nullptr, FLEXCO_EINVAL, "batch descriptor is NULL");
  FLEXCO_CHECK(d->n_req > 0, FLEXCO_EINVAL, "n_req must be positive (got %d)", d->n_req);
  FLEXCO_CHECK(d->kind && d->start_pos && d->n_new && d->adapter && d->req_page_off && d->req_pages,
               FLEXCO_EINVAL, "batch descriptor has a NULL array");
  FLEXCO_CHECK(page_size > 0, FLEXCO_EINVAL, "page_size must be positive (got %d)", page_size);
  FLEXCO_CHECK(nq > 0 && nkv > 0 && nq % nkv == 0, FLEXCO_ESHAPE,
               "n_kv_heads (%d) must divide n_q_heads (%d)", nkv, nq);
  return FLEXCO_OK;
}

// Fills `b`.  With count_only the page checks are skipped (sizes only).
int32_t build(const flexco_batch_desc* d, int32_t page_size, int32_t num_pages, int32_t nq, int32_t nkv,
              int32_t kv_split_pages, Built& b, bool count_only) {
  const int group = nq / nkv;
  b.tile_tokens = std::max(1, 16 / group);
  const int n_req = d->n_req;
  b.split_pages = kv_split_pages;
  if (kv_split_pages <= 0) {
    // Default: 128 pages per split (measured against 64 on the benchmark batch: the attention kernel 3 % and the
    // merge kernel a third faster) - or 256, the most the attention kernel's page-id table holds, when no request
    // sees more pages than that (then no tile is split and the merge launch falls away: 1.2 % of the benchmark
    // step) or when the one-token requests' pages outweigh the other requests' pages x column tiles, i.e. the
    // decode stream carries the attention (measured on such batches with contexts of up to 8192 keys: 1.6 - 4.7 %
    // of the attention against 128; where the chunks carry it 128 stays ahead by 2 - 7 %).  A batch of few
    // requests would leave most of the chip without an attention work item (one wavefront per item and kv
    // head): take the largest of these, 64, 32, 16, 8 pages that gives at least 1024 wavefronts, else 8.
    int64_t max_vis = 0, stream = 0, chunks = 0;
    for (int r = 0; r < n_req; ++r) {
      if (d->n_new[r] <= 0 || d->start_pos[r] < 0 || page_size <= 0) continue;   // rejected below
      max_vis = std::max<int64_t>(max_vis, ((int64_t)d->start_pos[r] + d->n_new[r] - 1) / page_size + 1);
      if (d->n_new[r] == 1) {
        stream += d->start_pos[r] / page_size + 1;
        continue;
      }
      const int tiles = (d->n_new[r] + b.tile_tokens - 1) / b.tile_tokens;
      for (int tl0 = 0; tl0 < tiles; tl0 += FLEXCO_ATTN_ITEM_TILES) {
        const int last_tile = std::min(tl0 + FLEXCO_ATTN_ITEM_TILES, tiles) - 1;
        const int last_tok = std::min((last_tile + 1) * b.tile_tokens, d->n_new[r]) - 1;
        chunks += (int64_t)((d->start_pos[r] + last_tok) / page_size + 1) * (last_tile - tl0 + 1);
      }
    }
    b.split_pages = 8;
    for (int cand = (max_vis <= 256 || stream > chunks) ? 256 : 128; cand >= 16; cand /= 2) {
      int64_t items = 0;
      for (int r = 0; r < n_req; ++r) {
        if (d->n_new[r] <= 0 || d->start_pos[r] < 0 || page_size <= 0) continue;   // rejected below
        const int tiles = (d->n_new[r] + b.tile_tokens - 1) / b.tile_tokens;
        for (int tl0 = 0; tl0 < tiles; tl0 += FLEXCO_ATTN_ITEM_TILES) {
          const int last_tile = std::min(tl0 + FLEXCO_ATTN_ITEM_TILES, tiles) - 1;
          const int last_tok = std::min((last_tile + 1) * b.tile_tokens, d->n_new[r]) - 1;
          const int vis_pages = (d->start_pos[r] + last_tok) / page_size + 1;
          items += (vis_pages + cand - 1) / cand;
        }
      }
      if (items * nkv >= 1024) { b.split_pages = cand; break; }
    }
  }
  FLEXCO_CHECK(b.split_pages % 2 == 0, FLEXCO_EINVAL, "kv_split_pages must be even (got %d)", b.split_pages);
  std::vector<int32_t> need(n_req);
  int64_t T64 = 0;
  for (int r = 0; r < n_req; ++r) {
    FLEXCO_CHECK(d->kind[r] >= 0 && d->kind[r] <= 2, FLEXCO_EINVAL, "request %d: unknown kind %d", r, d->kind[r]);
    FLEXCO_CHECK(d->n_new[r] > 0, FLEXCO_EINVAL, "request %d: n_new must be positive (got %d)", r, d->n_new[r]);
    FLEXCO_CHECK(d->start_pos[r] >= 0, FLEXCO_EINVAL, "request %d: negative start_pos", r);
    FLEXCO_CHECK(d->adapter[r] >= -1 && d->adapter[r] < FLEXCO_MAX_ADAPTERS, FLEXCO_EINVAL,
                 "request %d: adapter id %d outside [-1, %d)", r, d->adapter[r], FLEXCO_MAX_ADAPTERS);
    const int64_t kv_len = (int64_t)d->start_pos[r] + d->n_new[r];
    FLEXCO_CHECK(kv_len < (1ll << 30), FLEXCO_EINVAL, "request %d: kv_len too large", r);
    const int32_t n_have = d->req_page_off[r + 1] - d->req_page_off[r];
    FLEXCO_CHECK(n_have >= 0, FLEXCO_EINVAL, "request %d: req_page_off not ascending", r);
    need[r] = (int32_t)((kv_len + page_size - 1) / page_size);
    FLEXCO_CHECK(need[r] <= n_have, FLEXCO_EPAGE, "request %d: kv_len %lld exceeds its %d pages of %d", r,
                 (long long)kv_len, n_have, page_size);
    if (d->kind[r] == FLEXCO_FINETUNE) {
      FLEXCO_CHECK(b.ft_req < 0, FLEXCO_EUNSUPPORTED,
                   "more than one finetune request in a batch (requests %d and %d)", b.ft_req, r);
      b.ft_req = r;
      b.ft_pos0 = d->start_pos[r];
    }
    b.max_pages = std::max(b.max_pages, need[r]);
    b.max_kv_len = std::max<int32_t>(b.max_kv_len, (int32_t)kv_len);
    T64 += d->n_new[r];
  }
  FLEXCO_CHECK(T64 < (1ll << 24), FLEXCO_EINVAL, "batch of %lld tokens is too large", (long long)T64);
  b.T = (int32_t)T64;
  b.req_tok_off.assign(1, 0);
  b.block_table.assign((size_t)n_req * b.max_pages, -1);
  std::unordered_set<int64_t> seen;
  if (!count_only) seen.reserve((size_t)b.T * 2);
  int32_t prev_adapter = 0;
  for (int r = 0; r < n_req; ++r) {
    const int32_t* pages = d->req_pages + d->req_page_off[r];
    for (int p = 0; p < need[r]; ++p) {
      if (!count_only)
        FLEXCO_CHECK(pages[p] >= 0 && pages[p] < num_pages, FLEXCO_EPAGE,
                     "request %d: page id %d outside [0, %d)", r, pages[p], num_pages);
      b.block_table[(size_t)r * b.max_pages + p] = pages[p];
    }
    const int t_first = (int)b.tok_req.size();
    for (int i = 0; i < d->n_new[r]; ++i) {
      const int32_t pos = d->start_pos[r] + i;
      const int64_t slot = (int64_t)pages[pos / page_size] * page_size + pos % page_size;
      if (!count_only) {
        FLEXCO_CHECK(slot < (1ll << 31), FLEXCO_EPAGE, "request %d: slot index overflows int32", r);
        FLEXCO_CHECK(seen.insert(slot).second, FLEXCO_EPAGE,
                     "request %d position %d: cache slot %lld is written twice in this batch", r, pos,
                     (long long)slot);
      }
      const int t = (int)b.tok_req.size();
      if (t == 0 || d->adapter[r] != prev_adapter) {
        b.seg_off.push_back(t);
        b.seg_adapter.push_back(d->adapter[r]);
        prev_adapter = d->adapter[r];
      }
      b.tok_req.push_back(r);
      b.tok_pos.push_back(pos);
      b.slot.push_back((int32_t)slot);
      b.tok_adapter.push_back(d->adapter[r]);
      if (d->kind[r] == FLEXCO_FINETUNE) b.ft_tok.push_back(t);
    }
    b.req_tok_off.push_back((int32_t)b.tok_req.size());
    b.req_kv_len.push_back(d->start_pos[r] + d->n_new[r]);
    b.req_kind.push_back(d->kind[r]);
    // attention work list: column tiles of this request, each cut into key splits
    const int tile_first = (int)b.tile_req.size();
    for (int t0 = t_first; t0 < (int)b.tok_req.size(); t0 += b.tile_tokens) {
      const int ntok = std::min<int>(b.tile_tokens, (int)b.tok_req.size() - t0);
      const int last_pos = b.tok_pos[t0 + ntok - 1];
      const int vis_pages = last_pos / page_size + 1;
      const int nsplit = (vis_pages + b.split_pages - 1) / b.split_pages;
      const int tile = (int)b.tile_req.size();
      b.tile_req.push_back(r);
      b.tile_tok0.push_back(t0);
      b.tile_ntok.push_back(ntok);
      b.tile_nsplit.push_back(nsplit);
      b.tile_part0.push_back(b.n_parts);
      b.n_parts += nsplit;
      for (int i = 0; i < ntok; ++i) b.tok_tile.push_back(tile);
    }
    // work items: runs of up to FLEXCO_ATTN_ITEM_TILES tiles of this request x the splits of the run's
    // last tile (the one that sees the most keys)
    for (int tl0 = tile_first; tl0 < (int)b.tile_req.size(); tl0 += FLEXCO_ATTN_ITEM_TILES) {
      const int ntl = std::min<int>(FLEXCO_ATTN_ITEM_TILES, (int)b.tile_req.size() - tl0);
      for (int s = 0; s < b.tile_nsplit[tl0 + ntl - 1]; ++s) {
        b.item_tile.push_back(tl0);
        b.item_split.push_back(s);
        b.item_ntiles.push_back(ntl);
      }
    }
  }
  // Order of the work items = order in which the attention grid is dispatched.  Two classes, each
  // longest first (ties keep batch order; the grid ends with its last wavefront): items of a single
  // one-token tile (decode) stream their keys from HBM once; chunk items (prefill, finetune windows)
  // multiply every page against up to four tiles, run several times longer per page and mostly hit the
  // caches.  The chunk items, in runs of four, are dealt evenly into the first quarter of the streaming
  // items: early enough that none of them outlasts the stream, spread enough that the resident
  // wavefronts never are mostly chunk ones (the stream needs enough loads in flight to keep HBM busy).
  // Measured at the 8B shape: 462 us against 468-474 us for the first 1 % / 10 % / 75 %.
  {
    const size_t n = b.item_tile.size();
    std::vector<int32_t> len(n), order(n);
    for (size_t i = 0; i < n; ++i) {
      const int tile = b.item_tile[i] + b.item_ntiles[i] - 1;   // the item's last tile sees its whole key range
      const int vis_pages = b.tok_pos[b.tile_tok0[tile] + b.tile_ntok[tile] - 1] / page_size + 1;
      const int pb = b.item_split[i] * b.split_pages;
      len[i] = std::min(pb + b.split_pages, vis_pages) - pb;
      order[i] = (int32_t)i;
    }
    std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) { return len[x] > len[y]; });
    std::vector<int32_t> stream, chunk;
    for (size_t i = 0; i < n; ++i) {
      const int o = order[i];
      const bool one_token = b.item_ntiles[o] == 1 && b.tile_ntok[b.item_tile[o]] == 1;
      (one_token ? stream : chunk).push_back(o);
    }
    const size_t ns4 = (stream.size() + 3) / 4, nc4 = (chunk.size() + 3) / 4;
    const size_t span = std::max<size_t>(1, ns4 / 4);              // streaming fours the chunk fours are dealt into
    std::vector<int32_t> it, is, in;
    it.reserve(n); is.reserve(n); in.reserve(n);
    auto put4 = [&](const std::vector<int32_t>& src, size_t g) {
      for (size_t i = 4 * g; i < std::min(src.size(), 4 * g + 4); ++i) {
        it.push_back(b.item_tile[src[i]]);
        is.push_back(b.item_split[src[i]]);
        in.push_back(b.item_ntiles[src[i]]);
      }
    };
    size_t ic = 0;
    for (size_t k = 0; k < ns4; ++k) {
      // chunk fours due before streaming four k: ceil(nc4 * k / span), all of them from k = span on
      const size_t due = k >= span ? nc4 : (nc4 * k + span - 1) / span;
      while (ic < due) put4(chunk, ic++);
      put4(stream, k);
    }
    while (ic < nc4) put4(chunk, ic++);
    b.item_tile.swap(it);
    b.item_split.swap(is);
    b.item_ntiles.swap(in);
  }
  // tokens with an adapter, grouped by adapter id: the rows each adapter's bypass network works on
  b.tok_lora.assign(b.tok_adapter.size(), -1);
  for (int a = 0; a < FLEXCO_MAX_ADAPTERS; ++a) {
    b.adapter_tok_off[a] = (int32_t)b.lora_tok.size();
    for (size_t t = 0; t < b.tok_adapter.size(); ++t)
      if (b.tok_adapter[t] == a) {
        b.tok_lora[t] = (int32_t)b.lora_tok.size();
        b.lora_tok.push_back((int32_t)t);
        b.n_adapters = a + 1;
      }
  }
  b.adapter_tok_off[FLEXCO_MAX_ADAPTERS] = (int32_t)b.lora_tok.size();
  b.seg_off.push_back(b.T);
  b.n_seg = (int32_t)b.seg_adapter.size();
  b.n_ft = (int32_t)b.ft_tok.size();
  return FLEXCO_OK;
}

struct BlobWriter {
  int32_t* blob;
  size_t cap, used = 0;
  bool ok = true;
  const int32_t* put(const std::vector<int32_t>& v) {
    const size_t n = (v.size() + 3) / 4 * 4;   // keep every array 16-byte aligned
    if (used + n > cap) { ok = false; return nullptr; }
    int32_t* p = blob + used;
    if (!v.empty()) memcpy(p, v.data(), v.size() * sizeof(int32_t));
    for (size_t i = v.size(); i < n; ++i) p[i] = 0;
    used += n;
    return p;
  }
};

size_t blob_need(const Built& b) {
  size_t n = 0;
  auto add = [&](const std::vector<int32_t>& v) { n += (v.size() + 3) / 4 * 4; };
  add(b.tok_req); add(b.tok_pos); add(b.slot); add(b.req_tok_off); add(b.req_kv_len); add(b.req_kind);
  add(b.block_table); add(b.ft_tok); add(b.seg_off); add(b.seg_adapter); add(b.lora_tok); add(b.tile_req);
  add(b.tile_tok0); add(b.tile_ntok); add(b.tile_nsplit); add(b.tile_part0); add(b.item_tile);
  add(b.item_split); add(b.tok_tile); add(b.tok_lora); add(b.tok_adapter); add(b.item_ntiles);
  return n;
}

}  // namespace
}  // namespace flexco

using namespace flexco;

extern "C" const char* flexco_last_error(void) { return g_err; }

extern "C" int32_t flexco_abi_version(void) { return 8; }

extern "C" int32_t flexco_maps_blob_ints(const flexco_batch_desc* desc, int32_t page_size, int32_t n_q_heads,
                                         int32_t n_kv_heads, int32_t kv_split_pages, size_t* out_ints) {
  clear_error();
  FLEXCO_CHECK(out_ints != nullptr, FLEXCO_EINVAL, "out_ints is NULL");
  int32_t rc = validate_desc(desc, page_size, n_q_heads, n_kv_heads);
  if (rc) return rc;
  Built b;
  rc = build(desc, page_size, 0, n_q_heads, n_kv_heads, kv_split_pages, b, true);
  if (rc) return rc;
  *out_ints = blob_need(b);
  return FLEXCO_OK;
}

extern "C" int32_t flexco_build_maps(const flexco_batch_desc* desc, int32_t page_size, int32_t num_pages,
                                     int32_t n_q_heads, int32_t n_kv_heads, int32_t kv_split_pages,
                                     int32_t* blob, size_t blob_ints, flexco_maps* out) {
  clear_error();
  FLEXCO_CHECK(blob != nullptr && out != nullptr, FLEXCO_EINVAL, "blob or out is NULL");
  FLEXCO_CHECK(num_pages > 0, FLEXCO_EINVAL, "num_pages must be positive (got %d)", num_pages);
  int32_t rc = validate_desc(desc, page_size, n_q_heads, n_kv_heads);
  if (rc) return rc;
  Built b;
  rc = build(desc, page_size, num_pages, n_q_heads, n_kv_heads, kv_split_pages, b, false);
  if (rc) return rc;
  const size_t need = blob_need(b);
  FLEXCO_CHECK(need <= blob_ints, FLEXCO_EWORKSPACE, "maps need %zu int32 words, blob has %zu", need, blob_ints);
  BlobWriter w{blob, blob_ints};
  flexco_maps m;
  memset(&m, 0, sizeof(m));
  m.T = b.T; m.n_req = desc->n_req; m.n_ft = b.n_ft; m.n_seg = b.n_seg; m.max_pages = b.max_pages;
  m.page_size = page_size; m.n_tiles = (int32_t)b.tile_req.size(); m.n_items = (int32_t)b.item_tile.size();
  m.n_parts = b.n_parts; m.tile_tokens = b.tile_tokens; m.kv_split_pages = b.split_pages;
  m.ft_req = b.ft_req; m.max_kv_len = b.max_kv_len;
  m.ft_tok0 = b.ft_req >= 0 ? b.req_tok_off[b.ft_req] : 0; m.ft_pos0 = b.ft_pos0;
  m.n_lora = (int32_t)b.lora_tok.size();
  m.n_adapters = b.n_adapters;
  m.ft_adapter = b.ft_req >= 0 ? desc->adapter[b.ft_req] : -1;
  m.num_pages = num_pages;
  m.n_single = 0;
  int64_t stream_pages = 0, chunk_tile_pages = 0;
  for (size_t i = 0; i < b.item_tile.size(); ++i) {
    const int last = b.item_tile[i] + b.item_ntiles[i] - 1;       // the item's last tile sees its whole key range
    const int vis_pages = b.tok_pos[b.tile_tok0[last] + b.tile_ntok[last] - 1] / page_size + 1;
    const int pb = b.item_split[i] * b.split_pages;
    const int pages = std::min(pb + b.split_pages, vis_pages) - pb;
    if (b.item_ntiles[i] == 1 && b.tile_ntok[b.item_tile[i]] == 1) {
      ++m.n_single;
      stream_pages += pages;
    } else {
      chunk_tile_pages += (int64_t)pages * b.item_ntiles[i];
    }
  }
  m.stream_pages = (int32_t)std::min<int64_t>(stream_pages, INT32_MAX);
  m.chunk_tile_pages = (int32_t)std::min<int64_t>(chunk_tile_pages, INT32_MAX);
  memcpy(m.adapter_tok_off, b.adapter_tok_off, sizeof(m.adapter_tok_off));
  m.tok_req = w.put(b.tok_req); m.tok_pos = w.put(b.tok_pos); m.slot = w.put(b.slot);
  m.req_tok_off = w.put(b.req_tok_off); m.req_kv_len = w.put(b.req_kv_len); m.req_kind = w.put(b.req_kind);
  m.block_table = w.put(b.block_table); m.ft_tok = w.put(b.ft_tok); m.seg_off = w.put(b.seg_off);
  m.seg_adapter = w.put(b.seg_adapter); m.lora_tok = w.put(b.lora_tok); m.tile_req = w.put(b.tile_req);
  m.tile_tok0 = w.put(b.tile_tok0); m.tile_ntok = w.put(b.tile_ntok); m.tile_nsplit = w.put(b.tile_nsplit);
  m.tile_part0 = w.put(b.tile_part0); m.item_tile = w.put(b.item_tile); m.item_split = w.put(b.item_split);
  m.tok_tile = w.put(b.tok_tile); m.tok_lora = w.put(b.tok_lora); m.tok_adapter = w.put(b.tok_adapter);
  m.item_ntiles = w.put(b.item_ntiles);
  FLEXCO_CHECK(w.ok, FLEXCO_EWORKSPACE, "blob too small");
  m.blob_ints = (int32_t)w.used;
  *out = m;
  return FLEXCO_OK;
}

extern "C" int32_t flexco_maps_rebase(const flexco_maps* host_maps, const int32_t* host_blob,
                                      const int32_t* other_blob, flexco_maps* out) {
  clear_error();
  FLEXCO_CHECK(host_maps && host_blob && other_blob && out, FLEXCO_EINVAL, "NULL argument");
  flexco_maps m = *host_maps;
  const int32_t** fields[] = {&m.tok_req, &m.tok_pos, &m.slot, &m.req_tok_off, &m.req_kv_len, &m.req_kind,
                              &m.block_table, &m.ft_tok, &m.seg_off, &m.seg_adapter, &m.lora_tok, &m.tile_req,
                              &m.tile_tok0, &m.tile_ntok, &m.tile_nsplit, &m.tile_part0, &m.item_tile,
                              &m.item_split, &m.tok_tile, &m.tok_lora, &m.tok_adapter,
                              &m.item_ntiles};
  for (auto f : fields) {
    FLEXCO_CHECK(*f >= host_blob && *f <= host_blob + m.blob_ints, FLEXCO_EINVAL,
                 "maps do not point into host_blob");
    *f = other_blob + (*f - host_blob);
  }
  *out = m;
  return FLEXCO_OK;
}

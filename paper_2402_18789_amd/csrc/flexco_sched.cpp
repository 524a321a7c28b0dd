// Hybrid token scheduler (Sec. 6.2), host side.
//
// Stage 1 picks the inference work of an iteration by iteration-level scheduling with chunked
// prefill; stage 2 appends the largest finetuning window whose estimated iteration latency still
// meets the SLO, s = argmax f(c, s) <= SLO, with f interpolated from a profiled table.  The output of
// stage 1 plus the window is what flexco_build_maps takes.
//
// Floating point decides an integer here (the window size), so the arithmetic is spelled out one
// operation at a time in double, with contraction off: another implementation that follows the
// same order gets the same window.
#include <cstring>

#include "flexco_host.h"

#pragma STDC FP_CONTRACT OFF

namespace flexco {

namespace {

// index of the grid segment used for x: the one that contains it, the first below the grid,
// the last above it
int segment(const int32_t* grid, int n, double x) {
  int i = 0;
  while (i + 2 < n && x >= (double)grid[i + 1]) ++i;
  return i;
}

int32_t check_model(const flexco_latency_model* m) {
  FLEXCO_CHECK(m && m->c_grid && m->s_grid && m->ms, FLEXCO_EINVAL, "latency model: NULL pointer");
  FLEXCO_CHECK(m->n_c >= 2 && m->n_s >= 2, FLEXCO_EINVAL, "latency model: a grid needs at least two points");
  for (int i = 0; i + 1 < m->n_c; ++i)
    FLEXCO_CHECK(m->c_grid[i] < m->c_grid[i + 1], FLEXCO_EINVAL, "latency model: c_grid must ascend strictly");
  for (int j = 0; j + 1 < m->n_s; ++j)
    FLEXCO_CHECK(m->s_grid[j] < m->s_grid[j + 1], FLEXCO_EINVAL, "latency model: s_grid must ascend strictly");
  return FLEXCO_OK;
}

double estimate(const flexco_latency_model* m, int32_t c, int32_t s) {
  const int i = segment(m->c_grid, m->n_c, (double)c);
  const int j = segment(m->s_grid, m->n_s, (double)s);
  const double t = ((double)c - (double)m->c_grid[i]) / ((double)m->c_grid[i + 1] - (double)m->c_grid[i]);
  const double u = ((double)s - (double)m->s_grid[j]) / ((double)m->s_grid[j + 1] - (double)m->s_grid[j]);
  const double f00 = m->ms[(size_t)i * m->n_s + j], f10 = m->ms[(size_t)(i + 1) * m->n_s + j];
  const double f01 = m->ms[(size_t)i * m->n_s + j + 1], f11 = m->ms[(size_t)(i + 1) * m->n_s + j + 1];
  const double d0 = f10 - f00;
  const double p0 = t * d0;
  const double f0 = f00 + p0;          // along c at s_grid[j]
  const double d1 = f11 - f01;
  const double p1 = t * d1;
  const double f1 = f01 + p1;          // along c at s_grid[j + 1]
  const double dd = f1 - f0;
  const double pp = u * dd;
  return f0 + pp;
}

}  // namespace

}  // namespace flexco

using namespace flexco;

extern "C" int32_t flexco_latency_estimate(const flexco_latency_model* model, int32_t c, int32_t s, double* out_ms) {
  clear_error();
  FLEXCO_TRY(check_model(model));
  FLEXCO_CHECK(out_ms, FLEXCO_EINVAL, "NULL argument");
  *out_ms = estimate(model, c, s);
  return FLEXCO_OK;
}

extern "C" int32_t flexco_sched_window(const flexco_latency_model* model, int32_t c, double slo_ms, int32_t s_avail,
                                       int32_t quantum, int32_t* out_s) {
  clear_error();
  FLEXCO_TRY(check_model(model));
  FLEXCO_CHECK(out_s, FLEXCO_EINVAL, "NULL argument");
  FLEXCO_CHECK(quantum > 0 && s_avail >= 0, FLEXCO_EINVAL, "quantum must be positive and s_avail non-negative");
  // every candidate is evaluated: a profiled table need not be monotone in s
  int32_t best = 0;
  for (int64_t s = 0; s <= s_avail; s += quantum)
    if (estimate(model, c, (int32_t)s) <= slo_ms && s > best) best = (int32_t)s;
  if (s_avail % quantum != 0 && estimate(model, c, s_avail) <= slo_ms) best = s_avail;
  *out_s = best;
  return FLEXCO_OK;
}

extern "C" int32_t flexco_sched_inference(int32_t n_req, const int32_t* prompt_len, const int32_t* prefilled,
                                          const int32_t* gen_len, const int32_t* generated, int32_t* state,
                                          int32_t max_batch, int32_t token_budget, int32_t chunk, int32_t* out_req,
                                          int32_t* out_kind, int32_t* out_start_pos, int32_t* out_n_new,
                                          int32_t out_capacity, int32_t* out_n, int32_t* out_tokens) {
  clear_error();
  FLEXCO_CHECK(n_req >= 0 && out_n && out_tokens, FLEXCO_EINVAL, "bad argument");
  FLEXCO_CHECK(n_req == 0 || (prompt_len && prefilled && gen_len && generated && state), FLEXCO_EINVAL, "NULL request array");
  FLEXCO_CHECK(max_batch > 0 && token_budget > 0 && chunk > 0, FLEXCO_EINVAL,
               "max_batch, token_budget and chunk must be positive");
  FLEXCO_CHECK(out_capacity == 0 || (out_req && out_kind && out_start_pos && out_n_new), FLEXCO_EINVAL, "NULL output array");
  for (int r = 0; r < n_req; ++r) {
    FLEXCO_CHECK(state[r] >= FLEXCO_REQ_WAITING && state[r] <= FLEXCO_REQ_FINISHED, FLEXCO_EINVAL,
                 "request %d: unknown state %d", r, state[r]);
    FLEXCO_CHECK(prompt_len[r] > 0 && prefilled[r] >= 0 && prefilled[r] <= prompt_len[r] && gen_len[r] >= 0 &&
                     generated[r] >= 0 && generated[r] <= gen_len[r],
                 FLEXCO_EINVAL, "request %d: inconsistent progress", r);
  }
  int running = 0;
  for (int r = 0; r < n_req; ++r) running += state[r] == FLEXCO_REQ_RUNNING;
  for (int r = 0; r < n_req && running < max_batch; ++r)     // admission in arrival order
    if (state[r] == FLEXCO_REQ_WAITING) { state[r] = FLEXCO_REQ_RUNNING; ++running; }
  int n = 0, budget = token_budget;
  auto emit = [&](int r, int kind, int start, int n_new) -> bool {
    if (n >= out_capacity) return false;
    out_req[n] = r; out_kind[n] = kind; out_start_pos[n] = start; out_n_new[n] = n_new;
    ++n;
    return true;
  };
  for (int r = 0; r < n_req; ++r)                             // one token for every request that is generating
    if (state[r] == FLEXCO_REQ_RUNNING && prefilled[r] == prompt_len[r] && generated[r] < gen_len[r] && budget > 0) {
      FLEXCO_CHECK(emit(r, FLEXCO_DECODE, prompt_len[r] + generated[r], 1), FLEXCO_EWORKSPACE,
                   "more than %d entries in the iteration", out_capacity);
      budget -= 1;
    }
  for (int r = 0; r < n_req; ++r)                             // prompt chunks while the budget lasts
    if (state[r] == FLEXCO_REQ_RUNNING && prefilled[r] < prompt_len[r] && budget > 0) {
      int take = prompt_len[r] - prefilled[r];
      if (take > chunk) take = chunk;
      if (take > budget) take = budget;
      FLEXCO_CHECK(emit(r, FLEXCO_PREFILL, prefilled[r], take), FLEXCO_EWORKSPACE,
                   "more than %d entries in the iteration", out_capacity);
      budget -= take;
    }
  *out_n = n;
  *out_tokens = token_budget - budget;
  return FLEXCO_OK;
}

extern "C" int32_t flexco_sched_advance(int32_t n_entries, const int32_t* req, const int32_t* kind, const int32_t* n_new,
                                        int32_t n_req, const int32_t* prompt_len, int32_t* prefilled,
                                        const int32_t* gen_len, int32_t* generated, int32_t* state) {
  clear_error();
  FLEXCO_CHECK(n_entries >= 0 && n_req >= 0, FLEXCO_EINVAL, "bad argument");
  FLEXCO_CHECK(n_entries == 0 || (req && kind && n_new && prompt_len && prefilled && gen_len && generated && state),
               FLEXCO_EINVAL, "NULL argument");
  for (int e = 0; e < n_entries; ++e) {
    const int r = req[e];
    FLEXCO_CHECK(r >= 0 && r < n_req, FLEXCO_EINVAL, "entry %d: request %d out of range", e, r);
    if (kind[e] == FLEXCO_DECODE) generated[r] += 1; else prefilled[r] += n_new[e];
    if (prefilled[r] == prompt_len[r] && generated[r] >= gen_len[r]) state[r] = FLEXCO_REQ_FINISHED;
  }
  return FLEXCO_OK;
}

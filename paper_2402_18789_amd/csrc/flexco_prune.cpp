// Static graph pruning (Alg. 1, Sec. 5.2) on an operator graph handed over as integer arrays; host only.
//
// Step 1: one backward operator per forward operator (reverse-mode rules below); the gradients of
// frozen base weights are deleted, every backward operator's inputs shrink to what its remaining
// outputs need, outputs nobody consumes are deleted in turn (work queue), and what the surviving
// backward operators still read of the forward pass is the activation set.  Step 2: an activation
// whose producer is cheap and whose producer's inputs are all kept (or weights) is rematerialised
// instead of stored.  Readings of the listing: gradients of trainable weights and of tensors marked
// need_grad leave the graph and count as consumed; when an operator's inputs shrink, the producers of
// the dropped gradients are re-examined too; "inputs kept" in step 2 refers to the set step 1 left;
// a ReLU's backward reads only the sign of its output, and a tensor read in that form only is kept as
// a bitmask.
#include <cstdint>
#include <deque>
#include <vector>

#include "flexco_host.h"

namespace flexco {
namespace {

// What the gradient of input `slot` of an operator is computed from, besides the gradient of the
// operator's output: a list of (tensor, as_mask) reads of forward tensors or weights.
struct Read { int32_t tensor; bool mask; };

int32_t rule(int kind, const int32_t* in, int n_in, int32_t out, int slot, std::vector<Read>& reads) {
  reads.clear();
  switch (kind) {
    case FLEXCO_OP_SOURCE: return FLEXCO_OK;
    case FLEXCO_OP_MATMUL:                                  // y = x w: dx reads w, dw reads x
      FLEXCO_CHECK(n_in == 2, FLEXCO_ESHAPE, "matmul takes 2 inputs, got %d", n_in);
      reads.push_back({in[1 - slot], false});
      return FLEXCO_OK;
    case FLEXCO_OP_ADD: return FLEXCO_OK;                   // passes the gradient on
    case FLEXCO_OP_RMSNORM:                                 // h = rmsnorm(x; g): dx reads x and g, dg reads x
      FLEXCO_CHECK(n_in == 2, FLEXCO_ESHAPE, "rmsnorm takes 2 inputs, got %d", n_in);
      reads.push_back({in[0], false});
      if (slot == 0) reads.push_back({in[1], false});
      return FLEXCO_OK;
    case FLEXCO_OP_ROPE: return FLEXCO_OK;                  // a fixed rotation
    case FLEXCO_OP_ATTENTION:                               // reads q, k, v (probabilities are recomputed inside)
      for (int i = 0; i < n_in; ++i) reads.push_back({in[i], false});
      return FLEXCO_OK;
    case FLEXCO_OP_SWIGLU:                                  // act = silu(gate) up: dgate reads both, dup reads gate
      FLEXCO_CHECK(n_in == 2, FLEXCO_ESHAPE, "swiglu takes 2 inputs, got %d", n_in);
      reads.push_back({in[0], false});
      if (slot == 0) reads.push_back({in[1], false});
      return FLEXCO_OK;
    case FLEXCO_OP_MUL:                                     // y = a b elementwise: each gradient reads the other
      FLEXCO_CHECK(n_in == 2, FLEXCO_ESHAPE, "mul takes 2 inputs, got %d", n_in);
      reads.push_back({in[1 - slot], false});
      return FLEXCO_OK;
    case FLEXCO_OP_RELU:                                    // the gradient passes where the output is positive
      reads.push_back({out, true});
      return FLEXCO_OK;
    default: return fail(FLEXCO_EINVAL, "unknown operator kind %d", kind);
  }
}

}  // namespace
}  // namespace flexco

using namespace flexco;

extern "C" int32_t flexco_prune_graph(const flexco_graph* g, int32_t* keep) {
  clear_error();
  FLEXCO_CHECK(g && keep, FLEXCO_EINVAL, "NULL argument");
  FLEXCO_CHECK(g->n_ops > 0 && g->n_tensors > 0, FLEXCO_EINVAL, "empty graph");
  FLEXCO_CHECK(g->op_kind && g->op_cheap && g->op_in_off && g->op_in && g->op_out && g->tensor_class && g->need_grad,
               FLEXCO_EINVAL, "graph has a NULL array");
  const int n_ops = g->n_ops, nt = g->n_tensors;
  // every operator has one output here (op_out[op]); inputs op_in[op_in_off[op] .. op_in_off[op + 1])
  std::vector<int32_t> producer(nt, -1);
  for (int o = 0; o < n_ops; ++o) {
    FLEXCO_CHECK(g->op_in_off[o] <= g->op_in_off[o + 1], FLEXCO_ESHAPE, "operator %d: input offsets descend", o);
    FLEXCO_CHECK(g->op_out[o] >= 0 && g->op_out[o] < nt, FLEXCO_EINVAL, "operator %d: output tensor %d out of range", o,
                 g->op_out[o]);
    FLEXCO_CHECK(producer[g->op_out[o]] < 0, FLEXCO_ESHAPE, "tensor %d has two producers", g->op_out[o]);
    FLEXCO_CHECK(g->tensor_class[g->op_out[o]] == FLEXCO_TENSOR_ACTIVATION, FLEXCO_ESHAPE,
                 "operator %d writes a weight", o);
    producer[g->op_out[o]] = o;
    for (int i = g->op_in_off[o]; i < g->op_in_off[o + 1]; ++i)
      FLEXCO_CHECK(g->op_in[i] >= 0 && g->op_in[i] < nt, FLEXCO_EINVAL, "operator %d: input tensor %d out of range", o,
                   g->op_in[i]);
  }
  // ---- the backward graph: operator o may produce d(in_i) for each of its inputs ---------------------
  // out_alive[slot of op_in]: that gradient output still exists
  const int n_slots = g->op_in_off[n_ops];
  std::vector<char> out_alive(n_slots, 1);
  std::vector<int32_t> slot_op(n_slots);
  for (int o = 0; o < n_ops; ++o)
    for (int i = g->op_in_off[o]; i < g->op_in_off[o + 1]; ++i) slot_op[i] = o;
  // gradient producers of tensor t = the slots whose input is t
  std::vector<std::vector<int32_t>> grad_slots(nt);
  for (int i = 0; i < n_slots; ++i) grad_slots[g->op_in[i]].push_back(i);
  // what a backward operator reads, given its alive outputs: d(out) if any output is alive, plus the
  // forward reads of the alive outputs' rules
  std::vector<char> reads_dout(n_ops, 0);                       // reads the gradient of its own output
  std::vector<std::vector<char>> reads_full(n_ops, std::vector<char>()), reads_mask(n_ops, std::vector<char>());
  std::vector<Read> tmp;
  auto update = [&](int o) -> int32_t {
    reads_dout[o] = 0;
    reads_full[o].assign(nt, 0);
    reads_mask[o].assign(nt, 0);
    const int32_t* in = g->op_in + g->op_in_off[o];
    const int n_in = g->op_in_off[o + 1] - g->op_in_off[o];
    for (int s = 0; s < n_in; ++s) {
      if (!out_alive[g->op_in_off[o] + s]) continue;
      reads_dout[o] = 1;
      FLEXCO_TRY(rule(g->op_kind[o], in, n_in, g->op_out[o], s, tmp));
      for (const Read& r : tmp) (r.mask ? reads_mask : reads_full)[o][r.tensor] = 1;
    }
    return FLEXCO_OK;
  };
  for (int o = 0; o < n_ops; ++o) FLEXCO_TRY(update(o));
  std::deque<int32_t> queue;
  // shrinking an operator re-queues it and the producers of the gradient it no longer reads (its own d(out))
  auto shrink = [&](int o) -> int32_t {
    const char had = reads_dout[o];
    FLEXCO_TRY(update(o));
    queue.push_back(o);
    if (had && !reads_dout[o])
      for (int32_t s : grad_slots[g->op_out[o]]) queue.push_back(slot_op[s]);
    return FLEXCO_OK;
  };
  for (int i = 0; i < n_slots; ++i)
    if (g->tensor_class[g->op_in[i]] == FLEXCO_TENSOR_FROZEN) {   // gradients of frozen base weights
      out_alive[i] = 0;
      FLEXCO_TRY(shrink(slot_op[i]));
    }
  while (!queue.empty()) {
    const int o = queue.front();
    queue.pop_front();
    for (int i = g->op_in_off[o]; i < g->op_in_off[o + 1]; ++i) {
      if (!out_alive[i]) continue;
      const int32_t t = g->op_in[i];                             // this output is d(t)
      bool consumed = g->tensor_class[t] == FLEXCO_TENSOR_TRAINABLE || g->need_grad[t] != 0;
      if (!consumed && producer[t] >= 0) consumed = reads_dout[producer[t]] != 0;   // the only reader of d(t)
      if (!consumed) {
        out_alive[i] = 0;
        FLEXCO_TRY(shrink(o));
      }
    }
  }
  // ---- step 1 result: forward tensors (activations) the backward pass reads ---------------------------
  std::vector<char> full(nt, 0), mask(nt, 0);
  for (int o = 0; o < n_ops; ++o)
    for (int t = 0; t < nt; ++t) {
      if (reads_full[o][t]) full[t] = 1;
      if (reads_mask[o][t]) mask[t] = 1;
    }
  for (int t = 0; t < nt; ++t) {
    const bool act = producer[t] >= 0;                           // weights are not activations
    keep[t] = !act ? FLEXCO_KEEP_NONE : full[t] ? FLEXCO_KEEP_STORE : mask[t] ? FLEXCO_KEEP_BITMASK : FLEXCO_KEEP_NONE;
  }
  // ---- step 2: rematerialise what is cheap to recompute from kept inputs --------------------------------
  std::vector<int32_t> result(keep, keep + nt);
  for (int t = 0; t < nt; ++t) {
    if (keep[t] != FLEXCO_KEEP_STORE) continue;
    const int o = producer[t];
    if (g->op_kind[o] == FLEXCO_OP_SOURCE || !g->op_cheap[o]) continue;
    bool all_kept = true;
    for (int i = g->op_in_off[o]; i < g->op_in_off[o + 1]; ++i) {
      const int32_t x = g->op_in[i];
      const bool weight = g->tensor_class[x] != FLEXCO_TENSOR_ACTIVATION;
      if (!weight && keep[x] != FLEXCO_KEEP_STORE) all_kept = false;
    }
    if (all_kept) result[t] = FLEXCO_KEEP_REMAT;
  }
  for (int t = 0; t < nt; ++t) keep[t] = result[t];
  return FLEXCO_OK;
}
